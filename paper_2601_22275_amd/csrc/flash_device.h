// Device-side pieces shared by the bf16 MFMA blocked-softmax kernels (flash.hip, flash_kv.hip):
// tile constants, the kernel parameter block, LDS read helpers and the per-sub-tile softmax
// arithmetic.  Everything has internal linkage.
#pragma once
#include "../../include/vmonarch.h"
#include "common.h"

namespace vm {

namespace {

constexpr int BK = 64;          // key rows per LDS tile
// 32-query tiles per wave.  The code is written for any QT, but two tiles (half the LDS
// reads per MFMA) need about 300 registers per wave at d = 128 and a wave has 256 with two
// waves per SIMD, so 1 is the only value in use.
constexpr int QT = 1;
constexpr int NW = 8;             // waves per workgroup
constexpr int BQ = 32 * QT * NW;  // query rows per workgroup
constexpr int NSLOT = 4;          // LDS tile slots per tensor
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;
constexpr float RESCALE_TH = 8.0f;  // rescale the accumulators only when a row max grows by 2^8
constexpr float NEG_BIG = -1.0e30f;

struct FlashParams {
  const bf16_t* q;      // query rows
  const float* cR;      // per query row, may be null (= 1)
  const bf16_t* k;
  const bf16_t* v;
  bf16_t* outk;         // softmax(z) K   (alpha_L)
  bf16_t* outv;         // softmax(z) V   (y, or the first-frame output)
  float* cl;            // sum p log p    (c_L)
  float* lse;           // natural-log sum-exp of the row's logits, or null
  float* part_o;        // split mode: [split][problem][nq][D] normalised partial outputs
  float* part_lse;      // split mode: [split][problem][nq] log2-sum-exp of the partial
  long long q_rows_per_problem;  // row distance between problems in q / cR / outputs
  long long k_rows_per_problem;  // row distance between problems in k / v
  int nq;               // query rows per problem
  int nk;               // key rows per problem
  int nqb;              // query blocks per problem
  int nsplit;           // key splits per (problem, query block)
  int keys_per_split;   // multiple of BK
  int total_blocks;     // nproblems * nqb * nsplit
  int blocks_per_xcd;   // ceil(total_blocks / 8)
  float row_scale;
  float cr_min;
  int blend;            // outv <- (outv + result) / 2 instead of outv <- result
  // flash_kernel only.  Rows of a problem need not be adjacent: row r of problem p is row
  //   (p / inner) * rows_per_problem + (p % inner) * inner_rows + r * row_stride     (inner = 0 means 1)
  // of its tensor, the same rule for queries and keys.  The temporal factor walks frame-major tensors this
  // way: problem = (head, position), rows = frames, row_stride = b.  row_stride = 0 means 1.
  int inner;
  long long inner_rows;
  long long row_stride;
  // Biased modes (template parameter BIAS != 0): logit of (query r, key l) = sc (q . k) + kb_scale * kbias[key row l]
  // (kbias indexed like the key rows); BIAS == 2 additionally fixes the reference of query r at
  // qb_scale * qbias[query row r], keeps the sums unnormalised and stores the sum of the weights in `cl`.
  const float* kbias;
  const float* qbias;
  float kb_scale;
  float qb_scale;
  const int* q_index;   // query row r of a problem is row q_index[r] of it (null: row r); entries
                        // outside [0, q_index_limit) are skipped
  int q_index_limit;
  int own_tile_first;   // flash2: queries and keys are the same rows (R-update): start the key loop at the query block's own tile
};

__device__ __forceinline__ bf16x8 lds_read_b128(const char* p) { return *reinterpret_cast<const bf16x8*>(p); }

__device__ __forceinline__ bf16x4 lds_read_tr(const char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
      (bf16x4 __attribute__((address_space(3)))*)(reinterpret_cast<const bf16x4*>(p)));
}

__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  // two round-to-nearest-even conversions; the compiler emits v_cvt_pk_bf16_f32
  typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
  bf16x2 r;
  r[0] = (__bf16)a;
  r[1] = (__bf16)b;
  uint32_t u;
  __builtin_memcpy(&u, &r, 4);
  return u;
}

// acc *= alpha for an MFMA accumulator tile.  This file is compiled with the MFMA results
// in ordinary vector registers (-mllvm -amdgpu-mfma-vgpr-form=1): with two waves per SIMD
// a wave owns 256 registers in total, the accumulators need only 64 of them, and keeping
// everything in one register class lets plain VALU code rescale them and spares the
// accumulation-register round trips.
__device__ __forceinline__ void scale_acc(f32x16& acc, float alpha) {
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] *= alpha;
}

// Row maximum of one 32-key sub-tile for one 32-query tile.  `s` holds the raw logits
// (aR . K) of query `lane & 31` for keys {8c + 4g + r}; the partner lane (lane ^ 32) holds the
// other 16 keys and is reached with v_permlane32_swap (no LDS round trip).  Key rows past
// the end of the range are copies of the last valid row, so they never change a maximum.
__device__ __forceinline__ float subtile_max(const f32x16& s) {
  // v_max3: four independent chains of depth 2, then 2 more ops
  float m0 = fmaxf(fmaxf(s[0], s[1]), s[2]), m1 = fmaxf(fmaxf(s[3], s[4]), s[5]);
  float m2 = fmaxf(fmaxf(s[6], s[7]), s[8]), m3 = fmaxf(fmaxf(s[9], s[10]), s[11]);
  m0 = fmaxf(fmaxf(m0, s[12]), s[13]);
  m1 = fmaxf(fmaxf(m1, s[14]), s[15]);
  float mx = fmaxf(fmaxf(m0, m1), fmaxf(m2, m3));
  const unsigned u = __float_as_uint(mx);
  auto sw = __builtin_amdgcn_permlane32_swap(u, u, false, false);
  return fmaxf(__uint_as_float(sw[0]), __uint_as_float(sw[1]));
}

// Probabilities of the sub-tile relative to the reference max `msc` (log2 units):
// t = s * sc - msc, p = 2^t.  `pb[0..1]` receive the two bf16 B operands (16 keys each) of
// the O^T += X^T P^T products.  Running sums (Alg. 1's l and, when ENT == 1, h):
//   lt = sum of the bf16-ROUNDED p (v_dot2 against ones).  The accumulators are divided by
//        this one, so that the output is an exact convex combination of the rows with
//        slightly perturbed weights; dividing by the unrounded sum instead leaves a 2^-9
//        relative error on rows dominated by one key.  It also serves as l in the
//        log-sum-exp and in H = log l - h / l (error ~1e-3 in c_L, one VALU op per score saved);
//   h  = sum p * t with the unrounded p.
template <int ENT>
__device__ __forceinline__ void subtile_probs(const f32x16& s, float sc, float msc, float& lt, float& h,
                                              bf16x8 pb[2]) {
  typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
  bf16x2 ones2;
  ones2[0] = (__bf16)1.0f;
  ones2[1] = (__bf16)1.0f;
  float p[16];
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    float t = __builtin_fmaf(s[r], sc, -msc);
    p[r] = __builtin_amdgcn_exp2f(t);
    if (ENT == 1) h = __builtin_fmaf(p[r], t, h);
  }
#pragma unroll
  for (int c = 0; c < 2; ++c) {
    uint32_t w[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      w[e] = pack_bf16(p[8 * c + 2 * e], p[8 * c + 2 * e + 1]);
      bf16x2 pr;
      __builtin_memcpy(&pr, &w[e], 4);
      lt = __builtin_amdgcn_fdot2_f32_bf16(pr, ones2, lt, false);
    }
    __builtin_memcpy(&pb[c], w, 16);
  }
}

// One half (8 scores per lane, one B operand of 16 keys) of subtile_probs<1>: registers 8 c .. 8 c + 7 of `s`.
template <int C>
__device__ __forceinline__ bf16x8 halftile_probs(const f32x16& s, float sc, float msc, float& lt, float& h) {
  typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
  bf16x2 ones2;
  ones2[0] = (__bf16)1.0f;
  ones2[1] = (__bf16)1.0f;
  float p[8];
#pragma unroll
  for (int r = 0; r < 8; ++r) {
    float t = __builtin_fmaf(s[8 * C + r], sc, -msc);
    p[r] = __builtin_amdgcn_exp2f(t);
    h = __builtin_fmaf(p[r], t, h);
  }
  uint32_t w[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    w[e] = pack_bf16(p[2 * e], p[2 * e + 1]);
    bf16x2 pr;
    __builtin_memcpy(&pr, &w[e], 4);
    lt = __builtin_amdgcn_fdot2_f32_bf16(pr, ones2, lt, false);
  }
  bf16x8 out;
  __builtin_memcpy(&out, w, 16);
  return out;
}

}  // namespace

}  // namespace vm

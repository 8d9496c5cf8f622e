// Internal declarations shared by the translation units of libvmonarch (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace vm {

typedef uint16_t bf16_t;  // raw bfloat16 bits in memory

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;

__device__ __forceinline__ float bf16_to_f32(bf16_t h) { return __uint_as_float(((uint32_t)h) << 16); }
// round-to-nearest-even; NaN stays NaN
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
template <typename E> __device__ __forceinline__ float load_f(const E* p);
template <> __device__ __forceinline__ float load_f<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float load_f<bf16_t>(const bf16_t* p) { return bf16_to_f32(*p); }
template <typename E> __device__ __forceinline__ void store_f(E* p, float x);
template <> __device__ __forceinline__ void store_f<float>(float* p, float x) { *p = x; }
template <> __device__ __forceinline__ void store_f<bf16_t>(bf16_t* p, float x) { *p = f32_to_bf16(x); }

// Geometry of a bf16 row tile in LDS for head dimension D (64 or 128), shared by the MFMA
// kernels.  A row is D/8 chunks of 16 bytes; chunk c of row r is stored at chunk c ^ swz(r).
// swz depends on r & 15 only, so adding a multiple of 16 rows to an address is plain
// arithmetic.  It is chosen so that the two read patterns of the 32x32x16 MFMA operands
// spread over all 64 banks:
//   row reads (ds_read_b128, 16 consecutive rows, one logical chunk): 16 distinct 16-byte
//     bank groups.  D = 128: a row is the whole 256-byte bank window and swz is a bijection of
//     the 16 rows.  D = 64: two rows share the window and swz is a bijection of the 8 row pairs;
//   transpose reads (ds_read_b64_tr_b16, 8 consecutive rows x 4 consecutive chunks): every
//     bank group twice, the minimum for 512 bytes.
template <int D>
struct RowGeo {
  static_assert(D == 64 || D == 128, "head dimensions with an MFMA path");
  static constexpr int ROW_BYTES = D * 2;
  static constexpr int CH = D / 8;    // 16-byte chunks per row
  static constexpr int KS = D / 16;   // k-steps of a contraction over d
  static constexpr int CT = D / 32;   // 32-channel tiles of an output row
  static constexpr int RPI = 1024 / ROW_BYTES;  // rows covered by one 64-lane x 16-byte access
  __device__ static __forceinline__ int swz(int row) {
    if (D == 128) {
      const int x = row & 15;
      return ((x & 3) << 2) | (x >> 2);
    } else {
      const int p = (row >> 1) & 7;
      return ((p & 1) << 2) | (p >> 1);
    }
  }
};

// Problem description handed to every launcher.
struct Dims {
  int BH;     // B * heads
  int T;      // frames (m)
  int b;      // spatial positions per frame
  int d;      // head dimension
  long long N;  // T * b
};

// ---- launchers (host) -------------------------------------------------------------
// generic.hip : plain-ALU kernels, any T, b, d <= 256, element type float or bf16
template <typename E>
hipError_t launch_r_update_generic(const E* aR, const float* cR, const E* k, const E* v, E* aL, float* cL,
                                   E* y, float* lse, const Dims& dm, float row_scale, float cr_min, hipStream_t st);
// lse_scratch (BH * N floats) is needed for the fitting form when l_update_generic_needs_lse(): more frames than the
// kernel that keeps the T x T block in LDS can hold
bool l_update_generic_needs_lse(const Dims& dm);
template <typename E>
hipError_t launch_l_update_generic(const E* q, const E* aL, const float* cL, const E* y, E* aR, float* cR,
                                   E* out, float* lse_scratch, const Dims& dm, float q_scale, hipStream_t st);
template <typename E>
hipError_t launch_first_frame_generic(const E* q, const E* k, const E* v, E* out, float* lse, const Dims& dm,
                                      int nrows, const int* rows, hipStream_t st);
hipError_t launch_permute_tokens(const void* in, void* out, const Dims& dm, int row_bytes, int to_pos_major,
                                 hipStream_t st);
// out <- (out + softmax(q K_F1^T / sqrt(d)) V_F1) / 2 for every token, K_F1 / V_F1 the head's first b rows
template <typename E>
hipError_t launch_sink_average_generic(const E* q, const E* k, const E* v, E* out, const Dims& dm, hipStream_t st);
// p[h * head_stride + r] = value for r < count, h < nheads
hipError_t launch_fill_head_prefix(float* p, float value, long long count, long long head_stride, int nheads,
                                   hipStream_t st);

// backward.hip : Alg. 2 on the plain ALUs (D_scratch: BH * N floats)
size_t entropy_bwd_scratch_bytes(const Dims& dm);
template <typename E>
hipError_t launch_entropy_bwd_generic(const E* q, const float* cR, const E* k, const E* v, const E* o, const E* dO,
                                      const float* lse, const float* H, const float* dH, E* dq, E* dk, E* dv,
                                      float* D_scratch, const Dims& dm, float row_scale, float cr_min, hipStream_t st);

// backward_mfma.hip : Alg. 2 on the MFMA units (bf16, d == 64 or 128; scratch: one float4 per query row)
bool entropy_bwd_mfma_supported(const Dims& dm);
size_t entropy_bwd_mfma_scratch_bytes(const Dims& dm);
hipError_t launch_entropy_bwd_mfma(const bf16_t* q, const float* cR, const bf16_t* k, const bf16_t* v,
                                   const bf16_t* o, const bf16_t* dO, const float* lse, const float* H,
                                   const float* dH, bf16_t* dq, bf16_t* dk, bf16_t* dv, void* scratch, const Dims& dm,
                                   float row_scale, float cr_min, hipStream_t st);

hipError_t launch_mfma_probe(const void* operands, float* out, int blocks, int iters, hipStream_t st);

// flash.hip : bf16 MFMA blocked-softmax kernels (d == 64 or 128)
bool flash_supported(const Dims& dm);
// lse (optional, may be null): natural-log sum-exp of every query row's logits
// fused: when v is given and the entropy is accumulated online, form alpha_L, c_L and y in one pass
// (flash_kv.hip) instead of two
hipError_t launch_r_update_flash(const bf16_t* aR, const float* cR, const bf16_t* k, const bf16_t* v, bf16_t* aL,
                                 float* cL, bf16_t* y, float* lse, const Dims& dm, float row_scale, float cr_min,
                                 int entropy_mode, bool fused, hipStream_t st);
// flash_kv.hip : alpha_L, c_L, lse (optional) and y of one R-update in a single pass (d == 64 or 128)
hipError_t launch_r_update_flash_fused(const bf16_t* aR, const float* cR, const bf16_t* k, const bf16_t* v, bf16_t* aL,
                                       float* cL, bf16_t* y, float* lse, const Dims& dm, float row_scale, float cr_min,
                                       hipStream_t st);
// flash2.hip : the same passes with one wave per SIMD and two query tiles per wave (d == 64 or 128);
// v == nullptr: alpha_L, c_L (fitting sweep); v given: also y, from one evaluation of the softmax
hipError_t launch_r_update_flash2(const bf16_t* aR, const float* cR, const bf16_t* k, const bf16_t* v, bf16_t* aL,
                                  float* cL, bf16_t* y, float* lse, const Dims& dm, float row_scale, float cr_min,
                                  int entropy_mode, hipStream_t st);
// exact attention of nrows query rows per head (starting where q / out / lse point) over all N keys
size_t first_frame_flash_scratch_bytes(const Dims& dm, int nrows);
// rows (device, may be null): a list of nrows row numbers within a head, used for every head; q / out / lse then
// point at row 0; entries outside [0, N) are skipped.  two_tile: contiguous rows go to flash2.hip's kernel
hipError_t launch_first_frame_flash(const bf16_t* q, const bf16_t* k, const bf16_t* v, bf16_t* out, float* lse,
                                    void* scratch, size_t scratch_bytes, const Dims& dm, int nrows, const int* rows,
                                    bool two_tile, hipStream_t st);
int flash2_query_block();  // query rows per workgroup of flash2.hip's kernel
// flash2.hip : the same pass (contiguous rows only) on the kernel with two query tiles per wave; the caller has cut the
// keys into ns ranges of keys_per_split and owns the partial-result buffers
hipError_t launch_first_frame_flash2(const bf16_t* q, const bf16_t* k, const bf16_t* v, bf16_t* out, float* lse,
                                     float* part_o, float* part_lse, const Dims& dm, int nrows, int ns,
                                     int keys_per_split, hipStream_t st);

// the temporal factor for any T <= 8128 through the same kernel (see flash.hip); lse_scratch: BH * N floats, fitting sweep only
bool temporal_flash_supported(const Dims& dm);
hipError_t launch_l_update_flash(const bf16_t* q, const bf16_t* aL, const float* cL, const bf16_t* y, bf16_t* aR, float* cR,
                                 bf16_t* out, float* lse_scratch, const Dims& dm, float q_scale, hipStream_t st);

hipError_t launch_sink_average_flash(const bf16_t* q, const bf16_t* k, const bf16_t* v, bf16_t* out, const Dims& dm,
                                     hipStream_t st);

// lpass.hip : bf16 MFMA temporal kernels (d == 64 or 128, T <= 128)
bool lpass_supported(const Dims& dm);
hipError_t launch_l_update_mfma(const bf16_t* q, const bf16_t* aL, const float* cL, const bf16_t* y, bf16_t* aR,
                                float* cR, bf16_t* out, const Dims& dm, float q_scale, hipStream_t st);

}  // namespace vm

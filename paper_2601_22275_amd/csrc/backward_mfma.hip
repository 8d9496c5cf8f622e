// bf16 MFMA kernels for the backward of one blocked-softmax pass with entropy (App. "Backward
// pass of Flash-Entropy-Attention", Alg. 2) on gfx950, d = 64 or 128.
//
// Alg. 2 adds into dQ in HBM from every key block.  Here the three results are produced by
// three passes that accumulate nothing across workgroups (bit-reproducible):
//   dQ pass:  a workgroup owns 256 query rows and streams the frame's K and V tiles;
//   dV pass:  a workgroup owns 256 key rows and streams the frame's Q and dO tiles;
//   dK pass:  the same, with dP = dO V^T and dS as well.
// All three are one kernel template.  The "owner" rows (32 per wave) stay in registers as B
// operands for the whole loop; the "stream" rows pass through LDS in 64-row tiles exactly as
// in the forward kernel (same direct global -> LDS loads, same swizzle, same transpose reads):
//   G^T = X1 R1^T          rows = stream rows, columns = owner rows; lane owns one owner row
//   (dP^T = X2 R2^T)       dQ and dK passes
//   E    = elementwise     P = exp(S - L), dS = P (dP - D) - dH P (S - L + H)   (Alg. 2)
//   acc^T += Xa^T E        B = E converted to bf16 in place, A = Xa^T by LDS transpose reads
// Per query row the elementwise step needs sc (logit scale), L, D, dH, H.  A small kernel
// reduces them to four floats per row, {sc2, l2, a, b} with t = S_raw sc2 - l2 (log2 units),
// P = 2^t and dS = P (dP - a - b t):  a = D + dH H,  b = dH ln 2.  In the dQ pass they are
// per-lane scalars; in the dV / dK passes the stream rows are queries and the four floats of
// each come from a small LDS tile that travels with the Q tile.
#include <type_traits>

#include "common.h"

namespace vm {

namespace {

constexpr int BK = 64;    // stream rows per LDS tile
constexpr int NW = 8;     // waves per workgroup, 32 owner rows each
constexpr int BO = 32 * NW;
constexpr int NSLOT = 4;
constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;

enum { MODE_DQ = 0, MODE_DV = 1, MODE_DK = 2 };

struct BwdParams {
  const bf16_t* q;
  const bf16_t* k;
  const bf16_t* v;
  const bf16_t* dO;
  const float4* stats;   // per query row {sc2, l2, a, b}
  bf16_t* out;           // dq, dv or dk
  int n;                 // rows per problem (b): owner rows and stream rows alike
  int nob;               // owner blocks per problem
  int total_blocks;
  int blocks_per_xcd;
};

__device__ __forceinline__ bf16x8 lds_read_b128(const char* p) { return *reinterpret_cast<const bf16x8*>(p); }
__device__ __forceinline__ bf16x4 lds_read_tr(const char* p) {
  return __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
      (bf16x4 __attribute__((address_space(3)))*)(reinterpret_cast<const bf16x4*>(p)));
}
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
  bf16x2 r;
  r[0] = (__bf16)a;
  r[1] = (__bf16)b;
  uint32_t u;
  __builtin_memcpy(&u, &r, 4);
  return u;
}

// Sixteen lanes per query row: D = dO . O (Alg. 2, before the loops) and the four floats above.
// d is a multiple of 8 here (64 or 128): a lane reads 16 bytes of each tensor at a time.
__global__ void __launch_bounds__(256) bwd_stats_kernel(const bf16_t* __restrict__ o, const bf16_t* __restrict__ dO,
                                                        const float* __restrict__ cR, const float* __restrict__ lse,
                                                        const float* __restrict__ H, const float* __restrict__ dH,
                                                        float4* __restrict__ stats, long long rows, int d,
                                                        float row_scale, float cr_min) {
  const long long row = (long long)blockIdx.x * 16 + (threadIdx.x >> 4);
  const int sub = threadIdx.x & 15;
  float s = 0.f;
  if (row < rows) {
    for (int c = sub * 8; c < d; c += 128) {
      const uint4 a = *reinterpret_cast<const uint4*>(o + row * d + c);
      const uint4 b = *reinterpret_cast<const uint4*>(dO + row * d + c);
      const uint32_t aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        s += __uint_as_float(aw[j] << 16) * __uint_as_float(bw[j] << 16);
        s += __uint_as_float(aw[j] & 0xffff0000u) * __uint_as_float(bw[j] & 0xffff0000u);
      }
    }
  }
  for (int off = 8; off >= 1; off >>= 1) s += __shfl_xor(s, off);
  if (sub == 0 && row < rows) {
    const float c = fmaxf(cR ? cR[row] : 1.f, cr_min);
    const float g = dH ? dH[row] : 0.f;
    float4 w;
    w.x = row_scale / c * LOG2E;
    w.y = lse[row] * LOG2E;
    w.z = s + g * H[row];
    w.w = g * LN2;
    stats[row] = w;
  }
}

template <int D, int MODE>
__global__ void __launch_bounds__(64 * NW) bwd_kernel(BwdParams P) {
  using G = RowGeo<D>;
  constexpr int ROW_BYTES = G::ROW_BYTES;
  constexpr int TILE_BYTES = BK * ROW_BYTES;
  constexpr int KS = G::KS;
  constexpr int CT = G::CT;
  constexpr int CH = G::CH;
  constexpr int RPI = G::RPI;
  constexpr bool STREAM_STATS = MODE != MODE_DQ;     // stream rows are queries
  constexpr bool WITH_DP = MODE != MODE_DV;
  constexpr int STATS_OFF = 2 * NSLOT * TILE_BYTES;  // [NSLOT][64] float4 after the two tile regions
  // which stream tile feeds the accumulation: dQ: K (= X1); dV: dO (= X2); dK: Q (= X1)
  constexpr int XA_OFF = MODE == MODE_DV ? NSLOT * TILE_BYTES : 0;
  auto swz = [](int row) { return G::swz(row); };
  extern __shared__ __attribute__((aligned(16))) char smem[];

  const int bid = blockIdx.x;
  const int wid = (bid & 7) * P.blocks_per_xcd + (bid >> 3);  // XCD-aware, as in the forward kernel
  if (wid >= P.total_blocks) return;
  const int prob = wid / P.nob;
  const int ob = wid - prob * P.nob;
  const int tid = threadIdx.x;
  const int wave = tid >> 6;
  const int lane = tid & 63;
  const int ql = lane & 31;
  const int g = lane >> 5;
  const int n = P.n;
  const int ntiles = (n + BK - 1) / BK;
  const long long row0 = (long long)prob * n;  // first row of the problem in every tensor

  // owner / stream tensors of this pass
  const bf16_t* r1 = (MODE == MODE_DQ ? P.q : P.k) + row0 * D;   // B of G^T
  const bf16_t* r2 = (MODE == MODE_DQ ? P.dO : P.v) + row0 * D;  // B of dP^T
  const bf16_t* x1 = (MODE == MODE_DQ ? P.k : P.q) + row0 * D;   // A of G^T
  const bf16_t* x2 = (MODE == MODE_DQ ? P.v : P.dO) + row0 * D;  // A of dP^T (dV pass: A^T of the accumulation)
  const float4* stats = P.stats + row0;

  // ---- stream tiles: global -> LDS, as in the forward kernel --------------------------------
  static_assert(BK % (RPI * NW) == 0, "every wave issues the same number of loads per tile");
  const int st_row = RPI * wave + lane / CH;
  const int st_lc = (lane % CH) ^ swz(st_row);
  const unsigned lds_base = (unsigned)(unsigned long long)(__attribute__((address_space(3))) char*)smem;
  auto issue_tile = [&](int t) {
    const unsigned kb = lds_base + (t & (NSLOT - 1)) * TILE_BYTES;
#pragma unroll
    for (int r = 0; r < BK / (RPI * NW); ++r) {
      const int row = min(t * BK + RPI * NW * r + st_row, n - 1);  // rows past the end: copies, masked below
      const bf16_t* s1 = x1 + (long long)row * D + st_lc * 8;
      const bf16_t* s2 = x2 + (long long)row * D + st_lc * 8;
      const unsigned dst = __builtin_amdgcn_readfirstlane(kb + (RPI * NW * r + RPI * wave) * ROW_BYTES);
      asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(s1), "s"(dst) : "memory", "m0");
      const unsigned dst2 = dst + NSLOT * TILE_BYTES;
      asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(s2), "s"(dst2) : "memory", "m0");
    }
    if (STREAM_STATS && wave == 0) {
      // the four floats of the tile's 64 query rows: one 16-byte load per lane
      const float4* s3 = stats + min(t * BK + lane, n - 1);
      const unsigned dst3 = __builtin_amdgcn_readfirstlane(lds_base + STATS_OFF + (t & (NSLOT - 1)) * (BK * 16));
      asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(s3), "s"(dst3) : "memory", "m0");
    }
  };
  issue_tile(0);
  if (ntiles > 1) issue_tile(1);

  // ---- owner rows: B operands in registers -----------------------------------------------
  const int orow_raw = ob * BO + wave * 32 + ql;
  const bool ovalid = orow_raw < n;
  const int orow = ovalid ? orow_raw : n - 1;
  bf16x8 reg1[KS], reg2[WITH_DP ? KS : 1];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) {
    reg1[ks] = *reinterpret_cast<const bf16x8*>(r1 + (long long)orow * D + 8 * g + 16 * ks);
    if (WITH_DP) reg2[ks] = *reinterpret_cast<const bf16x8*>(r2 + (long long)orow * D + 8 * g + 16 * ks);
  }
  float4 ost = {0.f, 0.f, 0.f, 0.f};  // dQ pass: the owner row is a query
  if (!STREAM_STATS) ost = stats[orow];

  int a_off[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) a_off[ks] = ql * ROW_BYTES + (((2 * ks + g) ^ swz(ql)) << 4);
  int t_off[CT][2];
  {
    const int rp = lane & 15;
    const int chh = (lane >> 4) & 1;
#pragma unroll
    for (int ct = 0; ct < CT; ++ct)
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        const int row = 8 * hh + 4 * g + (rp >> 2);
        const int lc = 4 * ct + 2 * chh + ((rp >> 1) & 1);
        t_off[ct][hh] = row * ROW_BYTES + ((lc ^ swz(row)) << 4) + ((rp & 1) << 3) + XA_OFF;
      }
  }

  f32x16 acc[CT];
#pragma unroll
  for (int ct = 0; ct < CT; ++ct)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[ct][r] = 0.f;
  const bool active = ob * BO + wave * 32 < n;  // a wave whose owner rows are all padding only loads tiles

  // ---- one 32-row sub-tile of the stream ---------------------------------------------------
  auto step = [&](const char* tile, const char* stile, int st, int rows_left) {
    f32x16 s, dp;
#pragma unroll
    for (int r = 0; r < 16; ++r) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      bf16x8 a = lds_read_b128(tile + st * 32 * ROW_BYTES + a_off[ks]);
      s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, reg1[ks], s, 0, 0, 0);
    }
    if (WITH_DP) {
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        bf16x8 a = lds_read_b128(tile + NSLOT * TILE_BYTES + st * 32 * ROW_BYTES + a_off[ks]);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, reg2[ks], dp, 0, 0, 0);
      }
    }
    // elementwise: register r is stream row 8 (r / 4) + 4 g + (r % 4) of the sub-tile
    float e[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int srow = 8 * (r >> 2) + 4 * g + (r & 3);
      float4 w = ost;
      if (STREAM_STATS) w = *reinterpret_cast<const float4*>(stile + (st * 32 + srow) * 16);
      float t = __builtin_fmaf(s[r], w.x, -w.y);
      if (srow >= rows_left) t = -1.0e9f;  // rows past the end are copies of the last row: weight zero
      const float p = __builtin_amdgcn_exp2f(t);
      if (MODE == MODE_DV) {
        e[r] = p;
      } else {
        const float ds = p * (dp[r] - w.z - w.w * t);
        e[r] = MODE == MODE_DK ? ds * (w.x * (1.0f / LOG2E)) : ds;  // dK carries the query's logit scale
      }
    }
    bf16x8 eb[2];
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      uint32_t w4[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) w4[j] = pack_bf16(e[8 * c + 2 * j], e[8 * c + 2 * j + 1]);
      __builtin_memcpy(&eb[c], w4, 16);
    }
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      const int off = (st * 32 + c * 16) * ROW_BYTES;
#pragma unroll
      for (int ct = 0; ct < CT; ++ct) {
        bf16x4 lo = lds_read_tr(tile + off + t_off[ct][0]);
        bf16x4 hi = lds_read_tr(tile + off + t_off[ct][1]);
        bf16x8 a = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        acc[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, eb[c], acc[ct], 0, 0, 0);
      }
    }
  };

  // Tile t sits in slot t & 3 and is requested two iterations ahead; the barrier at the top
  // of iteration t publishes it (every wave has waited for its own part) and retires tile t-2.
  for (int t = 0; t < ntiles; ++t) {
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (t + 2 < ntiles) issue_tile(t + 2);
    if (active) {
      const char* tile = smem + (t & 3) * TILE_BYTES;
      const char* stile = smem + STATS_OFF + (t & 3) * (BK * 16);
      const int left = n - t * BK;
      step(tile, stile, 0, left);
      step(tile, stile, 1, left - 32);
    }
  }

  // ---- epilogue: rows staged in LDS, written as whole lines ---------------------------------
  __syncthreads();
  char* stage = smem + wave * (32 * ROW_BYTES);
  const float oscale = MODE == MODE_DQ ? ost.x * (1.0f / LOG2E) : 1.0f;  // dq carries its own row's logit scale
#pragma unroll
  for (int ct = 0; ct < CT; ++ct)
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      uint2 w;
      w.x = pack_bf16(acc[ct][4 * c + 0] * oscale, acc[ct][4 * c + 1] * oscale);
      w.y = pack_bf16(acc[ct][4 * c + 2] * oscale, acc[ct][4 * c + 3] * oscale);
      *reinterpret_cast<uint2*>(stage + ql * ROW_BYTES + (((4 * ct + c) ^ swz(ql)) << 4) + 8 * g) = w;
    }
  __builtin_amdgcn_s_waitcnt(0xc07f);  // lgkmcnt(0): the staged rows are private to the wave
  __builtin_amdgcn_wave_barrier();
  const int row_first = ob * BO + wave * 32;
#pragma unroll
  for (int ps = 0; ps < 32 / RPI; ++ps) {
    const int lr = ps * RPI + lane / CH;
    const int pc = lane % CH;
    const int lc = pc ^ swz(lr);
    if (row_first + lr < n) {
      uint4 w = *reinterpret_cast<const uint4*>(stage + lr * ROW_BYTES + pc * 16);
      *reinterpret_cast<uint4*>(P.out + (row0 + row_first + lr) * D + lc * 8) = w;
    }
  }
}

template <int D, int MODE>
hipError_t launch_bwd(const BwdParams& P, hipStream_t st) {
  constexpr int LDS_BYTES = 2 * NSLOT * BK * D * 2 + NSLOT * BK * 16;
  auto kern = bwd_kernel<D, MODE>;
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
    if (e != hipSuccess) return e;
    configured = true;
  }
  hipLaunchKernelGGL(kern, dim3(P.blocks_per_xcd * 8), dim3(64 * NW), LDS_BYTES, st, P);
  return hipGetLastError();
}

}  // namespace

bool entropy_bwd_mfma_supported(const Dims& dm) { return dm.d == 128 || dm.d == 64; }
size_t entropy_bwd_mfma_scratch_bytes(const Dims& dm) { return (size_t)dm.BH * dm.N * sizeof(float4); }

hipError_t launch_entropy_bwd_mfma(const bf16_t* q, const float* cR, const bf16_t* k, const bf16_t* v,
                                   const bf16_t* o, const bf16_t* dO, const float* lse, const float* H,
                                   const float* dH, bf16_t* dq, bf16_t* dk, bf16_t* dv, void* scratch, const Dims& dm,
                                   float row_scale, float cr_min, hipStream_t st) {
  const long long rows = (long long)dm.BH * dm.N;
  if (rows > 0x7fffffffLL) return hipErrorInvalidValue;
  float4* stats = (float4*)scratch;
  hipLaunchKernelGGL(bwd_stats_kernel, dim3((unsigned)((rows + 15) / 16)), dim3(256), 0, st, o, dO, cR, lse, H, dH,
                     stats, rows, dm.d, row_scale, cr_min);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  BwdParams P = {};
  P.q = q; P.k = k; P.v = v; P.dO = dO; P.stats = stats;
  P.n = dm.b;
  P.nob = (dm.b + BO - 1) / BO;
  const long long total = (long long)dm.BH * dm.T * P.nob;
  if (total > 0x3fffffffLL) return hipErrorInvalidValue;
  P.total_blocks = (int)total;
  P.blocks_per_xcd = (P.total_blocks + 7) / 8;
  auto run = [&](auto dc) -> hipError_t {
    constexpr int D = decltype(dc)::value;
    P.out = dq;
    hipError_t e2 = launch_bwd<D, MODE_DQ>(P, st);
    if (e2 != hipSuccess) return e2;
    P.out = dv;
    e2 = launch_bwd<D, MODE_DV>(P, st);
    if (e2 != hipSuccess) return e2;
    P.out = dk;
    return launch_bwd<D, MODE_DK>(P, st);
  };
  return dm.d == 128 ? run(std::integral_constant<int, 128>{}) : run(std::integral_constant<int, 64>{});
}

}  // namespace vm

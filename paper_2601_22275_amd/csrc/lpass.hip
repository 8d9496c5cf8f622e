// bf16 MFMA kernel for the L-update, the inter-frame (temporal) factor (Eq. L with
// Eq. alpha_R/c_R; App. A L_update), and for the final apply O = L y (App. A) on gfx950.
//
// One workgroup per (spatial position i, batch*head).  Its T query rows Q[:, i, :], the T
// rows alpha_L[:, i, :] (and y[:, i, :] on the last sweep) sit b*d elements apart in HBM:
// the stride permutation P of Sec. 3.1 is applied here, as addressing while the rows are
// gathered into LDS, and undone when the result rows are scattered back.  T is padded to
// TP = 32 * NW and wave w owns query frames 32w .. 32w+31:
//
//   U^T = aL Q^T        A = alpha_L rows from LDS, B = Q^T of the wave's frames.  Lane (j, g)
//                       then holds logits of query frame j for half of the key frames, so the
//                       softmax over key frames k is an in-lane reduction plus one exchange.
//   last sweep:         O^T = y^T L^T, B = L^T straight from the softmax registers,
//                       A = y^T by LDS transpose reads.
//   fitting sweep:      L goes to LDS as bf16 [j][k]; wave w then forms
//                       alpha_R^T[:, k-tile w] = Q^T L (contraction over all query frames j,
//                       both operands by LDS transpose reads) and c_R = 1^T L by one extra
//                       MFMA per step with an all-ones A operand.
// Results are staged in LDS and leave as whole rows.  Instantiated for d = 128 and d = 64.
#include "common.h"

namespace vm {

namespace {

constexpr float LOG2E = 1.4426950408889634f;

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

template <int D, int NW>
struct Lay {
  static constexpr int ROW_BYTES = RowGeo<D>::ROW_BYTES;
  static constexpr int TP = 32 * NW;
  static constexpr int TOK = TP * ROW_BYTES;       // one gathered tensor
  static constexpr int LMS = TP * 2 + 16;          // row stride of the bf16 L block
  static constexpr int OFF_Q = 0;
  static constexpr int OFF_A = TOK;
  static constexpr int OFF_X = 2 * TOK;            // y (last sweep) or the L block (fitting sweep)
  static constexpr int X_BYTES_FINAL = TOK;
  static constexpr int X_BYTES_FIT = TP * LMS;
  static constexpr int bytes(bool fin) { return 2 * TOK + (fin ? X_BYTES_FINAL : X_BYTES_FIT) + TP * 4; }
};

template <int D, int NW, bool FINAL>
__global__ void __launch_bounds__(64 * NW) l_update_mfma_kernel(const bf16_t* __restrict__ q,
                                                                const bf16_t* __restrict__ aL,
                                                                const float* __restrict__ cL,
                                                                const bf16_t* __restrict__ y, bf16_t* __restrict__ aR,
                                                                float* __restrict__ cR, bf16_t* __restrict__ out, int T,
                                                                int b, float q_scale) {
  using LY = Lay<D, NW>;
  using G = RowGeo<D>;
  constexpr int TP = LY::TP;
  constexpr int ROW_BYTES = G::ROW_BYTES;
  constexpr int CH = G::CH;    // 16-byte chunks per row
  constexpr int KS = G::KS;    // k-steps of a contraction over d
  constexpr int VT = G::CT;    // 32-channel tiles of a result row
  constexpr int RPI = G::RPI;  // rows covered by 64 lanes x 16 bytes
  auto swz = [](int row) { return G::swz(row); };
  extern __shared__ __attribute__((aligned(16))) char smem[];
  char* Qs = smem + LY::OFF_Q;
  char* As = smem + LY::OFF_A;
  char* Xs = smem + LY::OFF_X;
  float* sCL = reinterpret_cast<float*>(smem + LY::OFF_X + (FINAL ? LY::X_BYTES_FINAL : LY::X_BYTES_FIT));

  const int i = blockIdx.x;
  const long long head0 = (long long)blockIdx.y * T * b;
  const int tid = threadIdx.x;
  const int wave = tid >> 6;
  const int lane = tid & 63;
  const int ql = lane & 31;
  const int g = lane >> 5;

  // ---- gather the position's rows (stride b*d in HBM) into LDS -----------------------
  {
    const int sub = tid / CH;        // row within a pass
    const int pc = tid % CH;         // physical 16-byte chunk
    constexpr int NPS = 32 / RPI;    // passes: RPI * NW rows each
    uint4 rq[NPS], ra[NPS], ry[NPS];
#pragma unroll
    for (int ps = 0; ps < NPS; ++ps) {
      const int row = ps * RPI * NW + sub;
      const int lc = pc ^ swz(row);
      uint4 z = {0u, 0u, 0u, 0u};
      rq[ps] = z; ra[ps] = z;
      if (FINAL) ry[ps] = z;
      if (row < T) {
        const long long e = (head0 + (long long)row * b + i) * D + lc * 8;
        rq[ps] = *reinterpret_cast<const uint4*>(q + e);
        ra[ps] = *reinterpret_cast<const uint4*>(aL + e);
        if (FINAL) ry[ps] = *reinterpret_cast<const uint4*>(y + e);
      }
    }
    for (int kk = tid; kk < TP; kk += 64 * NW) sCL[kk] = kk < T ? cL[head0 + (long long)kk * b + i] * LOG2E : 0.f;
#pragma unroll
    for (int ps = 0; ps < NPS; ++ps) {
      const int row = ps * RPI * NW + sub;
      *reinterpret_cast<uint4*>(Qs + row * ROW_BYTES + pc * 16) = rq[ps];
      *reinterpret_cast<uint4*>(As + row * ROW_BYTES + pc * 16) = ra[ps];
      if (FINAL) *reinterpret_cast<uint4*>(Xs + row * ROW_BYTES + pc * 16) = ry[ps];
    }
  }
  __syncthreads();

  // ---- U^T = aL Q^T for the wave's 32 query frames -------------------------------------
  const int jrow = 32 * wave + ql;  // query frame of this lane
  bf16x8 qreg[KS];
#pragma unroll
  for (int ks = 0; ks < KS; ++ks)
    qreg[ks] = lds_read_b128(Qs + jrow * ROW_BYTES + (((2 * ks + g) ^ swz(ql)) << 4));
  f32x16 u[NW];
#pragma unroll
  for (int kt = 0; kt < NW; ++kt) {
#pragma unroll
    for (int r = 0; r < 16; ++r) u[kt][r] = 0.f;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      bf16x8 a = lds_read_b128(As + (32 * kt + ql) * ROW_BYTES + (((2 * ks + g) ^ swz(ql)) << 4));
      u[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[ks], u[kt], 0, 0, 0);
    }
  }
  // ---- softmax over key frames k (Eq. L), base-2 ------------------------------------------
  const float qs2 = q_scale * LOG2E;
  float mx = -3.0e38f;
#pragma unroll
  for (int kt = 0; kt < NW; ++kt)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int kf = 32 * kt + 8 * (r >> 2) + 4 * g + (r & 3);
      float val = __builtin_fmaf(u[kt][r], qs2, -sCL[kf]);
      if (kf >= T) val = -3.0e38f;
      u[kt][r] = val;
      mx = fmaxf(mx, val);
    }
  mx = fmaxf(mx, __shfl_xor(mx, 32));
  float sum = 0.f;
#pragma unroll
  for (int kt = 0; kt < NW; ++kt)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      float p = __builtin_amdgcn_exp2f(u[kt][r] - mx);
      u[kt][r] = p;
      sum += p;
    }
  sum += __shfl_xor(sum, 32);
  const float inv = (jrow < T) ? 1.0f / sum : 0.f;  // padded query frames contribute nothing
  if (!FINAL) {
#pragma unroll
    for (int kt = 0; kt < NW; ++kt)
#pragma unroll
      for (int r = 0; r < 16; ++r) u[kt][r] *= inv;
  }

  // transpose-read geometry shared by both second contractions
  const int rp = lane & 15;
  const int chh = (lane >> 4) & 1;
  f32x16 acc[VT];
#pragma unroll
  for (int vt = 0; vt < VT; ++vt)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[vt][r] = 0.f;

  char* Os;  // staging rows for the coalesced copy-out
  if (FINAL) {
    // ---- O^T = y^T L^T : contraction over key frames, B straight from registers ------------
    // The unnormalised 2^(u - max) go in as bf16 and the result is divided by the sum of those
    // ROUNDED values, so each output row is an exact convex combination of the y rows.
    typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
    bf16x2 ones2;
    ones2[0] = (__bf16)1.0f;
    ones2[1] = (__bf16)1.0f;
    float sumt = 0.f;
#pragma unroll
    for (int kt = 0; kt < NW; ++kt)
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        uint32_t w[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          w[e] = pack_bf16(u[kt][8 * c + 2 * e], u[kt][8 * c + 2 * e + 1]);
          bf16x2 pr;
          __builtin_memcpy(&pr, &w[e], 4);
          sumt = __builtin_amdgcn_fdot2_f32_bf16(pr, ones2, sumt, false);
        }
        bf16x8 pb;
        __builtin_memcpy(&pb, w, 16);
#pragma unroll
        for (int vt = 0; vt < VT; ++vt) {
          bf16x4 part[2];
#pragma unroll
          for (int hh = 0; hh < 2; ++hh) {
            const int key = 32 * kt + 16 * c + 8 * hh + 4 * g + (rp >> 2);
            const int lc = 4 * vt + 2 * chh + ((rp >> 1) & 1);
            part[hh] = lds_read_tr(Xs + key * ROW_BYTES + ((lc ^ swz(key)) << 4) + ((rp & 1) << 3));
          }
          bf16x8 a = __builtin_shufflevector(part[0], part[1], 0, 1, 2, 3, 4, 5, 6, 7);
          acc[vt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pb, acc[vt], 0, 0, 0);
        }
      }
    sumt += __shfl_xor(sumt, 32);
    const float invt = 1.0f / sumt;
#pragma unroll
    for (int vt = 0; vt < VT; ++vt)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[vt][r] *= invt;
    Os = Qs;  // rows 32w..32w+31 of Qs are read by this wave only, and it is done with them
  } else {
    // ---- L to LDS as bf16 [j][k] -------------------------------------------------------------
#pragma unroll
    for (int kt = 0; kt < NW; ++kt)
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        uint2 w;
        w.x = pack_bf16(u[kt][4 * c + 0], u[kt][4 * c + 1]);
        w.y = pack_bf16(u[kt][4 * c + 2], u[kt][4 * c + 3]);
        *reinterpret_cast<uint2*>(Xs + jrow * LY::LMS + (32 * kt + 8 * c + 4 * g) * 2) = w;
      }
    __syncthreads();
    // ---- alpha_R^T[:, k-tile w] = Q^T L and c_R = 1^T L : contraction over query frames j ----
    f32x16 accone;
#pragma unroll
    for (int r = 0; r < 16; ++r) accone[r] = 0.f;
    bf16x8 ones;
    {
      uint32_t w[4] = {0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u};
      __builtin_memcpy(&ones, w, 16);
    }
#pragma unroll
    for (int js = 0; js < TP / 16; ++js) {
      bf16x4 lpart[2];
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        const int j = 16 * js + 8 * hh + 4 * g + (rp >> 2);
        lpart[hh] = lds_read_tr(Xs + j * LY::LMS + (32 * wave + 16 * chh + 4 * (rp & 3)) * 2);
      }
      bf16x8 bL = __builtin_shufflevector(lpart[0], lpart[1], 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
      for (int vt = 0; vt < VT; ++vt) {
        bf16x4 part[2];
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
          const int j = 16 * js + 8 * hh + 4 * g + (rp >> 2);
          const int lc = 4 * vt + 2 * chh + ((rp >> 1) & 1);
          part[hh] = lds_read_tr(Qs + j * ROW_BYTES + ((lc ^ swz(j)) << 4) + ((rp & 1) << 3));
        }
        bf16x8 a = __builtin_shufflevector(part[0], part[1], 0, 1, 2, 3, 4, 5, 6, 7);
        acc[vt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bL, acc[vt], 0, 0, 0);
      }
      accone = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ones, bL, accone, 0, 0, 0);
    }
    if (g == 0 && jrow < T) cR[head0 + (long long)jrow * b + i] = accone[0];  // jrow doubles as key frame 32w+ql
    Os = As;  // alpha_L is dead after the barrier above; wave w writes rows 32w..32w+31 only
  }

  // ---- stage the wave's 32 result rows and write them out as whole rows ---------------------
#pragma unroll
  for (int vt = 0; vt < VT; ++vt)
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      uint2 w;
      w.x = pack_bf16(acc[vt][4 * c + 0], acc[vt][4 * c + 1]);
      w.y = pack_bf16(acc[vt][4 * c + 2], acc[vt][4 * c + 3]);
      *reinterpret_cast<uint2*>(Os + jrow * ROW_BYTES + (((4 * vt + c) ^ swz(ql)) << 4) + 8 * g) = w;
    }
  __syncthreads();
  bf16_t* dst = FINAL ? out : aR;
#pragma unroll
  for (int ps = 0; ps < 32 / RPI; ++ps) {
    const int row = 32 * wave + ps * RPI + lane / CH;
    const int pc = lane % CH;
    const int lc = pc ^ swz(row);
    if (row < T) {
      uint4 w = *reinterpret_cast<const uint4*>(Os + row * ROW_BYTES + pc * 16);
      *reinterpret_cast<uint4*>(dst + (head0 + (long long)row * b + i) * D + lc * 8) = w;
    }
  }
}

template <int D, int NW, bool FINAL>
hipError_t launch_nw(const bf16_t* q, const bf16_t* aL, const float* cL, const bf16_t* y, bf16_t* aR, float* cR,
                     bf16_t* out, const Dims& dm, float q_scale, hipStream_t st) {
  auto kern = l_update_mfma_kernel<D, NW, FINAL>;
  const int lds = Lay<D, NW>::bytes(FINAL);
  if (lds > 48 * 1024) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
  }
  hipLaunchKernelGGL(kern, dim3(dm.b, dm.BH), dim3(64 * NW), lds, st, q, aL, cL, y, aR, cR, out, dm.T, dm.b, q_scale);
  return hipGetLastError();
}

template <int D, bool FINAL>
hipError_t launch_fin(const bf16_t* q, const bf16_t* aL, const float* cL, const bf16_t* y, bf16_t* aR, float* cR,
                      bf16_t* out, const Dims& dm, float q_scale, hipStream_t st) {
  const int nw = (dm.T + 31) / 32;
  switch (nw) {
    case 1: return launch_nw<D, 1, FINAL>(q, aL, cL, y, aR, cR, out, dm, q_scale, st);
    case 2: return launch_nw<D, 2, FINAL>(q, aL, cL, y, aR, cR, out, dm, q_scale, st);
    case 3: return launch_nw<D, 3, FINAL>(q, aL, cL, y, aR, cR, out, dm, q_scale, st);
    case 4: return launch_nw<D, 4, FINAL>(q, aL, cL, y, aR, cR, out, dm, q_scale, st);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace

bool lpass_supported(const Dims& dm) { return (dm.d == 128 || dm.d == 64) && dm.T <= 128; }

hipError_t launch_l_update_mfma(const bf16_t* q, const bf16_t* aL, const float* cL, const bf16_t* y, bf16_t* aR,
                                float* cR, bf16_t* out, const Dims& dm, float q_scale, hipStream_t st) {
  if (dm.d == 128) {
    if (y != nullptr) return launch_fin<128, true>(q, aL, cL, y, aR, cR, out, dm, q_scale, st);
    return launch_fin<128, false>(q, aL, cL, y, aR, cR, out, dm, q_scale, st);
  }
  if (y != nullptr) return launch_fin<64, true>(q, aL, cL, y, aR, cR, out, dm, q_scale, st);
  return launch_fin<64, false>(q, aL, cL, y, aR, cR, out, dm, q_scale, st);
}

}  // namespace vm

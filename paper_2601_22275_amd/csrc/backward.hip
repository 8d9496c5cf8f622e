// Backward of one blocked-softmax pass with entropy (App. "Backward pass of
// Flash-Entropy-Attention", Alg. 2), plain-ALU kernels: any b and d <= 256, float or bf16
// tensors, float arithmetic.  Alg. 2 walks key blocks outside and query blocks inside and adds
// into dQ in HBM; here the two sums are separated so that nothing is accumulated across
// workgroups: one kernel owns a query row (dQ), one a key row (dK, dV), both recompute
// P = exp(S - L) from the stored log-sum-exp.  Results are bit-reproducible.
#include "common.h"

namespace vm {

namespace {

constexpr int kMaxD = 256;

// D = rowsum(dO o O), one wave per row (Alg. 2, the line before the loops)
template <typename E>
__global__ void __launch_bounds__(64) bwd_rowdot_kernel(const E* __restrict__ o, const E* __restrict__ dO,
                                                        float* __restrict__ D, int d) {
  const long long row = blockIdx.x;
  float s = 0.f;
  for (int c = threadIdx.x; c < d; c += 64) s += load_f<E>(o + row * d + c) * load_f<E>(dO + row * d + c);
  for (int off = 32; off >= 1; off >>= 1) s += __shfl_xor(s, off);
  if (threadIdx.x == 0) D[row] = s;
}

// The element of dS for query statistics (sc, lse, H, dH, D) and raw dot products qk = q . k,
// dov = dO . v:  S = sc * qk, P = exp(S - lse), dS = P (dov - D) - dH P (S - lse + H).
__device__ __forceinline__ void ds_element(float qk, float dov, float sc, float lse, float H, float dH, float D,
                                           float& P, float& dS) {
  const float S = sc * qk;
  P = expf(S - lse);
  dS = P * (dov - D) - dH * P * (S - lse + H);
}

// One wave per query row i of frame kf: dq[i] = sc_i * sum_l dS[i,l] K[l].
template <typename E>
__global__ void __launch_bounds__(64) bwd_dq_kernel(const E* __restrict__ q, const float* __restrict__ cR,
                                                    const E* __restrict__ k, const E* __restrict__ v,
                                                    const E* __restrict__ dO, const float* __restrict__ lse,
                                                    const float* __restrict__ H, const float* __restrict__ dH,
                                                    const float* __restrict__ D, E* __restrict__ dq, int T, int b,
                                                    int d, float row_scale, float cr_min) {
  __shared__ float sq[kMaxD], sdo[kMaxD], sp[64];
  const int lane = threadIdx.x;
  const int i = blockIdx.x, kf = blockIdx.y, bh = blockIdx.z;
  const long long frame0 = ((long long)bh * T + kf) * b;
  const long long row = frame0 + i;
  for (int c = lane; c < d; c += 64) {
    sq[c] = load_f<E>(q + row * d + c);
    sdo[c] = load_f<E>(dO + row * d + c);
  }
  __syncthreads();
  const float sc = row_scale / fmaxf(cR ? cR[row] : 1.f, cr_min);
  const float l_i = lse[row], H_i = H[row], dH_i = dH ? dH[row] : 0.f, D_i = D[row];
  float acc[kMaxD / 64];
#pragma unroll
  for (int u = 0; u < kMaxD / 64; ++u) acc[u] = 0.f;
  for (int l0 = 0; l0 < b; l0 += 64) {
    const int l = l0 + lane;
    float dS = 0.f;
    if (l < b) {
      const E* kr = k + (frame0 + l) * d;
      const E* vr = v + (frame0 + l) * d;
      float qk = 0.f, dov = 0.f;
      for (int c = 0; c < d; ++c) {
        qk += sq[c] * load_f<E>(kr + c);
        dov += sdo[c] * load_f<E>(vr + c);
      }
      float P;
      ds_element(qk, dov, sc, l_i, H_i, dH_i, D_i, P, dS);
    }
    __syncthreads();
    sp[lane] = dS;
    __syncthreads();
    const int cnt = b - l0 < 64 ? b - l0 : 64;
    for (int t = 0; t < cnt; ++t) {
      const float w = sp[t];
#pragma unroll
      for (int u = 0; u < kMaxD / 64; ++u) {
        const int c = lane + 64 * u;
        if (c < d) acc[u] += w * load_f<E>(k + (frame0 + l0 + t) * d + c);
      }
    }
  }
#pragma unroll
  for (int u = 0; u < kMaxD / 64; ++u) {
    const int c = lane + 64 * u;
    if (c < d) store_f<E>(dq + row * d + c, sc * acc[u]);
  }
}

// One wave per key row l of frame kf: dk[l] = sum_i sc_i dS[i,l] q[i], dv[l] = sum_i P[i,l] dO[i].
template <typename E>
__global__ void __launch_bounds__(64) bwd_dkv_kernel(const E* __restrict__ q, const float* __restrict__ cR,
                                                     const E* __restrict__ k, const E* __restrict__ v,
                                                     const E* __restrict__ dO, const float* __restrict__ lse,
                                                     const float* __restrict__ H, const float* __restrict__ dH,
                                                     const float* __restrict__ D, E* __restrict__ dk,
                                                     E* __restrict__ dv, int T, int b, int d, float row_scale,
                                                     float cr_min) {
  __shared__ float sk[kMaxD], sv[kMaxD], sds[64], spp[64];
  const int lane = threadIdx.x;
  const int l = blockIdx.x, kf = blockIdx.y, bh = blockIdx.z;
  const long long frame0 = ((long long)bh * T + kf) * b;
  const long long krow = frame0 + l;
  for (int c = lane; c < d; c += 64) {
    sk[c] = load_f<E>(k + krow * d + c);
    sv[c] = load_f<E>(v + krow * d + c);
  }
  __syncthreads();
  float acck[kMaxD / 64], accv[kMaxD / 64];
#pragma unroll
  for (int u = 0; u < kMaxD / 64; ++u) { acck[u] = 0.f; accv[u] = 0.f; }
  for (int i0 = 0; i0 < b; i0 += 64) {
    const int i = i0 + lane;
    float w = 0.f, P = 0.f;
    if (i < b) {
      const long long row = frame0 + i;
      const E* qr = q + row * d;
      const E* dor = dO + row * d;
      float qk = 0.f, dov = 0.f;
      for (int c = 0; c < d; ++c) {
        qk += load_f<E>(qr + c) * sk[c];
        dov += load_f<E>(dor + c) * sv[c];
      }
      const float sc = row_scale / fmaxf(cR ? cR[row] : 1.f, cr_min);
      float dS;
      ds_element(qk, dov, sc, lse[row], H[row], dH ? dH[row] : 0.f, D[row], P, dS);
      w = sc * dS;
    }
    __syncthreads();
    sds[lane] = w;
    spp[lane] = P;
    __syncthreads();
    const int cnt = b - i0 < 64 ? b - i0 : 64;
    for (int t = 0; t < cnt; ++t) {
      const float wt = sds[t], pt = spp[t];
#pragma unroll
      for (int u = 0; u < kMaxD / 64; ++u) {
        const int c = lane + 64 * u;
        if (c < d) {
          acck[u] += wt * load_f<E>(q + (frame0 + i0 + t) * d + c);
          accv[u] += pt * load_f<E>(dO + (frame0 + i0 + t) * d + c);
        }
      }
    }
  }
#pragma unroll
  for (int u = 0; u < kMaxD / 64; ++u) {
    const int c = lane + 64 * u;
    if (c < d) {
      store_f<E>(dk + krow * d + c, acck[u]);
      store_f<E>(dv + krow * d + c, accv[u]);
    }
  }
}

}  // namespace

size_t entropy_bwd_scratch_bytes(const Dims& dm) { return (size_t)dm.BH * dm.N * sizeof(float); }

template <typename E>
hipError_t launch_entropy_bwd_generic(const E* q, const float* cR, const E* k, const E* v, const E* o, const E* dO,
                                      const float* lse, const float* H, const float* dH, E* dq, E* dk, E* dv,
                                      float* D_scratch, const Dims& dm, float row_scale, float cr_min,
                                      hipStream_t st) {
  const long long rows = (long long)dm.BH * dm.N;
  if (rows > 0x7fffffffLL) return hipErrorInvalidValue;
  hipLaunchKernelGGL((bwd_rowdot_kernel<E>), dim3((unsigned)rows), dim3(64), 0, st, o, dO, D_scratch, dm.d);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  dim3 grid(dm.b, dm.T, dm.BH);
  hipLaunchKernelGGL((bwd_dq_kernel<E>), grid, dim3(64), 0, st, q, cR, k, v, dO, lse, H, dH, D_scratch, dq, dm.T, dm.b,
                     dm.d, row_scale, cr_min);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((bwd_dkv_kernel<E>), grid, dim3(64), 0, st, q, cR, k, v, dO, lse, H, dH, D_scratch, dk, dv, dm.T,
                     dm.b, dm.d, row_scale, cr_min);
  return hipGetLastError();
}

template hipError_t launch_entropy_bwd_generic<float>(const float*, const float*, const float*, const float*,
                                                      const float*, const float*, const float*, const float*,
                                                      const float*, float*, float*, float*, float*, const Dims&, float,
                                                      float, hipStream_t);
template hipError_t launch_entropy_bwd_generic<bf16_t>(const bf16_t*, const float*, const bf16_t*, const bf16_t*,
                                                       const bf16_t*, const bf16_t*, const float*, const float*,
                                                       const float*, bf16_t*, bf16_t*, bf16_t*, float*, const Dims&,
                                                       float, float, hipStream_t);

}  // namespace vm

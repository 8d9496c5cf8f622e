// Plain-ALU kernels for spatio-temporal Monarch attention: any T, b and d <= 256, float or
// bf16 tensors, float accumulation.  They serve the fp32 entry points and every bf16 shape
// the MFMA kernels do not cover.  Written for clarity first; each follows the paper's
// update equations directly (Sec. 3.1 Eqs. R / alpha_L, c_L / L / alpha_R, c_R; App. A).
#include "common.h"

namespace vm {

namespace {

constexpr int kMaxD = 256;

struct EntState {  // App. B running state: max, sum exp(x-m), sum exp(x-m)(x-m)
  float m, S, L;
};

__device__ __forceinline__ EntState ent_merge(EntState a, EntState c) {
  // Combine two partial states; the rescale rule of App. B applied to both sides.
  float mm = fmaxf(a.m, c.m);
  EntState r;
  r.m = mm;
  float da = a.S > 0.f ? a.m - mm : 0.f;
  float dc = c.S > 0.f ? c.m - mm : 0.f;
  float ea = a.S > 0.f ? expf(da) : 0.f;
  float ec = c.S > 0.f ? expf(dc) : 0.f;
  r.S = a.S * ea + c.S * ec;
  r.L = a.L * ea + a.S * ea * da + c.L * ec + c.S * ec * dc;
  return r;
}

// One wave (64 lanes) per query row.  nk keys starting at kbase (and vbase) with row
// stride d.  Emits out_k = softmax(z) K (if OUT_K), out_v = softmax(z) V (if OUT_V) and
// cl = sum p log p (if cl != nullptr) and lse = log sum exp z (if lse != nullptr), with
// z = scale * (qrow . K[l]).  BLEND: out_v <- (out_v + softmax(z) V) / 2 instead.
template <typename E, bool OUT_K, bool OUT_V, bool BLEND = false>
__device__ void attend_row(const E* __restrict__ qrow, float scale, const E* __restrict__ kbase,
                           const E* __restrict__ vbase, long long nk, int d, E* __restrict__ out_k,
                           E* __restrict__ out_v, float* __restrict__ cl, float* __restrict__ lse, float* sq,
                           float* sp) {
  const int lane = threadIdx.x;
  for (int c = lane; c < d; c += 64) sq[c] = load_f<E>(qrow + c);
  __syncthreads();
  // pass 1: online (m, S, L) per lane over its keys, App. B recurrences
  EntState st = {-INFINITY, 0.f, 0.f};
  for (long long l = lane; l < nk; l += 64) {
    const E* kr = kbase + l * d;
    float z = 0.f;
    for (int c = 0; c < d; ++c) z += sq[c] * load_f<E>(kr + c);
    z *= scale;
    float mn = fmaxf(st.m, z);
    if (mn > st.m && st.S > 0.f) {
      float dl = st.m - mn;
      float al = expf(dl);
      st.L = st.L * al + st.S * al * dl;
      st.S = st.S * al;
    }
    float p = expf(z - mn);
    st.S += p;
    st.L += p * (z - mn);
    st.m = mn;
  }
  for (int off = 32; off >= 1; off >>= 1) {
    EntState o;
    o.m = __shfl_xor(st.m, off);
    o.S = __shfl_xor(st.S, off);
    o.L = __shfl_xor(st.L, off);
    st = ent_merge(st, o);
  }
  const float lse_shift = st.m;
  const float inv_S = 1.f / st.S;
  if (cl != nullptr && lane == 0) *cl = -(logf(st.S) - st.L * inv_S);  // c_L = -H
  if (lse != nullptr && lane == 0) *lse = st.m + logf(st.S);
  // pass 2: out = sum_l p_l row_l, 64 keys at a time through LDS
  float acck[kMaxD / 64], accv[kMaxD / 64];
#pragma unroll
  for (int u = 0; u < kMaxD / 64; ++u) { acck[u] = 0.f; accv[u] = 0.f; }
  for (long long l0 = 0; l0 < nk; l0 += 64) {
    long long l = l0 + lane;
    float p = 0.f;
    if (l < nk) {
      const E* kr = kbase + l * d;
      float z = 0.f;
      for (int c = 0; c < d; ++c) z += sq[c] * load_f<E>(kr + c);
      p = expf(z * scale - lse_shift) * inv_S;
    }
    __syncthreads();
    sp[lane] = p;
    __syncthreads();
    int cnt = (int)((nk - l0) < 64 ? (nk - l0) : 64);
    for (int t = 0; t < cnt; ++t) {
      float pt = sp[t];
#pragma unroll
      for (int u = 0; u < kMaxD / 64; ++u) {
        int c = lane + 64 * u;
        if (c < d) {
          if (OUT_K) acck[u] += pt * load_f<E>(kbase + (l0 + t) * d + c);
          if (OUT_V) accv[u] += pt * load_f<E>(vbase + (l0 + t) * d + c);
        }
      }
    }
  }
#pragma unroll
  for (int u = 0; u < kMaxD / 64; ++u) {
    int c = lane + 64 * u;
    if (c < d) {
      if (OUT_K) store_f<E>(out_k + c, acck[u]);
      if (OUT_V) store_f<E>(out_v + c, BLEND ? 0.5f * (accv[u] + load_f<E>(out_v + c)) : accv[u]);
    }
  }
}

template <typename E, bool HAS_V>
__global__ void __launch_bounds__(64) r_update_generic_kernel(const E* __restrict__ aR, const float* __restrict__ cR,
                                                              const E* __restrict__ k, const E* __restrict__ v,
                                                              E* __restrict__ aL, float* __restrict__ cL,
                                                              E* __restrict__ y, float* __restrict__ lse, int T, int b,
                                                              int d, float row_scale, float cr_min) {
  __shared__ float sq[kMaxD];
  __shared__ float sp[64];
  const int i = blockIdx.x, kf = blockIdx.y, bh = blockIdx.z;
  const long long row = ((long long)bh * T + kf) * b + i;
  const long long frame0 = ((long long)bh * T + kf) * b;
  float c = cR ? cR[row] : 1.f;
  c = fmaxf(c, cr_min);
  attend_row<E, true, HAS_V>(aR + row * d, row_scale / c, k + frame0 * d, HAS_V ? v + frame0 * d : nullptr, b, d,
                             aL + row * d, HAS_V ? y + row * d : nullptr, cL + row, lse ? lse + row : nullptr, sq, sp);
}

template <typename E>
__global__ void __launch_bounds__(64) first_frame_generic_kernel(const E* __restrict__ q, const E* __restrict__ k,
                                                                 const E* __restrict__ v, E* __restrict__ out,
                                                                 float* __restrict__ lse, int T, int b, int d,
                                                                 float scale, const int* __restrict__ rows) {
  __shared__ float sq[kMaxD];
  __shared__ float sp[64];
  int i = blockIdx.x;
  const int bh = blockIdx.y;
  const long long N = (long long)T * b;
  if (rows != nullptr) {
    i = rows[i];
    if (i < 0 || i >= N) return;  // not a row of the head: skipped (uniform over the workgroup)
  }
  const long long head0 = (long long)bh * N;
  attend_row<E, false, true>(q + (head0 + i) * d, scale, k + head0 * d, v + head0 * d, N, d, nullptr,
                             out + (head0 + i) * d, nullptr, lse ? lse + head0 + i : nullptr, sq, sp);
}

// Attention-sink averaging (Sec. 4.4, the variant marked with a double dagger): every token
// attends to the first frame's keys and values; the result is averaged into `out`.
template <typename E>
__global__ void __launch_bounds__(64) sink_average_generic_kernel(const E* __restrict__ q, const E* __restrict__ k,
                                                                  const E* __restrict__ v, E* __restrict__ out,
                                                                  long long N, int b, int d, float scale) {
  __shared__ float sq[kMaxD];
  __shared__ float sp[64];
  const long long row = (long long)blockIdx.y * N + blockIdx.x;
  const long long head0 = (long long)blockIdx.y * N;
  attend_row<E, false, true, true>(q + row * d, scale, k + head0 * d, v + head0 * d, b, d, nullptr, out + row * d,
                                   nullptr, nullptr, sq, sp);
}

__global__ void __launch_bounds__(256) fill_head_prefix_kernel(float* __restrict__ p, float value, long long count,
                                                               long long head_stride) {
  const long long r = (long long)blockIdx.x * 256 + threadIdx.x;
  if (r < count) p[(long long)blockIdx.y * head_stride + r] = value;
}

// One workgroup per (position i, batch*head).  The T x T block L_i lives in LDS.
template <typename E, bool FINAL>
__global__ void __launch_bounds__(256) l_update_generic_kernel(const E* __restrict__ q, const E* __restrict__ aL,
                                                               const float* __restrict__ cL, const E* __restrict__ y,
                                                               E* __restrict__ aR, float* __restrict__ cR,
                                                               E* __restrict__ out, int T, int b, int d,
                                                               float q_scale) {
  extern __shared__ float Lm[];  // [T][T], Lm[j*T + k]
  const int i = blockIdx.x, bh = blockIdx.y;
  const long long head0 = (long long)bh * T * b;
  const int tid = threadIdx.x;
  // logits u[j,k] = q_scale * Q[j,i] . aL[k,i] - cL[k,i]
  for (int e = tid; e < T * T; e += 256) {
    int j = e / T, kf = e % T;
    const E* qr = q + (head0 + (long long)j * b + i) * d;
    const E* ar = aL + (head0 + (long long)kf * b + i) * d;
    float s = 0.f;
    for (int c = 0; c < d; ++c) s += load_f<E>(qr + c) * load_f<E>(ar + c);
    Lm[e] = s * q_scale - cL[head0 + (long long)kf * b + i];
  }
  __syncthreads();
  // row softmax over k
  for (int j = tid; j < T; j += 256) {
    float mx = -INFINITY;
    for (int kf = 0; kf < T; ++kf) mx = fmaxf(mx, Lm[j * T + kf]);
    float s = 0.f;
    for (int kf = 0; kf < T; ++kf) {
      float p = expf(Lm[j * T + kf] - mx);
      Lm[j * T + kf] = p;
      s += p;
    }
    float inv = 1.f / s;
    for (int kf = 0; kf < T; ++kf) Lm[j * T + kf] *= inv;
  }
  __syncthreads();
  if (FINAL) {
    // out[j,i,:] = sum_k L[j,k] y[k,i,:]
    for (int e = tid; e < T * d; e += 256) {
      int j = e / d, c = e % d;
      float s = 0.f;
      for (int kf = 0; kf < T; ++kf) s += Lm[j * T + kf] * load_f<E>(y + (head0 + (long long)kf * b + i) * d + c);
      store_f<E>(out + (head0 + (long long)j * b + i) * d + c, s);
    }
  } else {
    // aR[k,i,:] = sum_j L[j,k] Q[j,i,:] ; cR[k,i] = sum_j L[j,k]
    for (int e = tid; e < T * d; e += 256) {
      int kf = e / d, c = e % d;
      float s = 0.f;
      for (int j = 0; j < T; ++j) s += Lm[j * T + kf] * load_f<E>(q + (head0 + (long long)j * b + i) * d + c);
      store_f<E>(aR + (head0 + (long long)kf * b + i) * d + c, s);
    }
    for (int kf = tid; kf < T; kf += 256) {
      float s = 0.f;
      for (int j = 0; j < T; ++j) s += Lm[j * T + kf];
      cR[head0 + (long long)kf * b + i] = s;
    }
  }
}

// The temporal factor for any number of frames, without a T x T block in LDS: one wave per row of a position's
// block, two passes over the other side's rows (statistics, then sums), the logits recomputed in the second.
//   weight of row l:  w[l] = exp(scale * (x . A[l]) + add_scale * add[l] - ref)
//   FIXED == false:   ref = the row's log-sum-exp (a softmax); out = sum_l w[l] V[l]; lse_out = ref
//   FIXED == true:    ref is given, the weights are final as they are; out = sum_l w[l] V[l], sum_out = sum_l w[l]
// A, add and V are rows of frame-major tensors `stride` rows apart (the position's frames).
template <typename E, bool FIXED>
__device__ void temporal_row(const E* __restrict__ x, float scale, const E* __restrict__ A, const float* __restrict__ add,
                             float add_scale, const E* __restrict__ V, long long stride, int n, int d, float ref_fixed,
                             E* __restrict__ out, float* __restrict__ lse_out, float* __restrict__ sum_out, float* sq,
                             float* sp) {
  const int lane = threadIdx.x;
  for (int c = lane; c < d; c += 64) sq[c] = load_f<E>(x + c);
  __syncthreads();
  auto logit = [&](int l) {
    const E* ar = A + (long long)l * stride * d;
    float z = 0.f;
    for (int c = 0; c < d; ++c) z += sq[c] * load_f<E>(ar + c);
    return z * scale + add_scale * add[(long long)l * stride];
  };
  float ref = ref_fixed;
  if (!FIXED) {
    float m = -INFINITY, S = 0.f;  // online max / sum per lane, merged across the wave
    for (int l = lane; l < n; l += 64) {
      const float z = logit(l);
      const float mn = fmaxf(m, z);
      S = S * expf(m - mn) + expf(z - mn);  // exp(-inf) = 0 on the first key
      m = mn;
    }
    for (int off = 32; off >= 1; off >>= 1) {
      const float mo = __shfl_xor(m, off), So = __shfl_xor(S, off);
      const float mn = fmaxf(m, mo);
      S = (S > 0.f ? S * expf(m - mn) : 0.f) + (So > 0.f ? So * expf(mo - mn) : 0.f);
      m = mn;
    }
    ref = m + logf(S);
    if (lse_out != nullptr && lane == 0) *lse_out = ref;
  }
  if (out == nullptr) return;
  float acc[kMaxD / 64];
#pragma unroll
  for (int u = 0; u < kMaxD / 64; ++u) acc[u] = 0.f;
  float wsum = 0.f;
  for (int l0 = 0; l0 < n; l0 += 64) {
    const int l = l0 + lane;
    const float w = l < n ? expf(logit(l) - ref) : 0.f;
    wsum += w;
    __syncthreads();
    sp[lane] = w;
    __syncthreads();
    const int cnt = n - l0 < 64 ? n - l0 : 64;
    for (int t = 0; t < cnt; ++t) {
      const float wt = sp[t];
      const E* vr = V + (long long)(l0 + t) * stride * d;
#pragma unroll
      for (int u = 0; u < kMaxD / 64; ++u) {
        const int c = lane + 64 * u;
        if (c < d) acc[u] += wt * load_f<E>(vr + c);
      }
    }
  }
#pragma unroll
  for (int u = 0; u < kMaxD / 64; ++u) {
    const int c = lane + 64 * u;
    if (c < d) store_f<E>(out + c, acc[u]);
  }
  if (sum_out != nullptr) {
    for (int off = 32; off >= 1; off >>= 1) wsum += __shfl_xor(wsum, off);
    if (lane == 0) *sum_out = wsum;
  }
}

// MODE 0: last sweep, out[j,i] = sum_k L[j,k] y[k,i]           (Eq. L and the apply-to-V of App. A)
// MODE 1: fitting sweep, first pass: lse[j,i] = log sum_k exp(q_scale Q[j,i] . aL[k,i] - cL[k,i])
// MODE 2: fitting sweep, second pass: aR[k,i] = sum_j L[j,k] Q[j,i], cR[k,i] = sum_j L[j,k]   (Eq. alpha_R / c_R),
//         L[j,k] = exp(q_scale Q[j,i] . aL[k,i] - cL[k,i] - lse[j,i])
template <typename E, int MODE>
__global__ void __launch_bounds__(64) l_update_rows_kernel(const E* __restrict__ q, const E* __restrict__ aL,
                                                           const float* __restrict__ cL, const E* __restrict__ y,
                                                           E* __restrict__ aR, float* __restrict__ cR,
                                                           E* __restrict__ out, float* __restrict__ lse, int T, int b,
                                                           int d, float q_scale) {
  __shared__ float sq[kMaxD];
  __shared__ float sp[64];
  const int i = blockIdx.x, f = blockIdx.y;  // position, frame of the row this wave owns
  const long long col = (long long)blockIdx.z * T * b + i;  // frame 0 of this position
  const long long row = col + (long long)f * b;
  if (MODE == 0)
    temporal_row<E, false>(q + row * d, q_scale, aL + col * d, cL + col, -1.f, y + col * d, b, T, d, 0.f, out + row * d,
                           nullptr, nullptr, sq, sp);
  else if (MODE == 1)
    temporal_row<E, false>(q + row * d, q_scale, aL + col * d, cL + col, -1.f, nullptr, b, T, d, 0.f, nullptr, lse + row,
                           nullptr, sq, sp);
  else
    temporal_row<E, true>(aL + row * d, q_scale, q + col * d, lse + col, -1.f, q + col * d, b, T, d, cL[row], aR + row * d,
                          nullptr, cR + row, sq, sp);
}

// Token-row permutation copy (the stride permutation P of Sec. 3.1 applied to the rows of a [T*b, row] tensor and
// its inverse).  Element = one W-byte word of a destination row; every thread moves UNR of them, all loads issued
// before the first store.  IDX is the integer type of the flat word index (32-bit whenever it fits: the two
// divisions per word are what the copy costs beside its memory traffic).
template <typename W, typename IDX, int UNR>
__global__ void __launch_bounds__(256) permute_tokens_kernel(const W* __restrict__ in, W* __restrict__ out, int T, int b,
                                                             int row_words, int to_pos_major) {
  const IDX N = (IDX)T * (IDX)b;
  const long long head0 = (long long)blockIdx.y * (long long)N * row_words;
  const IDX total = N * (IDX)row_words;
  const IDX stride = (IDX)gridDim.x * 256;
  for (IDX e0 = (IDX)blockIdx.x * 256 + threadIdx.x; e0 < total; e0 += stride * UNR) {
    W val[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const IDX e = e0 + (IDX)u * stride;
      if (e < total) {
        const IDX p = e / (IDX)row_words;   // destination row
        const IDX w = e - p * (IDX)row_words;
        IDX src;
        if (to_pos_major) {                 // out[i*T + j] = in[j*b + i]
          const IDX i = p / (IDX)T, j = p - i * (IDX)T;
          src = j * (IDX)b + i;
        } else {                            // out[j*b + i] = in[i*T + j]
          const IDX j = p / (IDX)b, i = p - j * (IDX)b;
          src = i * (IDX)T + j;
        }
        val[u] = in[head0 + (long long)src * row_words + w];
      }
    }
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const IDX e = e0 + (IDX)u * stride;
      if (e < total) out[head0 + (long long)e] = val[u];
    }
  }
}

// Measurement aid: nothing but v_mfma_f32_32x32x16_bf16, eight per loop trip on four independent
// accumulators, two waves per SIMD, on operand data supplied by the caller.  The sustained rate
// depends on that data: the matrix pipe of this device is power-limited, and operands that
// toggle more bits lower the clock.
__global__ void __launch_bounds__(512) mfma_probe_kernel(const uint4* __restrict__ ops, float* __restrict__ out,
                                                         int iters) {
  bf16x8 a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint4 x = ops[((size_t)blockIdx.x * 512 + threadIdx.x) * 8 + i];
    const uint4 y = ops[((size_t)blockIdx.x * 512 + threadIdx.x) * 8 + 4 + i];
    __builtin_memcpy(&a[i], &x, 16);
    __builtin_memcpy(&b[i], &y, 16);
  }
  f32x16 c[4];
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int i = 0; i < 16; ++i) c[q][i] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 8; ++j)
      c[j & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j & 3], b[(j + (j >> 2)) & 3], c[j & 3], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int q = 0; q < 4; ++q)
#pragma unroll
    for (int i = 0; i < 16; ++i) s += c[q][i];
  out[(size_t)blockIdx.x * 512 + threadIdx.x] = s;
}

}  // namespace

hipError_t launch_mfma_probe(const void* operands, float* out, int blocks, int iters, hipStream_t st) {
  hipLaunchKernelGGL(mfma_probe_kernel, dim3(blocks), dim3(512), 0, st, (const uint4*)operands, out, iters);
  return hipGetLastError();
}

template <typename E>
hipError_t launch_r_update_generic(const E* aR, const float* cR, const E* k, const E* v, E* aL, float* cL, E* y,
                                   float* lse, const Dims& dm, float row_scale, float cr_min, hipStream_t st) {
  dim3 grid(dm.b, dm.T, dm.BH);
  if (v != nullptr)
    hipLaunchKernelGGL((r_update_generic_kernel<E, true>), grid, dim3(64), 0, st, aR, cR, k, v, aL, cL, y, lse, dm.T,
                       dm.b, dm.d, row_scale, cr_min);
  else
    hipLaunchKernelGGL((r_update_generic_kernel<E, false>), grid, dim3(64), 0, st, aR, cR, k, v, aL, cL, y, lse, dm.T,
                       dm.b, dm.d, row_scale, cr_min);
  return hipGetLastError();
}

constexpr int kBlockInLdsMaxT = 200;  // l_update_generic_kernel keeps T * T floats in LDS

bool l_update_generic_needs_lse(const Dims& dm) { return dm.T > kBlockInLdsMaxT; }

template <typename E>
hipError_t launch_l_update_generic(const E* q, const E* aL, const float* cL, const E* y, E* aR, float* cR, E* out,
                                   float* lse_scratch, const Dims& dm, float q_scale, hipStream_t st) {
  if (dm.T > kBlockInLdsMaxT) {
    // more frames than the block-in-LDS kernel holds: one wave per row, logits recomputed
    dim3 grid(dm.b, dm.T, dm.BH);
    if (y != nullptr) {
      hipLaunchKernelGGL((l_update_rows_kernel<E, 0>), grid, dim3(64), 0, st, q, aL, cL, y, aR, cR, out, lse_scratch, dm.T,
                         dm.b, dm.d, q_scale);
      return hipGetLastError();
    }
    if (lse_scratch == nullptr) return hipErrorInvalidValue;
    hipLaunchKernelGGL((l_update_rows_kernel<E, 1>), grid, dim3(64), 0, st, q, aL, cL, y, aR, cR, out, lse_scratch, dm.T,
                       dm.b, dm.d, q_scale);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((l_update_rows_kernel<E, 2>), grid, dim3(64), 0, st, q, aL, cL, y, aR, cR, out, lse_scratch, dm.T,
                       dm.b, dm.d, q_scale);
    return hipGetLastError();
  }
  dim3 grid(dm.b, dm.BH);
  size_t lds = (size_t)dm.T * dm.T * sizeof(float);
  hipError_t e;
  if (y != nullptr) {
    auto kern = l_update_generic_kernel<E, true>;
    if (lds > 48 * 1024) {
      e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kern, grid, dim3(256), lds, st, q, aL, cL, y, aR, cR, out, dm.T, dm.b, dm.d, q_scale);
  } else {
    auto kern = l_update_generic_kernel<E, false>;
    if (lds > 48 * 1024) {
      e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kern, grid, dim3(256), lds, st, q, aL, cL, y, aR, cR, out, dm.T, dm.b, dm.d, q_scale);
  }
  return hipGetLastError();
}

template <typename E>
hipError_t launch_first_frame_generic(const E* q, const E* k, const E* v, E* out, float* lse, const Dims& dm,
                                      int nrows, const int* rows, hipStream_t st) {
  dim3 grid(nrows, dm.BH);  // q, out, lse point at the first row to recompute of head 0 (row 0 with a row list)
  hipLaunchKernelGGL((first_frame_generic_kernel<E>), grid, dim3(64), 0, st, q, k, v, out, lse, dm.T, dm.b, dm.d,
                     1.0f / sqrtf((float)dm.d), rows);
  return hipGetLastError();
}

template <typename E>
hipError_t launch_sink_average_generic(const E* q, const E* k, const E* v, E* out, const Dims& dm, hipStream_t st) {
  if (dm.N > 0x7fffffffLL) return hipErrorInvalidValue;
  dim3 grid((unsigned)dm.N, dm.BH);
  hipLaunchKernelGGL((sink_average_generic_kernel<E>), grid, dim3(64), 0, st, q, k, v, out, dm.N, dm.b, dm.d,
                     1.0f / sqrtf((float)dm.d));
  return hipGetLastError();
}

hipError_t launch_fill_head_prefix(float* p, float value, long long count, long long head_stride, int nheads,
                                   hipStream_t st) {
  if (count <= 0 || nheads <= 0) return hipSuccess;
  const long long blocks = (count + 255) / 256;
  if (blocks > 0x7fffffffLL || nheads > 65535) return hipErrorInvalidValue;
  hipLaunchKernelGGL(fill_head_prefix_kernel, dim3((unsigned)blocks, nheads), dim3(256), 0, st, p, value, count,
                     head_stride);
  return hipGetLastError();
}

template <typename W>
hipError_t launch_permute_words(const void* in, void* out, const Dims& dm, int row_words, int to_pos_major,
                                hipStream_t st) {
  constexpr int UNR = 4;
  const long long total = dm.N * row_words;
  long long blocks = (total + 256 * UNR - 1) / (256 * UNR);
  if (blocks > 16384) blocks = 16384;
  dim3 grid((unsigned)blocks, dm.BH);
  // the flat index runs up to total + UNR * grid * 256 before its bound is tested
  if (total + (long long)UNR * 16384 * 256 < 0x7fffffffLL)
    hipLaunchKernelGGL((permute_tokens_kernel<W, unsigned, UNR>), grid, dim3(256), 0, st, (const W*)in, (W*)out, dm.T,
                       dm.b, row_words, to_pos_major);
  else
    hipLaunchKernelGGL((permute_tokens_kernel<W, long long, UNR>), grid, dim3(256), 0, st, (const W*)in, (W*)out, dm.T,
                       dm.b, row_words, to_pos_major);
  return hipGetLastError();
}

// in and out are rows of row_bytes (a multiple of 4); 16-byte words when the rows and both pointers allow it
hipError_t launch_permute_tokens(const void* in, void* out, const Dims& dm, int row_bytes, int to_pos_major,
                                 hipStream_t st) {
  const bool wide = row_bytes % 16 == 0 && ((uintptr_t)in | (uintptr_t)out) % 16 == 0;
  if (wide) return launch_permute_words<uint4>(in, out, dm, row_bytes / 16, to_pos_major, st);
  return launch_permute_words<uint32_t>(in, out, dm, row_bytes / 4, to_pos_major, st);
}

template hipError_t launch_r_update_generic<float>(const float*, const float*, const float*, const float*, float*,
                                                   float*, float*, float*, const Dims&, float, float, hipStream_t);
template hipError_t launch_r_update_generic<bf16_t>(const bf16_t*, const float*, const bf16_t*, const bf16_t*, bf16_t*,
                                                    float*, bf16_t*, float*, const Dims&, float, float, hipStream_t);
template hipError_t launch_l_update_generic<float>(const float*, const float*, const float*, const float*, float*,
                                                   float*, float*, float*, const Dims&, float, hipStream_t);
template hipError_t launch_l_update_generic<bf16_t>(const bf16_t*, const bf16_t*, const float*, const bf16_t*, bf16_t*,
                                                    float*, bf16_t*, float*, const Dims&, float, hipStream_t);
template hipError_t launch_first_frame_generic<float>(const float*, const float*, const float*, float*, float*,
                                                      const Dims&, int, const int*, hipStream_t);
template hipError_t launch_first_frame_generic<bf16_t>(const bf16_t*, const bf16_t*, const bf16_t*, bf16_t*, float*,
                                                       const Dims&, int, const int*, hipStream_t);
template hipError_t launch_sink_average_generic<float>(const float*, const float*, const float*, float*, const Dims&,
                                                       hipStream_t);
template hipError_t launch_sink_average_generic<bf16_t>(const bf16_t*, const bf16_t*, const bf16_t*, bf16_t*,
                                                        const Dims&, hipStream_t);

}  // namespace vm

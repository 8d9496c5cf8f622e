/*
 * vmonarch.h -- C ABI of the MI355X (gfx950) spatio-temporal Monarch attention library.
 *
 * The method is VMonarch's attention (paper Sec. 3): N = T*Hs*Ws video tokens are viewed
 * as m = T frames of b = Hs*Ws spatial positions, token n = j*b + i (frame j, position i;
 * the reshape(m, b, d) of App. A).  softmax(Q K^T / sqrt(d)) is replaced by a Monarch
 * matrix M[(j,i),(k,l)] = L[i][j,k] * R[k][i,l] (Sec. 3.1) whose factors are fitted by
 * `iters` sweeps of the closed-form alternating updates (Eqs. R, alpha_R/c_R, L,
 * alpha_L/c_L; App. A) and applied to V; optionally the rows of frame 0 are recomputed
 * with exact attention (Sec. 3.3).
 *
 * Conventions shared by every entry point
 *   - All tensor pointers are DEVICE pointers unless a parameter says "host".
 *   - Token tensors (q, k, v, out, aR, aL, y) are contiguous [B][heads][T][b][d]
 *     (= [B][heads][N][d]); per-token scalars (cR, cL) are float32 [B][heads][T][b].
 *     Note aL and cL are stored frame-major like everything else; "position-major"
 *     (App. A's transposes) is only the order in which the L-update walks them.
 *   - Entry points without suffix take bfloat16 token tensors; `_f32` twins take float32.
 *     Scalars c_R, c_L are float32 in both.  Accumulation is float32 everywhere.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Calls only
 *     enqueue work; they never synchronise the host, with one exception: when no workspace
 *     has been given and the library's own arena has to grow (see vmonarch_set_workspace).
 *   - The library never frees or retains caller memory.  Outputs must not alias inputs.
 *   - Return value: 0 on success, a negative VMONARCH_ERR_* otherwise; nothing is
 *     launched when validation fails.  vmonarch_last_error() describes the last failure
 *     of the calling thread.  No exception crosses this boundary.
 *   - Concurrency.  vmonarch_attention[_f32], vmonarch_recompute_rows / _tokens,
 *     vmonarch_first_frame_attention* and vmonarch_entropy_attention_bwd* keep intermediates in
 *     ONE workspace per process (the buffer of vmonarch_set_workspace, else the library's arena of
 *     the current device): at most one such call may be in flight per device, on whatever stream,
 *     unless every concurrent call brings its own buffer (vmonarch_attention_ex with
 *     options.workspace).  The vmonarch_set_* settings are process-wide and not synchronised: they
 *     are read when a call is made (a HIP graph captured from a call keeps what was set then);
 *     vmonarch_attention_ex carries them per call instead.
 *   - Sizes.  d <= 256, B*heads <= 65535, T <= 65535, N < 2^31 for every entry point; no other
 *     shape is refused.  bf16 with d == 128 or d == 64 runs on the MFMA kernels (the temporal factor
 *     on a kernel of its own up to T = 128 and through the blocked-softmax kernel up to T = 8128);
 *     other shapes and every `_f32` entry point run on slower plain-ALU kernels with the same results.
 *   - (T, Hs, Ws) only enter as m = T blocks of b = Hs*Ws tokens: a general Monarch split
 *     (m, b) of a sequence that is no video is T = m, Hs = 1, Ws = b.
 */
#ifndef VMONARCH_H_
#define VMONARCH_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define VMONARCH_OK 0
#define VMONARCH_ERR_INVALID_ARG (-1) /* null pointer, non-positive size, iters < 1 */
#define VMONARCH_ERR_UNSUPPORTED (-2) /* d > 256, or a size whose index does not fit (see "Sizes" above) */
#define VMONARCH_ERR_WORKSPACE (-3)   /* caller workspace too small / allocation failed */
#define VMONARCH_ERR_HIP (-4)         /* a HIP runtime call failed */

/* How the R-update obtains c_L = sum_l R log R (Eq. alpha_L/c_L). */
#define VMONARCH_ENTROPY_ONLINE 0   /* Alg. 1 / App. B: third running statistic h beside (m, l) */
#define VMONARCH_ENTROPY_IDENTITY 1 /* c_L = (aR . alpha_L) * scale - logsumexp, from the outputs */

/* The `recompute` argument of vmonarch_attention[_f32]. */
#define VMONARCH_RECOMPUTE_NONE 0
#define VMONARCH_RECOMPUTE_FIRST_FRAME 1 /* Sec. 3.3 */
#define VMONARCH_SINK_AVERAGE 2          /* Sec. 4.4 ablation: see vmonarch_sink_average */

/* Manual control of c_R / c_L (App. "Manual Control of Monarch Parameters"). */
#define VMONARCH_CONTROL_NONE 0
#define VMONARCH_CONTROL_FIRST_FRAME 1 /* key frame k = 0 only */
#define VMONARCH_CONTROL_ALL_FRAMES 2

/* Library version: major*10000 + minor*100 + patch. */
int vmonarch_version(void);

/* Text of the calling thread's last error ("" if none).  Pointer stays valid until the
 * thread's next failing call. */
const char* vmonarch_last_error(void);

/* Lower bound applied to c_R where it divides the logits (Sec. 4.1 "clamp c_R to 0.1").
 * Default 0.1; 0 disables.  Process-wide; affects vmonarch_attention[_f32] only. */
int vmonarch_set_cr_min(float cr_min);
float vmonarch_get_cr_min(void);

/* bf16 MFMA R-update with values (the last sweep; vmonarch_r_update[_lse] with v != NULL) and online
 * entropy, when it runs on the kernels with two waves per SIMD (flash variant 0, and variant 2 for
 * frames of at most 128 tokens): 1 (default) forms alpha_L, c_L and y = R V from one evaluation of
 * the logits and the softmax, two waves sharing a query tile; 0 runs one pass for alpha_L / c_L and
 * a second for y.  The kernel with one wave per SIMD (see vmonarch_set_flash_variant) always takes
 * one pass.  Same results up to rounding order.  Process-wide. */
int vmonarch_set_fused_apply(int enable);
int vmonarch_get_fused_apply(void);

/* Ablation of App. "Manual Control of Monarch Parameters", applied inside
 * vmonarch_attention[_f32] in every sweep: right after the L-update c_R is overwritten with 1,
 * right after the R-update c_L is overwritten with cl_value, each for no frame, key frame 0, or
 * all frames (VMONARCH_CONTROL_*).  cl_value = NaN selects -log(Hs*Ws): the paper's log M, the
 * entropy of a uniform row of the b x b factor, with this library's sign c_L = sum R log R.
 * Defaults: none, none, NaN.  Process-wide.  The getter's pointers may be NULL. */
int vmonarch_set_manual_control(int cr_control, int cl_control, float cl_value);
int vmonarch_get_manual_control(int* cr_control, int* cl_control, float* cl_value);

/* Which bf16 MFMA kernel runs an R-update: 0 the kernels with two waves per SIMD and one 32-query
 * tile per wave; 1 the kernel with one wave per SIMD and two query tiles per wave, whose
 * accumulators live in accumulation registers (measured a few per cent faster for the update with
 * values and, at d = 64, without; slower without values at d = 128); 2 (default) each update on
 * the kernel measured faster for it: that of 1 for the update with values (frames of more than
 * 128 tokens) and for d = 64, those of 0 otherwise.  Exact attention of a contiguous row range
 * (first frame, vmonarch_recompute_rows) runs on the kernel of 1 unless the variant is 0; a row
 * list (vmonarch_recompute_tokens) and the sink averaging always run on the kernels of 0.  Same results up to rounding order.  Process-wide. */
int vmonarch_set_flash_variant(int variant);
int vmonarch_get_flash_variant(void);

/* Selects VMONARCH_ENTROPY_* for the bf16 MFMA R-update (default ONLINE).  Process-wide. */
int vmonarch_set_entropy_mode(int mode);
int vmonarch_get_entropy_mode(void);

/* Bytes of device scratch vmonarch_attention[_f32] needs for these sizes
 * (elem_bytes = 2 for bf16, 4 for f32).  0 on invalid sizes. */
size_t vmonarch_workspace_bytes(int B, int heads, int T, int Hs, int Ws, int d, int iters,
                                int recompute, int elem_bytes);

/* Hands the library a caller-owned device buffer to use as scratch (256-byte aligned) by every later
 * call of the process.  Passing NULL/0 returns to the library-owned arena (one per device), which
 * grows on demand: hipDeviceSynchronize + hipFree + hipMalloc, once per size increase, released by
 * vmonarch_shutdown().  A call that would have to grow the arena while its stream is being captured
 * into a HIP graph returns VMONARCH_ERR_WORKSPACE instead. */
int vmonarch_set_workspace(void* dev_ptr, size_t bytes);
int vmonarch_shutdown(void);

/*
 * Whole path (Eq. 5: O = MonarchAttention(Q, K, V; m = T, b = Hs*Ws, t = iters), then
 * Sec. 3.3 if recompute == VMONARCH_RECOMPUTE_FIRST_FRAME, or the sink averaging of Sec. 4.4 if
 * recompute == VMONARCH_SINK_AVERAGE; other values are rejected).  q, k, v, out:
 * [B][heads][N][d].  1/sqrt(d) multiplies Q everywhere Q enters (fit and recomputation alike).
 */
int vmonarch_attention(const void* q, const void* k, const void* v, void* out, int B, int heads,
                       int T, int Hs, int Ws, int d, int iters, int recompute, void* stream);
int vmonarch_attention_f32(const void* q, const void* k, const void* v, void* out, int B, int heads,
                           int T, int Hs, int Ws, int d, int iters, int recompute, void* stream);

/*
 * The same call with every setting and the workspace carried by the call instead of the process:
 * concurrent calls (different streams, different threads) with different settings or different
 * workspaces do not interfere.  vmonarch_options_init fills in the library's defaults (c_R bound
 * 0.1 of Sec. 4.1, online entropy of Alg. 1, one-pass last R-update, default kernels, no manual
 * control, cl_value = NaN for -log(Hs*Ws), no workspace); change fields afterwards.  The process-wide
 * setters do not affect these calls.  workspace == NULL uses the process-wide workspace / arena.
 */
typedef struct vmonarch_options {
  uint32_t struct_bytes;  /* sizeof(vmonarch_options), set by vmonarch_options_init */
  float cr_min;           /* see vmonarch_set_cr_min */
  int entropy_mode;       /* VMONARCH_ENTROPY_* */
  int fused_apply;        /* see vmonarch_set_fused_apply */
  int flash_variant;      /* see vmonarch_set_flash_variant */
  int cr_control;         /* VMONARCH_CONTROL_*, see vmonarch_set_manual_control */
  int cl_control;
  float cl_value;
  void* workspace;        /* device, 256-byte aligned, at least vmonarch_workspace_bytes(...) bytes, or NULL */
  size_t workspace_bytes;
} vmonarch_options;
int vmonarch_options_init(vmonarch_options* options);
int vmonarch_attention_ex(const void* q, const void* k, const void* v, void* out, int B, int heads, int T, int Hs,
                          int Ws, int d, int iters, int recompute, const vmonarch_options* options, void* stream);
int vmonarch_attention_ex_f32(const void* q, const void* k, const void* v, void* out, int B, int heads, int T,
                              int Hs, int Ws, int d, int iters, int recompute, const vmonarch_options* options,
                              void* stream);

/*
 * R-update, the intra-frame (spatial) factor (Eq. R with Eq. alpha_L/c_L; App. A R_update;
 * computed as one blocked softmax pass with running max, sum and entropy, Alg. 1).
 * For every frame k and query position i:
 *     z[l]      = row_scale * (aR[k,i,:] . K[k,l,:]) / max(cR[k,i], cr_min)
 *     R[k,i,:]  = softmax_l z                      (never stored)
 *     aL[k,i,:] = sum_l R[k,i,l] K[k,l,:]          cL[k,i] = sum_l R[k,i,l] log R[k,i,l]
 *     y[k,i,:]  = sum_l R[k,i,l] V[k,l,:]          (only if v and y_out are non-NULL)
 * cR == NULL means all ones (the first sweep, where aR is Q itself).
 */
int vmonarch_r_update(const void* aR, const float* cR, const void* k, const void* v, void* aL_out,
                      float* cL_out, void* y_out, int B, int heads, int T, int Hs, int Ws, int d,
                      float row_scale, float cr_min, void* stream);
int vmonarch_r_update_f32(const void* aR, const float* cR, const void* k, const void* v,
                          void* aL_out, float* cL_out, void* y_out, int B, int heads, int T, int Hs,
                          int Ws, int d, float row_scale, float cr_min, void* stream);

/*
 * The same R-update, which also returns the log-sum-exp of every query row's logits, the
 * per-row statistic Alg. 1 hands to the backward pass (Alg. 2) beside the entropy:
 *     lse_out[k,i] = log sum_l exp z[l]        (natural log; float32 [B][heads][T][b])
 * The row entropy of Alg. 1 is H = -cL_out.  On the bf16 MFMA path the sum inside the
 * logarithm is taken over the bf16-rounded probabilities (absolute error about 1e-3).
 * lse_out must not be NULL.
 */
int vmonarch_r_update_lse(const void* aR, const float* cR, const void* k, const void* v, void* aL_out,
                          float* cL_out, void* y_out, float* lse_out, int B, int heads, int T, int Hs,
                          int Ws, int d, float row_scale, float cr_min, void* stream);
int vmonarch_r_update_lse_f32(const void* aR, const float* cR, const void* k, const void* v,
                              void* aL_out, float* cL_out, void* y_out, float* lse_out, int B, int heads,
                              int T, int Hs, int Ws, int d, float row_scale, float cr_min, void* stream);

/*
 * L-update, the inter-frame (temporal) factor (Eq. L with Eq. alpha_R/c_R; App. A
 * L_update), walking the frame-major tensors with stride b*d (the permutation P of
 * Sec. 3.1 is applied as addressing, never as a copy).  For every position i:
 *     L[i][j,:]  = softmax_k ( q_scale * (Q[j,i,:] . aL[k,i,:]) - cL[k,i] )   (never stored)
 *   if y == NULL (fitting sweep):
 *     aR_out[k,i,:] = sum_j L[i][j,k] Q[j,i,:]  (unscaled Q)     cR_out[k,i] = sum_j L[i][j,k]
 *   else (last sweep, the apply-to-V of App. A):
 *     out[j,i,:] = sum_k L[i][j,k] y[k,i,:]
 * Exactly one of {aR_out and cR_out} / {y and out} must be given.
 */
int vmonarch_l_update(const void* q, const void* aL, const float* cL, const void* y, void* aR_out,
                      float* cR_out, void* out, int B, int heads, int T, int Hs, int Ws, int d,
                      float q_scale, void* stream);
int vmonarch_l_update_f32(const void* q, const void* aL, const float* cL, const void* y,
                          void* aR_out, float* cR_out, void* out, int B, int heads, int T, int Hs,
                          int Ws, int d, float q_scale, void* stream);

/*
 * First-frame recomputation (Sec. 3.3): out[0:b] = softmax(Q[0:b] K^T / sqrt(d)) V over all
 * N keys, per (batch, head).  Only rows 0..b-1 of each head of `out` are written.
 * The bf16 MFMA path splits the keys over several workgroups and merges the partial
 * results; it uses the workspace (see vmonarch_workspace_bytes with recompute != 0).
 */
int vmonarch_first_frame_attention(const void* q, const void* k, const void* v, void* out, int B,
                                   int heads, int T, int Hs, int Ws, int d, void* stream);
int vmonarch_first_frame_attention_f32(const void* q, const void* k, const void* v, void* out,
                                       int B, int heads, int T, int Hs, int Ws, int d, void* stream);

/*
 * The same recomputation, which also returns lse_out[0:b] = log sum_n exp(Q[i] . K[n] / sqrt(d))
 * over all N keys (natural log).  lse_out: float32 [B][heads][T][b] like every per-token scalar;
 * only the entries of frame 0 are written.  lse_out must not be NULL.
 */
int vmonarch_first_frame_attention_lse(const void* q, const void* k, const void* v, void* out,
                                       float* lse_out, int B, int heads, int T, int Hs, int Ws, int d,
                                       void* stream);
int vmonarch_first_frame_attention_lse_f32(const void* q, const void* k, const void* v, void* out,
                                           float* lse_out, int B, int heads, int T, int Hs, int Ws,
                                           int d, void* stream);

/*
 * Recomputation of an arbitrary contiguous range of tokens (Sec. 3.3 names the first frame;
 * the strategy applies to any tokens): out[row_begin : row_begin + row_count] of every head =
 * softmax(Q[rows] K^T / sqrt(d)) V over all N keys.  Only those rows of `out` are written.
 * 0 <= row_begin, 1 <= row_count, row_begin + row_count <= N.  The first-frame call is
 * row_begin = 0, row_count = Hs*Ws.
 */
int vmonarch_recompute_rows(const void* q, const void* k, const void* v, void* out, int B, int heads, int T,
                            int Hs, int Ws, int d, long long row_begin, long long row_count, void* stream);
int vmonarch_recompute_rows_f32(const void* q, const void* k, const void* v, void* out, int B, int heads,
                                int T, int Hs, int Ws, int d, long long row_begin, long long row_count,
                                void* stream);

/*
 * Recomputation of an arbitrary set of tokens (the paper's closing remark: recomputation of
 * specific tokens in general, not only of the first frame): for every r < n_rows and every head,
 *     out[rows_dev[r]] = softmax(Q[rows_dev[r]] K^T / sqrt(d)) V     over all N keys,
 * the listed query rows gathered when they are loaded and the results scattered when they are
 * stored (no staging copy).  rows_dev: DEVICE int32[n_rows], row numbers within a head, the same
 * list for every (batch, head); any order; n_rows >= 1.  The host cannot see the list: an entry
 * outside [0, N) is skipped on the device (nothing is read or written for it); a row listed twice is
 * computed twice and stored twice with the same value.  All other rows of `out` are left as they are.
 * Uses the workspace like vmonarch_recompute_rows.
 */
int vmonarch_recompute_tokens(const void* q, const void* k, const void* v, void* out, const int32_t* rows_dev,
                              long long n_rows, int B, int heads, int T, int Hs, int Ws, int d, void* stream);
int vmonarch_recompute_tokens_f32(const void* q, const void* k, const void* v, void* out, const int32_t* rows_dev,
                                  long long n_rows, int B, int heads, int T, int Hs, int Ws, int d, void* stream);

/*
 * vmonarch_recompute_rows (bf16) for callers that cannot allocate device memory: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same
 * kernels, same results; the partial results of the key ranges go to a buffer built into the
 * library (64 MiB per device, held until the process ends) instead of the workspace, and the
 * call makes no hipMalloc / hipFree and uses neither the arena nor vmonarch_set_workspace.
 * B*heads*row_count*ranges*(4 d + 4) bytes must fit the buffer (the range count is the one
 * vmonarch_recompute_rows would choose); otherwise VMONARCH_ERR_WORKSPACE is returned and nothing
 * is launched.  All calls on one device share the buffer: calls that overlap in time on one
 * device (different streams or threads) race; calls on one stream do not.  The first call on a
 * device looks the buffer's address up (hipGetSymbolAddress): make one call before capturing.
 */
int vmonarch_recompute_rows_noalloc(const void* q, const void* k, const void* v, void* out, int B, int heads, int T,
                                    int Hs, int Ws, int d, long long row_begin, long long row_count, void* stream);

/*
 * Attention-sink averaging, the alternative to recomputation that Sec. 4.4 compares against:
 * out <- (out + softmax(Q K_F1^T / sqrt(d)) V_F1) / 2 in place, for all N tokens of every head,
 * K_F1 / V_F1 the first frame's Hs*Ws keys and values.  `out` holds MonarchAttention(Q, K, V) on
 * entry (vmonarch_attention with recompute = VMONARCH_SINK_AVERAGE does both).
 */
int vmonarch_sink_average(const void* q, const void* k, const void* v, void* out, int B, int heads, int T,
                          int Hs, int Ws, int d, void* stream);
int vmonarch_sink_average_f32(const void* q, const void* k, const void* v, void* out, int B, int heads, int T,
                              int Hs, int Ws, int d, void* stream);

/*
 * Permutation P_(b,N) of Sec. 3.1 (its footnote: reshape to m x b, transpose, flatten).
 * perm, inv: HOST int32[N]; position-major slot p = i*T + j holds token perm[p] = j*b + i,
 * and inv[j*b + i] = i*T + j.
 */
int vmonarch_index_maps(int T, int Hs, int Ws, int32_t* perm_host, int32_t* inv_host);

/*
 * Applies that permutation to token rows as a stand-alone copy (the fused path never
 * calls it; it exists to check the index maps on the device and to measure the HBM rate
 * of the strided walk).  in, out: [B][heads][N][row_bytes]; to_position_major != 0 writes
 * out[i*T + j] = in[j*b + i], otherwise out[j*b + i] = in[i*T + j].  row_bytes % 4 == 0.
 */
int vmonarch_permute_tokens(const void* in, void* out, int B, int heads, int T, int Hs, int Ws,
                            int row_bytes, int to_position_major, void* stream);

/*
 * Backward of one blocked-softmax pass with entropy (App. "Backward pass of
 * Flash-Entropy-Attention", Alg. 2), for the same batch of per-frame problems as
 * vmonarch_r_update.  With, for every frame k and query position i,
 *     z[l] = row_scale * (q[k,i,:] . K[k,l,:]) / max(cR[k,i], cr_min)    (cR == NULL: all ones)
 *     P = softmax_l z,   O[k,i,:] = sum_l P[l] V[k,l,:],   H[k,i] = -sum_l P[l] log P[l]
 * it returns the gradients of  <dO, O> + <dH, H>  with respect to q, K and V:
 *     dS[i,l]  = P (dO[i].V[l] - D[i]) - dH[i] P (z[l] - lse[i] + H[i]),  D[i] = dO[i] . O[i]
 *     dq[k,i,:] = scale_i sum_l dS[i,l] K[k,l,:]    (scale_i = row_scale / max(cR, cr_min))
 *     dk[k,l,:] = sum_i scale_i dS[i,l] q[k,i,:]    dv[k,l,:] = sum_i P[i,l] dO[k,i,:]
 * q, k, v, o, dO, dq_out, dk_out, dv_out: [B][heads][T][b][d]; lse, H, dH: float32 [B][heads][T][b].
 * o, lse and H are the forward results (vmonarch_r_update_lse returns lse and cL = -H; its aL is
 * O for V := K, its y is O for V).  dH == NULL means no gradient through the entropy, which is
 * how the paper trains.  No gradient with respect to cR is returned.  Uses the workspace
 * (four floats per query row).  bf16 with d == 64 or 128 runs on MFMA kernels (three passes: dq,
 * dv, dk), everything else on plain-ALU kernels; results are bit-reproducible: nothing is
 * accumulated across workgroups.
 */
int vmonarch_entropy_attention_bwd(const void* q, const float* cR, const void* k, const void* v, const void* o,
                                   const void* dO, const float* lse, const float* H, const float* dH,
                                   void* dq_out, void* dk_out, void* dv_out, int B, int heads, int T, int Hs,
                                   int Ws, int d, float row_scale, float cr_min, void* stream);
int vmonarch_entropy_attention_bwd_f32(const void* q, const float* cR, const void* k, const void* v,
                                       const void* o, const void* dO, const float* lse, const float* H,
                                       const float* dH, void* dq_out, void* dk_out, void* dv_out, int B,
                                       int heads, int T, int Hs, int Ws, int d, float row_scale, float cr_min,
                                       void* stream);

#ifdef __cplusplus
}
#endif
#endif /* VMONARCH_H_ */

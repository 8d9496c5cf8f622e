// C ABI of libvmonarch: argument validation, workspace management and the launch sequence of
// the whole path (App. A monarch_attention loop + Sec. 3.3 recomputation).  See
// include/vmonarch.h for the contract of every entry point.
#include "../../include/vmonarch.h"
#include "../../include/vmonarch_bench.h"

#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <mutex>

#include <cmath>

#include "common.h"

using namespace vm;

// Device memory of the entry point that allocates nothing (vmonarch_recompute_rows_noalloc): the
// partial results of its key ranges.  Every device the library runs on holds one copy until the
// process ends.  Host code never uses this name as an address: it asks the runtime for the
// device's copy once (noalloc_scratch below) and passes that pointer on.
constexpr size_t kNoAllocScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kNoAllocScratchBytes];

namespace {

thread_local char g_err[512] = "";
float g_cr_min = 0.1f;
int g_fused_apply = 1;
int g_cr_control = VMONARCH_CONTROL_NONE;
int g_cl_control = VMONARCH_CONTROL_NONE;
float g_cl_value = NAN;  // NaN: -log(b), the c_L of a uniform row of R
int g_entropy_mode = VMONARCH_ENTROPY_ONLINE;
// which bf16 MFMA kernel runs an R-update: 0 the two-waves-per-SIMD kernels (flash.hip, flash_kv.hip; the faster
// ones as measured on MI355X), 1 the one-wave-per-SIMD kernel with two query tiles per wave (flash2.hip)
int g_flash_variant = 2;

std::mutex g_ws_mutex;
void* g_user_ws = nullptr;
size_t g_user_ws_bytes = 0;
void* g_arena[64] = {nullptr};  // per device, library-owned
size_t g_arena_bytes[64] = {0};

// Optional per-phase timing of vmonarch_attention (benchmarks only): events recorded on the
// caller's stream between the kernels of one call.
constexpr int kMaxPhases = 32;
bool g_timing = false;
hipEvent_t g_ev[kMaxPhases + 1];
bool g_ev_created = false;
int g_n_phases = 0;
char g_phase_name[kMaxPhases][32];

void phase_mark(hipStream_t st, const char* name_of_phase_that_starts) {
  if (!g_timing) return;
  if (!g_ev_created) {
    for (int i = 0; i <= kMaxPhases; ++i) (void)hipEventCreate(&g_ev[i]);
    g_ev_created = true;
  }
  if (name_of_phase_that_starts == nullptr) {  // closing mark
    (void)hipEventRecord(g_ev[g_n_phases], st);
    return;
  }
  if (g_n_phases >= kMaxPhases) return;
  (void)hipEventRecord(g_ev[g_n_phases], st);
  snprintf(g_phase_name[g_n_phases], sizeof(g_phase_name[0]), "%s", name_of_phase_that_starts);
  ++g_n_phases;
}

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

int hip_fail(hipError_t e, const char* what) {
  return fail(VMONARCH_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
}

int make_dims(int B, int heads, int T, int Hs, int Ws, int d, Dims* dm) {
  if (B <= 0 || heads <= 0 || T <= 0 || Hs <= 0 || Ws <= 0 || d <= 0)
    return fail(VMONARCH_ERR_INVALID_ARG, "sizes must be positive (B=%d heads=%d T=%d Hs=%d Ws=%d d=%d)", B, heads, T,
                Hs, Ws, d);
  if (d > 256) return fail(VMONARCH_ERR_UNSUPPORTED, "d=%d exceeds 256", d);
  long long bh = (long long)B * heads;
  long long b = (long long)Hs * Ws;
  long long N = b * T;
  if (bh > 65535) return fail(VMONARCH_ERR_UNSUPPORTED, "B*heads=%lld exceeds 65535", bh);
  if (T > 65535) return fail(VMONARCH_ERR_UNSUPPORTED, "T=%d exceeds 65535", T);
  if (N > 0x7fffffffLL) return fail(VMONARCH_ERR_UNSUPPORTED, "N=%lld tokens per head exceeds 2^31-1", N);
  dm->BH = (int)bh;
  dm->T = T;
  dm->b = (int)b;
  dm->d = d;
  dm->N = N;
  return VMONARCH_OK;
}

size_t align_up(size_t x) { return (x + 255) & ~(size_t)255; }

// Address of the current device's copy of `scratch`, looked up on the first call per device.
std::mutex g_scratch_mutex;
void* g_scratch_ptr[64] = {nullptr};
void* noalloc_scratch(int* err) {
  *err = VMONARCH_OK;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= 64) {
    *err = fail(VMONARCH_ERR_HIP, "hipGetDevice failed");
    return nullptr;
  }
  std::lock_guard<std::mutex> lk(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || p == nullptr) {
      *err = hip_fail(e, "hipGetSymbolAddress(scratch)");
      return nullptr;
    }
    g_scratch_ptr[dev] = p;
  }
  return g_scratch_ptr[dev];
}

struct WsLayout {
  size_t aL, aR, y, cL, cR, tl, ff, total;
};

// bf16 temporal factor with more frames than the one-workgroup-per-position kernel holds: the blocked-softmax
// kernel takes it in two passes and keeps the rows' log-sum-exp in between
bool temporal_needs_lse(const Dims& dm, int elem_bytes) {
  if (elem_bytes == 2 && lpass_supported(dm)) return false;
  if (elem_bytes == 2 && temporal_flash_supported(dm)) return true;
  return l_update_generic_needs_lse(dm);  // plain-ALU kernels
}

WsLayout ws_layout(const Dims& dm, int iters, int recompute, int elem_bytes) {
  WsLayout w;
  size_t tok = align_up((size_t)dm.BH * dm.N * dm.d * elem_bytes);
  size_t sc = align_up((size_t)dm.BH * dm.N * sizeof(float));
  size_t off = 0;
  w.aL = off; off += tok;
  w.y = off; off += tok;
  w.cL = off; off += sc;
  w.aR = off; if (iters > 1) off += tok;
  w.cR = off; if (iters > 1) off += sc;
  w.tl = off; if (iters > 1 && temporal_needs_lse(dm, elem_bytes)) off += sc;
  w.ff = off;
  if (recompute == VMONARCH_RECOMPUTE_FIRST_FRAME && elem_bytes == 2 && flash_supported(dm)) off += align_up(first_frame_flash_scratch_bytes(dm, dm.b));
  w.total = off;
  return w;
}

// Returns scratch of at least `bytes` on the current device, or nullptr with g_err set: the call's own buffer
// if it brought one, else the process-wide caller workspace, else the library's grow-only arena.  Growing the
// arena synchronises the device and allocates, which a stream that is being captured into a graph forbids:
// then the call fails instead.
void* get_workspace(size_t bytes, int* err, void* call_ws = nullptr, size_t call_ws_bytes = 0, hipStream_t st = nullptr) {
  *err = VMONARCH_OK;
  if (call_ws != nullptr) {
    if (call_ws_bytes < bytes) {
      *err = fail(VMONARCH_ERR_WORKSPACE, "the call's workspace has %zu bytes, %zu needed", call_ws_bytes, bytes);
      return nullptr;
    }
    return call_ws;
  }
  std::lock_guard<std::mutex> lk(g_ws_mutex);
  if (g_user_ws != nullptr) {
    if (g_user_ws_bytes < bytes) {
      *err = fail(VMONARCH_ERR_WORKSPACE, "caller workspace has %zu bytes, %zu needed", g_user_ws_bytes, bytes);
      return nullptr;
    }
    return g_user_ws;
  }
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= 64) {
    *err = fail(VMONARCH_ERR_HIP, "hipGetDevice failed");
    return nullptr;
  }
  if (g_arena_bytes[dev] < bytes) {
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &cap) == hipSuccess && cap != hipStreamCaptureStatusNone) {
      *err = fail(VMONARCH_ERR_WORKSPACE,
                  "the library's arena would have to grow to %zu bytes while the stream is being captured: give the "
                  "call a workspace (vmonarch_set_workspace or vmonarch_options) or run it once before capturing",
                  bytes);
      return nullptr;
    }
    if (g_arena[dev] != nullptr) {
      (void)hipDeviceSynchronize();
      (void)hipFree(g_arena[dev]);
      g_arena[dev] = nullptr;
      g_arena_bytes[dev] = 0;
    }
    e = hipMalloc(&g_arena[dev], bytes);
    if (e != hipSuccess) {
      g_arena[dev] = nullptr;
      *err = fail(VMONARCH_ERR_WORKSPACE, "hipMalloc of %zu workspace bytes failed: %s", bytes, hipGetErrorString(e));
      return nullptr;
    }
    g_arena_bytes[dev] = bytes;
  }
  return g_arena[dev];
}

// Settings of one call: the process-wide defaults (the setters above write them), or a caller's vmonarch_options.
struct Settings {
  float cr_min;
  int entropy_mode;
  int fused_apply;
  int flash_variant;
  int cr_control;
  int cl_control;
  float cl_value;
  void* workspace;  // null: the process-wide workspace / arena
  size_t workspace_bytes;
};

Settings current_settings() {
  Settings s;
  s.cr_min = g_cr_min;
  s.entropy_mode = g_entropy_mode;
  s.fused_apply = g_fused_apply;
  s.flash_variant = g_flash_variant;
  s.cr_control = g_cr_control;
  s.cl_control = g_cl_control;
  s.cl_value = g_cl_value;
  s.workspace = nullptr;
  s.workspace_bytes = 0;
  return s;
}

template <typename E>
int r_update_any(const E* aR, const float* cR, const E* k, const E* v, E* aL, float* cL, E* y, float* lse,
                 const Dims& dm, float row_scale, float cr_min, const Settings& cfg, hipStream_t st);
template <>
int r_update_any<float>(const float* aR, const float* cR, const float* k, const float* v, float* aL, float* cL,
                        float* y, float* lse, const Dims& dm, float row_scale, float cr_min, const Settings&,
                        hipStream_t st) {
  hipError_t e = launch_r_update_generic<float>(aR, cR, k, v, aL, cL, y, lse, dm, row_scale, cr_min, st);
  return e == hipSuccess ? VMONARCH_OK : hip_fail(e, "r_update (plain-ALU f32) launch");
}
template <>
int r_update_any<bf16_t>(const bf16_t* aR, const float* cR, const bf16_t* k, const bf16_t* v, bf16_t* aL, float* cL,
                         bf16_t* y, float* lse, const Dims& dm, float row_scale, float cr_min, const Settings& cfg,
                         hipStream_t st) {
  hipError_t e;
  // variant 2: every update on the kernel that was measured faster for it.  With values: the two-tile kernel, unless a
  // frame has at most 128 tokens (its 256-row query blocks would be mostly padding; the wave-pair kernel's hold 128).
  // Without values: the two-tile kernel at d = 64, the one-tile kernel at d = 128.
  const bool two_tiles = cfg.flash_variant == 1 ||
                         (cfg.flash_variant == 2 && (v != nullptr ? dm.b > 128 : dm.d == 64));
  if (flash_supported(dm) && two_tiles)
    e = launch_r_update_flash2(aR, cR, k, v, aL, cL, y, lse, dm, row_scale, cr_min, cfg.entropy_mode, st);
  else if (flash_supported(dm))
    e = launch_r_update_flash(aR, cR, k, v, aL, cL, y, lse, dm, row_scale, cr_min, cfg.entropy_mode, cfg.fused_apply != 0, st);
  else
    e = launch_r_update_generic<bf16_t>(aR, cR, k, v, aL, cL, y, lse, dm, row_scale, cr_min, st);
  return e == hipSuccess ? VMONARCH_OK : hip_fail(e, "r_update (bf16) launch");
}

// lse_scratch: BH * N floats, needed only when temporal_needs_lse() and the fitting form (y == null) is asked for
template <typename E>
int l_update_any(const E* q, const E* aL, const float* cL, const E* y, E* aR, float* cR, E* out, float* lse_scratch,
                 const Dims& dm, float q_scale, hipStream_t st);
template <>
int l_update_any<float>(const float* q, const float* aL, const float* cL, const float* y, float* aR, float* cR,
                        float* out, float* lse_scratch, const Dims& dm, float q_scale, hipStream_t st) {
  hipError_t e = launch_l_update_generic<float>(q, aL, cL, y, aR, cR, out, lse_scratch, dm, q_scale, st);
  return e == hipSuccess ? VMONARCH_OK : hip_fail(e, "l_update (plain-ALU f32) launch");
}
template <>
int l_update_any<bf16_t>(const bf16_t* q, const bf16_t* aL, const float* cL, const bf16_t* y, bf16_t* aR, float* cR,
                         bf16_t* out, float* lse_scratch, const Dims& dm, float q_scale, hipStream_t st) {
  hipError_t e;
  if (lpass_supported(dm)) {
    e = launch_l_update_mfma(q, aL, cL, y, aR, cR, out, dm, q_scale, st);
  } else if (temporal_flash_supported(dm)) {
    e = launch_l_update_flash(q, aL, cL, y, aR, cR, out, lse_scratch, dm, q_scale, st);
  } else {
    e = launch_l_update_generic<bf16_t>(q, aL, cL, y, aR, cR, out, lse_scratch, dm, q_scale, st);
  }
  return e == hipSuccess ? VMONARCH_OK : hip_fail(e, "l_update (bf16) launch");
}

template <typename E>
int first_frame_any(const E* q, const E* k, const E* v, E* out, float* lse, void* scratch, size_t scratch_bytes,
                    const Dims& dm, int nrows, const int* rows, int flash_variant, hipStream_t st);
template <>
int first_frame_any<float>(const float* q, const float* k, const float* v, float* out, float* lse, void*, size_t,
                           const Dims& dm, int nrows, const int* rows, int, hipStream_t st) {
  hipError_t e = launch_first_frame_generic<float>(q, k, v, out, lse, dm, nrows, rows, st);
  return e == hipSuccess ? VMONARCH_OK : hip_fail(e, "first_frame (plain-ALU f32) launch");
}
template <>
int first_frame_any<bf16_t>(const bf16_t* q, const bf16_t* k, const bf16_t* v, bf16_t* out, float* lse, void* scratch,
                            size_t scratch_bytes, const Dims& dm, int nrows, const int* rows, int flash_variant,
                            hipStream_t st) {
  hipError_t e;
  if (flash_supported(dm))
    e = launch_first_frame_flash(q, k, v, out, lse, scratch, scratch_bytes, dm, nrows, rows, flash_variant != 0, st);
  else
    e = launch_first_frame_generic<bf16_t>(q, k, v, out, lse, dm, nrows, rows, st);
  return e == hipSuccess ? VMONARCH_OK : hip_fail(e, "first_frame (bf16) launch");
}

template <typename E>
int sink_average_any(const E* q, const E* k, const E* v, E* out, const Dims& dm, hipStream_t st);
template <>
int sink_average_any<float>(const float* q, const float* k, const float* v, float* out, const Dims& dm, hipStream_t st) {
  hipError_t e = launch_sink_average_generic<float>(q, k, v, out, dm, st);
  return e == hipSuccess ? VMONARCH_OK : hip_fail(e, "sink_average (f32) launch");
}
template <>
int sink_average_any<bf16_t>(const bf16_t* q, const bf16_t* k, const bf16_t* v, bf16_t* out, const Dims& dm,
                             hipStream_t st) {
  hipError_t e = flash_supported(dm) ? launch_sink_average_flash(q, k, v, out, dm, st)
                                     : launch_sink_average_generic<bf16_t>(q, k, v, out, dm, st);
  return e == hipSuccess ? VMONARCH_OK : hip_fail(e, "sink_average (bf16) launch");
}

template <typename E>
int sink_average_impl(const void* q, const void* k, const void* v, void* out, int B, int heads, int T, int Hs, int Ws,
                      int d, void* stream) {
  if (!q || !k || !v || !out) return fail(VMONARCH_ERR_INVALID_ARG, "null tensor pointer");
  if (out == q || out == k || out == v) return fail(VMONARCH_ERR_INVALID_ARG, "out aliases an input");
  Dims dm;
  int rc = make_dims(B, heads, T, Hs, Ws, d, &dm);
  if (rc) return rc;
  return sink_average_any<E>((const E*)q, (const E*)k, (const E*)v, (E*)out, dm, (hipStream_t)stream);
}

template <typename E>
int attention_impl(const void* q_, const void* k_, const void* v_, void* out_, int B, int heads, int T, int Hs, int Ws,
                   int d, int iters, int recompute, const Settings& cfg, void* stream) {
  if (!q_ || !k_ || !v_ || !out_) return fail(VMONARCH_ERR_INVALID_ARG, "null tensor pointer");
  if (iters < 1) return fail(VMONARCH_ERR_INVALID_ARG, "iters=%d must be >= 1", iters);
  if (recompute < 0 || recompute > VMONARCH_SINK_AVERAGE)
    return fail(VMONARCH_ERR_INVALID_ARG, "recompute=%d: 0 none, 1 first-frame recomputation, 2 sink averaging", recompute);
  Dims dm;
  int rc = make_dims(B, heads, T, Hs, Ws, d, &dm);
  if (rc) return rc;
  if (out_ == q_ || out_ == k_ || out_ == v_) return fail(VMONARCH_ERR_INVALID_ARG, "out aliases an input");
  const E* q = (const E*)q_;
  const E* k = (const E*)k_;
  const E* v = (const E*)v_;
  E* out = (E*)out_;
  hipStream_t st = (hipStream_t)stream;
  WsLayout w = ws_layout(dm, iters, recompute, (int)sizeof(E));
  // w.total > 0: alpha_L, y and c_L are always needed
  char* ws = (char*)get_workspace(w.total, &rc, cfg.workspace, cfg.workspace_bytes, st);
  if (!ws) return rc;
  E* aL = (E*)(ws + w.aL);
  E* y = (E*)(ws + w.y);
  float* cL = (float*)(ws + w.cL);
  E* aR = (E*)(ws + w.aR);
  float* cR = (float*)(ws + w.cR);
  const float s = 1.0f / sqrtf((float)d);
  const float cr_min = cfg.cr_min;
  const int cr_control = cfg.cr_control, cl_control = cfg.cl_control;
  const float cl_value = std::isnan(cfg.cl_value) ? -logf((float)dm.b) : cfg.cl_value;
  // App. A: aR = Q, cR = 1, then `iters` times (R-update; L-update); y = R V and O = L y
  // ride on the last sweep.  Q carries 1/sqrt(d) through row_scale / q_scale.
  if (g_timing) g_n_phases = 0;
  for (int sweep = 0; sweep < iters; ++sweep) {
    const bool last = sweep == iters - 1;
    phase_mark(st, last ? "r_update_last" : "r_update");
    rc = r_update_any<E>(sweep == 0 ? q : aR, sweep == 0 ? nullptr : cR, k, last ? v : nullptr, aL, cL,
                         last ? y : nullptr, nullptr, dm, s, cr_min, cfg, st);
    if (rc) return rc;
    // manual control (App. "Manual Control of Monarch Parameters"): overwrite the term just produced,
    // for key frame 0 (the head's first b entries) or for all frames
    if (cl_control != VMONARCH_CONTROL_NONE) {
      hipError_t e = launch_fill_head_prefix(cL, cl_value, cl_control == VMONARCH_CONTROL_ALL_FRAMES ? dm.N : dm.b,
                                             dm.N, dm.BH, st);
      if (e != hipSuccess) return hip_fail(e, "c_L control fill");
    }
    phase_mark(st, last ? "l_update_last" : "l_update");
    rc = l_update_any<E>(q, aL, cL, last ? y : nullptr, last ? nullptr : aR, last ? nullptr : cR, last ? out : nullptr,
                         (float*)(ws + w.tl), dm, s, st);
    if (rc) return rc;
    if (!last && cr_control != VMONARCH_CONTROL_NONE) {
      hipError_t e = launch_fill_head_prefix(cR, 1.0f, cr_control == VMONARCH_CONTROL_ALL_FRAMES ? dm.N : dm.b, dm.N,
                                             dm.BH, st);
      if (e != hipSuccess) return hip_fail(e, "c_R control fill");
    }
  }
  if (recompute == VMONARCH_SINK_AVERAGE) {
    phase_mark(st, "sink_average");
    rc = sink_average_any<E>(q, k, v, out, dm, st);
    if (rc) return rc;
  } else if (recompute) {
    phase_mark(st, "first_frame");
    rc = first_frame_any<E>(q, k, v, out, nullptr, ws + w.ff, w.total - w.ff, dm, dm.b, nullptr, cfg.flash_variant, st);
    if (rc) return rc;
  }
  phase_mark(st, nullptr);
  return VMONARCH_OK;
}

template <typename E>
int r_update_impl(const void* aR, const float* cR, const void* k, const void* v, void* aL, float* cL, void* y,
                  float* lse, int B, int heads, int T, int Hs, int Ws, int d, float row_scale, float cr_min,
                  void* stream) {
  if (!aR || !k || !aL || !cL) return fail(VMONARCH_ERR_INVALID_ARG, "null tensor pointer");
  if ((v == nullptr) != (y == nullptr)) return fail(VMONARCH_ERR_INVALID_ARG, "v and y_out must be given together");
  if (!(row_scale > 0.f) || !(cr_min >= 0.f)) return fail(VMONARCH_ERR_INVALID_ARG, "row_scale must be > 0 and cr_min >= 0");
  Dims dm;
  int rc = make_dims(B, heads, T, Hs, Ws, d, &dm);
  if (rc) return rc;
  return r_update_any<E>((const E*)aR, cR, (const E*)k, (const E*)v, (E*)aL, cL, (E*)y, lse, dm, row_scale, cr_min,
                         current_settings(), (hipStream_t)stream);
}

template <typename E>
int l_update_impl(const void* q, const void* aL, const float* cL, const void* y, void* aR, float* cR, void* out, int B,
                  int heads, int T, int Hs, int Ws, int d, float q_scale, void* stream) {
  if (!q || !aL || !cL) return fail(VMONARCH_ERR_INVALID_ARG, "null tensor pointer");
  const bool fin = y != nullptr;
  if (fin && (!out || aR || cR)) return fail(VMONARCH_ERR_INVALID_ARG, "with y, give out and neither aR_out nor cR_out");
  if (!fin && (!aR || !cR || out)) return fail(VMONARCH_ERR_INVALID_ARG, "without y, give aR_out and cR_out and not out");
  Dims dm;
  int rc = make_dims(B, heads, T, Hs, Ws, d, &dm);
  if (rc) return rc;
  float* lse_scratch = nullptr;
  if (!fin && temporal_needs_lse(dm, (int)sizeof(E))) {
    lse_scratch = (float*)get_workspace(align_up((size_t)dm.BH * dm.N * sizeof(float)), &rc, nullptr, 0, (hipStream_t)stream);
    if (!lse_scratch) return rc;
  }
  return l_update_any<E>((const E*)q, (const E*)aL, cL, (const E*)y, (E*)aR, cR, (E*)out, lse_scratch, dm, q_scale,
                         (hipStream_t)stream);
}

template <typename E>
int first_frame_impl(const void* q, const void* k, const void* v, void* out, float* lse, int B, int heads, int T,
                     int Hs, int Ws, int d, long long row_begin, long long row_count, void* stream) {
  if (!q || !k || !v || !out) return fail(VMONARCH_ERR_INVALID_ARG, "null tensor pointer");
  Dims dm;
  int rc = make_dims(B, heads, T, Hs, Ws, d, &dm);
  if (rc) return rc;
  if (row_count < 0) row_count = dm.b;  // the first frame
  if (row_begin < 0 || row_count < 1 || row_begin + row_count > dm.N)
    return fail(VMONARCH_ERR_INVALID_ARG, "rows [%lld, %lld) do not lie inside the %lld tokens of a head", row_begin,
                row_begin + row_count, dm.N);
  const int nrows = (int)row_count;
  void* scratch = nullptr;
  size_t sb = 0;
  if (sizeof(E) == 2 && flash_supported(dm)) {
    sb = align_up(first_frame_flash_scratch_bytes(dm, nrows));
    if (sb > 0) {
      scratch = get_workspace(sb, &rc, nullptr, 0, (hipStream_t)stream);
      if (!scratch) return rc;
    }
  }
  // the kernels index query rows from the pointers they are given: hand them the first row of the range
  return first_frame_any<E>((const E*)q + row_begin * d, (const E*)k, (const E*)v, (E*)out + row_begin * d,
                            lse ? lse + row_begin : nullptr, scratch, sb, dm, nrows, nullptr, g_flash_variant,
                            (hipStream_t)stream);
}

// Exact attention of a list of rows (the same list for every head).
template <typename E>
int recompute_tokens_impl(const void* q, const void* k, const void* v, void* out, const int32_t* rows, long long n_rows,
                          int B, int heads, int T, int Hs, int Ws, int d, void* stream) {
  if (!q || !k || !v || !out || !rows) return fail(VMONARCH_ERR_INVALID_ARG, "null pointer");
  Dims dm;
  int rc = make_dims(B, heads, T, Hs, Ws, d, &dm);
  if (rc) return rc;
  if (n_rows < 1 || n_rows > 0x7fffffffLL / 2)
    return fail(VMONARCH_ERR_INVALID_ARG, "n_rows=%lld must lie in [1, 2^30)", n_rows);
  const int nrows = (int)n_rows;
  void* scratch = nullptr;
  size_t sb = 0;
  if (sizeof(E) == 2 && flash_supported(dm)) {
    sb = align_up(first_frame_flash_scratch_bytes(dm, nrows));
    if (sb > 0) {
      scratch = get_workspace(sb, &rc, nullptr, 0, (hipStream_t)stream);
      if (!scratch) return rc;
    }
  }
  return first_frame_any<E>((const E*)q, (const E*)k, (const E*)v, (E*)out, nullptr, scratch, sb, dm, nrows, rows,
                            g_flash_variant, (hipStream_t)stream);
}

template <typename E>
int entropy_bwd_impl(const void* q, const float* cR, const void* k, const void* v, const void* o, const void* dO,
                     const float* lse, const float* H, const float* dH, void* dq, void* dk, void* dv, int B, int heads,
                     int T, int Hs, int Ws, int d, float row_scale, float cr_min, void* stream) {
  if (!q || !k || !v || !o || !dO || !lse || !H || !dq || !dk || !dv)
    return fail(VMONARCH_ERR_INVALID_ARG, "null tensor pointer");
  if (!(row_scale > 0.f) || !(cr_min >= 0.f)) return fail(VMONARCH_ERR_INVALID_ARG, "row_scale must be > 0 and cr_min >= 0");
  Dims dm;
  int rc = make_dims(B, heads, T, Hs, Ws, d, &dm);
  if (rc) return rc;
  const bool mfma = sizeof(E) == 2 && entropy_bwd_mfma_supported(dm);
  void* scratch = get_workspace(align_up(mfma ? entropy_bwd_mfma_scratch_bytes(dm) : entropy_bwd_scratch_bytes(dm)), &rc,
                                nullptr, 0, (hipStream_t)stream);
  if (!scratch) return rc;
  if (mfma) {
    hipError_t e = launch_entropy_bwd_mfma((const bf16_t*)q, cR, (const bf16_t*)k, (const bf16_t*)v, (const bf16_t*)o,
                                           (const bf16_t*)dO, lse, H, dH, (bf16_t*)dq, (bf16_t*)dk, (bf16_t*)dv, scratch,
                                           dm, row_scale, cr_min, (hipStream_t)stream);
    return e == hipSuccess ? VMONARCH_OK : hip_fail(e, "entropy_attention_bwd (MFMA) launch");
  }
  hipError_t e = launch_entropy_bwd_generic<E>((const E*)q, cR, (const E*)k, (const E*)v, (const E*)o, (const E*)dO, lse,
                                               H, dH, (E*)dq, (E*)dk, (E*)dv, (float*)scratch, dm, row_scale, cr_min,
                                               (hipStream_t)stream);
  return e == hipSuccess ? VMONARCH_OK : hip_fail(e, "entropy_attention_bwd launch");
}

}  // namespace

extern "C" {
#pragma GCC visibility push(default)

int vmonarch_version(void) { return 100; }
const char* vmonarch_last_error(void) { return g_err; }

int vmonarch_set_cr_min(float cr_min) {
  if (!(cr_min >= 0.f)) return fail(VMONARCH_ERR_INVALID_ARG, "cr_min must be >= 0");
  g_cr_min = cr_min;
  return VMONARCH_OK;
}
float vmonarch_get_cr_min(void) { return g_cr_min; }

int vmonarch_set_fused_apply(int enable) {
  g_fused_apply = enable != 0;
  return VMONARCH_OK;
}
int vmonarch_get_fused_apply(void) { return g_fused_apply; }

int vmonarch_set_flash_variant(int variant) {
  if (variant < 0 || variant > 2) return fail(VMONARCH_ERR_INVALID_ARG, "flash variant is 0, 1 or 2");
  g_flash_variant = variant;
  return VMONARCH_OK;
}
int vmonarch_get_flash_variant(void) { return g_flash_variant; }

int vmonarch_set_manual_control(int cr_control, int cl_control, float cl_value) {
  if (cr_control < VMONARCH_CONTROL_NONE || cr_control > VMONARCH_CONTROL_ALL_FRAMES ||
      cl_control < VMONARCH_CONTROL_NONE || cl_control > VMONARCH_CONTROL_ALL_FRAMES)
    return fail(VMONARCH_ERR_INVALID_ARG, "control modes are 0 (none), 1 (first frame), 2 (all frames)");
  if (std::isinf(cl_value)) return fail(VMONARCH_ERR_INVALID_ARG, "cl_value must be finite, or NaN for -log(b)");
  g_cr_control = cr_control;
  g_cl_control = cl_control;
  g_cl_value = cl_value;
  return VMONARCH_OK;
}
int vmonarch_get_manual_control(int* cr_control, int* cl_control, float* cl_value) {
  if (cr_control) *cr_control = g_cr_control;
  if (cl_control) *cl_control = g_cl_control;
  if (cl_value) *cl_value = g_cl_value;
  return VMONARCH_OK;
}

int vmonarch_set_phase_timing(int enable) {
  g_timing = enable != 0;
  return VMONARCH_OK;
}

int vmonarch_get_phase_timing(int* n_phases, float* ms_host, char* names_host, int cap) {
  if (!n_phases || !ms_host || !names_host || cap <= 0) return fail(VMONARCH_ERR_INVALID_ARG, "null output or cap <= 0");
  *n_phases = 0;
  if (!g_timing || !g_ev_created || g_n_phases == 0) return VMONARCH_OK;
  hipError_t e = hipEventSynchronize(g_ev[g_n_phases]);
  if (e != hipSuccess) return hip_fail(e, "hipEventSynchronize");
  const int n = g_n_phases < cap ? g_n_phases : cap;
  for (int i = 0; i < n; ++i) {
    e = hipEventElapsedTime(&ms_host[i], g_ev[i], g_ev[i + 1]);
    if (e != hipSuccess) return hip_fail(e, "hipEventElapsedTime");
    snprintf(names_host + 32 * i, 32, "%s", g_phase_name[i]);
  }
  *n_phases = n;
  return VMONARCH_OK;
}

int vmonarch_set_entropy_mode(int mode) {
  if (mode != VMONARCH_ENTROPY_ONLINE && mode != VMONARCH_ENTROPY_IDENTITY)
    return fail(VMONARCH_ERR_INVALID_ARG, "unknown entropy mode %d", mode);
  g_entropy_mode = mode;
  return VMONARCH_OK;
}
int vmonarch_get_entropy_mode(void) { return g_entropy_mode; }

size_t vmonarch_workspace_bytes(int B, int heads, int T, int Hs, int Ws, int d, int iters, int recompute,
                                int elem_bytes) {
  Dims dm;
  if (iters < 1 || (elem_bytes != 2 && elem_bytes != 4)) return 0;
  if (make_dims(B, heads, T, Hs, Ws, d, &dm)) return 0;
  return ws_layout(dm, iters, recompute, elem_bytes).total;
}

int vmonarch_set_workspace(void* dev_ptr, size_t bytes) {
  std::lock_guard<std::mutex> lk(g_ws_mutex);
  if ((dev_ptr == nullptr) != (bytes == 0)) return fail(VMONARCH_ERR_INVALID_ARG, "pointer and size must both be zero or both non-zero");
  if (((uintptr_t)dev_ptr & 255) != 0) return fail(VMONARCH_ERR_INVALID_ARG, "workspace must be 256-byte aligned");
  g_user_ws = dev_ptr;
  g_user_ws_bytes = bytes;
  return VMONARCH_OK;
}

int vmonarch_shutdown(void) {
  std::lock_guard<std::mutex> lk(g_ws_mutex);
  int cur = 0;
  (void)hipGetDevice(&cur);
  for (int dev = 0; dev < 64; ++dev) {
    if (g_arena[dev] != nullptr) {
      (void)hipSetDevice(dev);
      (void)hipDeviceSynchronize();
      (void)hipFree(g_arena[dev]);
      g_arena[dev] = nullptr;
      g_arena_bytes[dev] = 0;
    }
  }
  (void)hipSetDevice(cur);
  g_user_ws = nullptr;
  g_user_ws_bytes = 0;
  return VMONARCH_OK;
}

int vmonarch_attention(const void* q, const void* k, const void* v, void* out, int B, int heads, int T, int Hs, int Ws,
                       int d, int iters, int recompute, void* stream) {
  return attention_impl<bf16_t>(q, k, v, out, B, heads, T, Hs, Ws, d, iters, recompute, current_settings(), stream);
}
int vmonarch_attention_f32(const void* q, const void* k, const void* v, void* out, int B, int heads, int T, int Hs,
                           int Ws, int d, int iters, int recompute, void* stream) {
  return attention_impl<float>(q, k, v, out, B, heads, T, Hs, Ws, d, iters, recompute, current_settings(), stream);
}

static int settings_from_options(const vmonarch_options* o, Settings* cfg) {
  if (o == nullptr) return fail(VMONARCH_ERR_INVALID_ARG, "null options");
  if (o->struct_bytes != sizeof(vmonarch_options))
    return fail(VMONARCH_ERR_INVALID_ARG, "options.struct_bytes is %u, this library's vmonarch_options has %zu bytes",
                o->struct_bytes, sizeof(vmonarch_options));
  if (!(o->cr_min >= 0.f)) return fail(VMONARCH_ERR_INVALID_ARG, "options.cr_min must be >= 0");
  if (o->entropy_mode != VMONARCH_ENTROPY_ONLINE && o->entropy_mode != VMONARCH_ENTROPY_IDENTITY)
    return fail(VMONARCH_ERR_INVALID_ARG, "unknown options.entropy_mode %d", o->entropy_mode);
  if (o->flash_variant < 0 || o->flash_variant > 2) return fail(VMONARCH_ERR_INVALID_ARG, "options.flash_variant is 0, 1 or 2");
  if (o->cr_control < VMONARCH_CONTROL_NONE || o->cr_control > VMONARCH_CONTROL_ALL_FRAMES ||
      o->cl_control < VMONARCH_CONTROL_NONE || o->cl_control > VMONARCH_CONTROL_ALL_FRAMES)
    return fail(VMONARCH_ERR_INVALID_ARG, "options control modes are 0 (none), 1 (first frame), 2 (all frames)");
  if (std::isinf(o->cl_value)) return fail(VMONARCH_ERR_INVALID_ARG, "options.cl_value must be finite, or NaN for -log(b)");
  if ((o->workspace == nullptr) != (o->workspace_bytes == 0))
    return fail(VMONARCH_ERR_INVALID_ARG, "options.workspace and workspace_bytes must both be zero or both non-zero");
  if (((uintptr_t)o->workspace & 255) != 0) return fail(VMONARCH_ERR_INVALID_ARG, "options.workspace must be 256-byte aligned");
  cfg->cr_min = o->cr_min;
  cfg->entropy_mode = o->entropy_mode;
  cfg->fused_apply = o->fused_apply != 0;
  cfg->flash_variant = o->flash_variant;
  cfg->cr_control = o->cr_control;
  cfg->cl_control = o->cl_control;
  cfg->cl_value = o->cl_value;
  cfg->workspace = o->workspace;
  cfg->workspace_bytes = o->workspace_bytes;
  return VMONARCH_OK;
}

int vmonarch_options_init(vmonarch_options* options) {
  if (options == nullptr) return fail(VMONARCH_ERR_INVALID_ARG, "null options");
  options->struct_bytes = (uint32_t)sizeof(vmonarch_options);
  options->cr_min = 0.1f;
  options->entropy_mode = VMONARCH_ENTROPY_ONLINE;
  options->fused_apply = 1;
  options->flash_variant = 2;
  options->cr_control = VMONARCH_CONTROL_NONE;
  options->cl_control = VMONARCH_CONTROL_NONE;
  options->cl_value = NAN;
  options->workspace = nullptr;
  options->workspace_bytes = 0;
  return VMONARCH_OK;
}

int vmonarch_attention_ex(const void* q, const void* k, const void* v, void* out, int B, int heads, int T, int Hs, int Ws,
                          int d, int iters, int recompute, const vmonarch_options* options, void* stream) {
  Settings cfg;
  int rc = settings_from_options(options, &cfg);
  if (rc) return rc;
  return attention_impl<bf16_t>(q, k, v, out, B, heads, T, Hs, Ws, d, iters, recompute, cfg, stream);
}
int vmonarch_attention_ex_f32(const void* q, const void* k, const void* v, void* out, int B, int heads, int T, int Hs,
                              int Ws, int d, int iters, int recompute, const vmonarch_options* options, void* stream) {
  Settings cfg;
  int rc = settings_from_options(options, &cfg);
  if (rc) return rc;
  return attention_impl<float>(q, k, v, out, B, heads, T, Hs, Ws, d, iters, recompute, cfg, stream);
}

int vmonarch_r_update(const void* aR, const float* cR, const void* k, const void* v, void* aL_out, float* cL_out,
                      void* y_out, int B, int heads, int T, int Hs, int Ws, int d, float row_scale, float cr_min,
                      void* stream) {
  return r_update_impl<bf16_t>(aR, cR, k, v, aL_out, cL_out, y_out, nullptr, B, heads, T, Hs, Ws, d, row_scale, cr_min,
                               stream);
}
int vmonarch_r_update_f32(const void* aR, const float* cR, const void* k, const void* v, void* aL_out, float* cL_out,
                          void* y_out, int B, int heads, int T, int Hs, int Ws, int d, float row_scale, float cr_min,
                          void* stream) {
  return r_update_impl<float>(aR, cR, k, v, aL_out, cL_out, y_out, nullptr, B, heads, T, Hs, Ws, d, row_scale, cr_min,
                              stream);
}
int vmonarch_r_update_lse(const void* aR, const float* cR, const void* k, const void* v, void* aL_out, float* cL_out,
                          void* y_out, float* lse_out, int B, int heads, int T, int Hs, int Ws, int d, float row_scale,
                          float cr_min, void* stream) {
  if (!lse_out) return fail(VMONARCH_ERR_INVALID_ARG, "null lse_out");
  return r_update_impl<bf16_t>(aR, cR, k, v, aL_out, cL_out, y_out, lse_out, B, heads, T, Hs, Ws, d, row_scale, cr_min,
                               stream);
}
int vmonarch_r_update_lse_f32(const void* aR, const float* cR, const void* k, const void* v, void* aL_out,
                              float* cL_out, void* y_out, float* lse_out, int B, int heads, int T, int Hs, int Ws,
                              int d, float row_scale, float cr_min, void* stream) {
  if (!lse_out) return fail(VMONARCH_ERR_INVALID_ARG, "null lse_out");
  return r_update_impl<float>(aR, cR, k, v, aL_out, cL_out, y_out, lse_out, B, heads, T, Hs, Ws, d, row_scale, cr_min,
                              stream);
}

int vmonarch_l_update(const void* q, const void* aL, const float* cL, const void* y, void* aR_out, float* cR_out,
                      void* out, int B, int heads, int T, int Hs, int Ws, int d, float q_scale, void* stream) {
  return l_update_impl<bf16_t>(q, aL, cL, y, aR_out, cR_out, out, B, heads, T, Hs, Ws, d, q_scale, stream);
}
int vmonarch_l_update_f32(const void* q, const void* aL, const float* cL, const void* y, void* aR_out, float* cR_out,
                          void* out, int B, int heads, int T, int Hs, int Ws, int d, float q_scale, void* stream) {
  return l_update_impl<float>(q, aL, cL, y, aR_out, cR_out, out, B, heads, T, Hs, Ws, d, q_scale, stream);
}

int vmonarch_first_frame_attention(const void* q, const void* k, const void* v, void* out, int B, int heads, int T,
                                   int Hs, int Ws, int d, void* stream) {
  return first_frame_impl<bf16_t>(q, k, v, out, nullptr, B, heads, T, Hs, Ws, d, 0, -1, stream);
}
int vmonarch_first_frame_attention_f32(const void* q, const void* k, const void* v, void* out, int B, int heads, int T,
                                       int Hs, int Ws, int d, void* stream) {
  return first_frame_impl<float>(q, k, v, out, nullptr, B, heads, T, Hs, Ws, d, 0, -1, stream);
}
int vmonarch_first_frame_attention_lse(const void* q, const void* k, const void* v, void* out, float* lse_out, int B,
                                       int heads, int T, int Hs, int Ws, int d, void* stream) {
  if (!lse_out) return fail(VMONARCH_ERR_INVALID_ARG, "null lse_out");
  return first_frame_impl<bf16_t>(q, k, v, out, lse_out, B, heads, T, Hs, Ws, d, 0, -1, stream);
}
int vmonarch_first_frame_attention_lse_f32(const void* q, const void* k, const void* v, void* out, float* lse_out,
                                           int B, int heads, int T, int Hs, int Ws, int d, void* stream) {
  if (!lse_out) return fail(VMONARCH_ERR_INVALID_ARG, "null lse_out");
  return first_frame_impl<float>(q, k, v, out, lse_out, B, heads, T, Hs, Ws, d, 0, -1, stream);
}

int vmonarch_recompute_rows(const void* q, const void* k, const void* v, void* out, int B, int heads, int T, int Hs,
                            int Ws, int d, long long row_begin, long long row_count, void* stream) {
  if (row_count < 1) return fail(VMONARCH_ERR_INVALID_ARG, "row_count must be positive");
  return first_frame_impl<bf16_t>(q, k, v, out, nullptr, B, heads, T, Hs, Ws, d, row_begin, row_count, stream);
}
int vmonarch_recompute_rows_f32(const void* q, const void* k, const void* v, void* out, int B, int heads, int T, int Hs,
                                int Ws, int d, long long row_begin, long long row_count, void* stream) {
  if (row_count < 1) return fail(VMONARCH_ERR_INVALID_ARG, "row_count must be positive");
  return first_frame_impl<float>(q, k, v, out, nullptr, B, heads, T, Hs, Ws, d, row_begin, row_count, stream);
}

int vmonarch_recompute_tokens(const void* q, const void* k, const void* v, void* out, const int32_t* rows_dev,
                              long long n_rows, int B, int heads, int T, int Hs, int Ws, int d, void* stream) {
  return recompute_tokens_impl<bf16_t>(q, k, v, out, rows_dev, n_rows, B, heads, T, Hs, Ws, d, stream);
}
int vmonarch_recompute_tokens_f32(const void* q, const void* k, const void* v, void* out, const int32_t* rows_dev,
                                  long long n_rows, int B, int heads, int T, int Hs, int Ws, int d, void* stream) {
  return recompute_tokens_impl<float>(q, k, v, out, rows_dev, n_rows, B, heads, T, Hs, Ws, d, stream);
}

int vmonarch_recompute_rows_noalloc(const void* q, const void* k, const void* v, void* out, int B, int heads, int T,
                                    int Hs, int Ws, int d, long long row_begin, long long row_count, void* stream) {
  if (!q || !k || !v || !out) return fail(VMONARCH_ERR_INVALID_ARG, "null tensor pointer");
  Dims dm;
  int rc = make_dims(B, heads, T, Hs, Ws, d, &dm);
  if (rc) return rc;
  if (row_begin < 0 || row_count < 1 || row_begin + row_count > dm.N)
    return fail(VMONARCH_ERR_INVALID_ARG, "rows [%lld, %lld) do not lie inside the %lld tokens of a head", row_begin,
                row_begin + row_count, dm.N);
  const int nrows = (int)row_count;
  void* sp = nullptr;
  size_t sb = 0;
  if (flash_supported(dm)) {  // the plain-ALU kernel keeps no partial results
    sb = align_up(first_frame_flash_scratch_bytes(dm, nrows));
    if (sb > kNoAllocScratchBytes)
      return fail(VMONARCH_ERR_WORKSPACE,
                  "the key-range partials of %d rows x %d heads need %zu bytes, the built-in buffer holds %zu: use "
                  "vmonarch_recompute_rows, or recompute fewer rows per call",
                  nrows, dm.BH, sb, kNoAllocScratchBytes);
    if (sb > 0) {
      sp = noalloc_scratch(&rc);
      if (!sp) return rc;
    }
  }
  // every partial the merge reads is written by the key-range pass of the same call: nothing to clear
  return first_frame_any<bf16_t>((const bf16_t*)q + row_begin * d, (const bf16_t*)k, (const bf16_t*)v,
                                 (bf16_t*)out + row_begin * d, nullptr, sp, sb, dm, nrows, nullptr, g_flash_variant,
                                 (hipStream_t)stream);
}

int vmonarch_sink_average(const void* q, const void* k, const void* v, void* out, int B, int heads, int T, int Hs,
                          int Ws, int d, void* stream) {
  return sink_average_impl<bf16_t>(q, k, v, out, B, heads, T, Hs, Ws, d, stream);
}
int vmonarch_sink_average_f32(const void* q, const void* k, const void* v, void* out, int B, int heads, int T, int Hs,
                              int Ws, int d, void* stream) {
  return sink_average_impl<float>(q, k, v, out, B, heads, T, Hs, Ws, d, stream);
}

int vmonarch_index_maps(int T, int Hs, int Ws, int32_t* perm_host, int32_t* inv_host) {
  if (!perm_host || !inv_host) return fail(VMONARCH_ERR_INVALID_ARG, "null table pointer");
  if (T <= 0 || Hs <= 0 || Ws <= 0) return fail(VMONARCH_ERR_INVALID_ARG, "sizes must be positive");
  long long b = (long long)Hs * Ws, N = b * T;
  if (N > 0x7fffffffLL) return fail(VMONARCH_ERR_UNSUPPORTED, "N=%lld does not fit int32", N);
  for (long long i = 0; i < b; ++i)
    for (long long j = 0; j < T; ++j) {
      perm_host[i * T + j] = (int32_t)(j * b + i);
      inv_host[j * b + i] = (int32_t)(i * T + j);
    }
  return VMONARCH_OK;
}

int vmonarch_permute_tokens(const void* in, void* out, int B, int heads, int T, int Hs, int Ws, int row_bytes,
                            int to_position_major, void* stream) {
  if (!in || !out || in == out) return fail(VMONARCH_ERR_INVALID_ARG, "null or aliased tensor pointer");
  if (row_bytes <= 0 || (row_bytes & 3)) return fail(VMONARCH_ERR_INVALID_ARG, "row_bytes must be a positive multiple of 4");
  Dims dm;
  int rc = make_dims(B, heads, T, Hs, Ws, 1, &dm);
  if (rc) return rc;
  hipError_t e = launch_permute_tokens(in, out, dm, row_bytes, to_position_major, (hipStream_t)stream);
  return e == hipSuccess ? VMONARCH_OK : hip_fail(e, "permute_tokens launch");
}

int vmonarch_entropy_attention_bwd(const void* q, const float* cR, const void* k, const void* v, const void* o,
                                   const void* dO, const float* lse, const float* H, const float* dH, void* dq_out,
                                   void* dk_out, void* dv_out, int B, int heads, int T, int Hs, int Ws, int d,
                                   float row_scale, float cr_min, void* stream) {
  return entropy_bwd_impl<bf16_t>(q, cR, k, v, o, dO, lse, H, dH, dq_out, dk_out, dv_out, B, heads, T, Hs, Ws, d,
                                  row_scale, cr_min, stream);
}
int vmonarch_entropy_attention_bwd_f32(const void* q, const float* cR, const void* k, const void* v, const void* o,
                                       const void* dO, const float* lse, const float* H, const float* dH,
                                       void* dq_out, void* dk_out, void* dv_out, int B, int heads, int T, int Hs,
                                       int Ws, int d, float row_scale, float cr_min, void* stream) {
  return entropy_bwd_impl<float>(q, cR, k, v, o, dO, lse, H, dH, dq_out, dk_out, dv_out, B, heads, T, Hs, Ws, d,
                                 row_scale, cr_min, stream);
}

int vmonarch_mfma_probe(const void* operands, float* out, int blocks, int iters, double* flops_host, void* stream) {
  if (!operands || !out) return fail(VMONARCH_ERR_INVALID_ARG, "null pointer");
  if (blocks <= 0 || iters <= 0) return fail(VMONARCH_ERR_INVALID_ARG, "blocks and iters must be positive");
  if (flops_host) *flops_host = (double)blocks * 8.0 * (double)iters * 8.0 * (2.0 * 32 * 32 * 16);
  hipError_t e = launch_mfma_probe(operands, out, blocks, iters, (hipStream_t)stream);
  return e == hipSuccess ? VMONARCH_OK : hip_fail(e, "mfma_probe launch");
}

#pragma GCC visibility pop
}  // extern "C"

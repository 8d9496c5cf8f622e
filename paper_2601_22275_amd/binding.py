"""Thin ctypes binding of libvmonarch.so (argument marshalling only).

Every function takes torch CUDA tensors for device memory, hands their raw
pointers and the current HIP stream to the C ABI declared in
``include/vmonarch.h`` and raises ``VMonarchError`` on a non-zero return code.
No arithmetic of the method happens on the Python side, and there is no
fallback: if the shared library has not been built, importing this module's
library handle raises.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import c_char_p, c_float, c_int, c_size_t, c_void_p

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libvmonarch.so")

ENTROPY_ONLINE = 0
ENTROPY_IDENTITY = 1

EXPORTS = [
    "vmonarch_version", "vmonarch_last_error", "vmonarch_set_cr_min", "vmonarch_get_cr_min",
    "vmonarch_set_entropy_mode", "vmonarch_get_entropy_mode", "vmonarch_workspace_bytes",
    "vmonarch_set_workspace", "vmonarch_shutdown", "vmonarch_attention", "vmonarch_attention_f32",
    "vmonarch_r_update", "vmonarch_r_update_f32", "vmonarch_l_update", "vmonarch_l_update_f32",
    "vmonarch_first_frame_attention", "vmonarch_first_frame_attention_f32", "vmonarch_index_maps",
    "vmonarch_permute_tokens", "vmonarch_set_phase_timing", "vmonarch_get_phase_timing",
    "vmonarch_r_update_lse", "vmonarch_r_update_lse_f32", "vmonarch_first_frame_attention_lse",
    "vmonarch_first_frame_attention_lse_f32", "vmonarch_mfma_probe", "vmonarch_entropy_attention_bwd",
    "vmonarch_entropy_attention_bwd_f32", "vmonarch_recompute_rows", "vmonarch_recompute_rows_f32",
    "vmonarch_sink_average", "vmonarch_sink_average_f32", "vmonarch_set_manual_control", "vmonarch_get_manual_control",
    "vmonarch_set_fused_apply", "vmonarch_get_fused_apply", "vmonarch_recompute_rows_noalloc",
    "vmonarch_set_flash_variant", "vmonarch_get_flash_variant",
    "vmonarch_options_init", "vmonarch_attention_ex", "vmonarch_attention_ex_f32",
    "vmonarch_recompute_tokens", "vmonarch_recompute_tokens_f32",
]


class VMonarchError(RuntimeError):
    pass


class Options(ctypes.Structure):
    """vmonarch_options of include/vmonarch.h: the settings and the workspace of one call."""
    _fields_ = [("struct_bytes", ctypes.c_uint32), ("cr_min", c_float), ("entropy_mode", c_int),
                ("fused_apply", c_int), ("flash_variant", c_int), ("cr_control", c_int), ("cl_control", c_int),
                ("cl_value", c_float), ("workspace", c_void_p), ("workspace_bytes", c_size_t)]


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded library; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise VMonarchError(f"{LIB_PATH} is missing: run `python -m paper_2601_22275_amd.build` "
                                "(or __graft_entry__.build()) first")
        L = ctypes.CDLL(LIB_PATH)
        dims = [c_int] * 6
        L.vmonarch_version.restype = c_int
        L.vmonarch_last_error.restype = c_char_p
        L.vmonarch_set_cr_min.argtypes = [c_float]
        L.vmonarch_get_cr_min.restype = c_float
        L.vmonarch_set_entropy_mode.argtypes = [c_int]
        L.vmonarch_set_fused_apply.argtypes = [c_int]
        L.vmonarch_workspace_bytes.restype = c_size_t
        L.vmonarch_workspace_bytes.argtypes = dims + [c_int, c_int, c_int]
        L.vmonarch_set_workspace.argtypes = [c_void_p, c_size_t]
        L.vmonarch_set_phase_timing.argtypes = [c_int]
        L.vmonarch_get_phase_timing.argtypes = [c_void_p, c_void_p, c_void_p, c_int]
        for name in ("vmonarch_attention", "vmonarch_attention_f32"):
            getattr(L, name).argtypes = [c_void_p] * 4 + dims + [c_int, c_int, c_void_p]
        for name in ("vmonarch_r_update", "vmonarch_r_update_f32"):
            getattr(L, name).argtypes = [c_void_p] * 7 + dims + [c_float, c_float, c_void_p]
        for name in ("vmonarch_r_update_lse", "vmonarch_r_update_lse_f32"):
            getattr(L, name).argtypes = [c_void_p] * 8 + dims + [c_float, c_float, c_void_p]
        for name in ("vmonarch_first_frame_attention_lse", "vmonarch_first_frame_attention_lse_f32"):
            getattr(L, name).argtypes = [c_void_p] * 5 + dims + [c_void_p]
        for name in ("vmonarch_l_update", "vmonarch_l_update_f32"):
            getattr(L, name).argtypes = [c_void_p] * 7 + dims + [c_float, c_void_p]
        for name in ("vmonarch_first_frame_attention", "vmonarch_first_frame_attention_f32"):
            getattr(L, name).argtypes = [c_void_p] * 4 + dims + [c_void_p]
        for name in ("vmonarch_entropy_attention_bwd", "vmonarch_entropy_attention_bwd_f32"):
            getattr(L, name).argtypes = [c_void_p] * 12 + dims + [c_float, c_float, c_void_p]
        for name in ("vmonarch_recompute_tokens", "vmonarch_recompute_tokens_f32"):
            getattr(L, name).argtypes = [c_void_p] * 5 + [ctypes.c_longlong] + dims + [c_void_p]
        L.vmonarch_options_init.argtypes = [ctypes.POINTER(Options)]
        for name in ("vmonarch_attention_ex", "vmonarch_attention_ex_f32"):
            getattr(L, name).argtypes = [c_void_p] * 4 + dims + [c_int, c_int, ctypes.POINTER(Options), c_void_p]
        for name in ("vmonarch_recompute_rows", "vmonarch_recompute_rows_f32", "vmonarch_recompute_rows_noalloc"):
            getattr(L, name).argtypes = [c_void_p] * 4 + dims + [ctypes.c_longlong, ctypes.c_longlong, c_void_p]
        for name in ("vmonarch_sink_average", "vmonarch_sink_average_f32"):
            getattr(L, name).argtypes = [c_void_p] * 4 + dims + [c_void_p]
        L.vmonarch_set_manual_control.argtypes = [c_int, c_int, c_float]
        L.vmonarch_get_manual_control.argtypes = [c_void_p, c_void_p, c_void_p]
        L.vmonarch_mfma_probe.argtypes = [c_void_p, c_void_p, c_int, c_int, c_void_p, c_void_p]
        L.vmonarch_index_maps.argtypes = [c_int, c_int, c_int, c_void_p, c_void_p]
        L.vmonarch_permute_tokens.argtypes = [c_void_p, c_void_p, c_int, c_int, c_int, c_int, c_int, c_int, c_int,
                                              c_void_p]
        _lib = L
    return _lib


def _check(rc: int) -> None:
    if rc != 0:
        raise VMonarchError(f"vmonarch error {rc}: {lib().vmonarch_last_error().decode()}")


def _ptr(t):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous CUDA tensors"
    return c_void_p(t.data_ptr())


def _stream():
    return c_void_p(torch.cuda.current_stream().cuda_stream)


def _suffix(t: torch.Tensor) -> str:
    if t.dtype == torch.bfloat16:
        return ""
    if t.dtype == torch.float32:
        return "_f32"
    raise VMonarchError(f"unsupported dtype {t.dtype}")


def version() -> int:
    return lib().vmonarch_version()


def set_cr_min(x: float) -> None:
    _check(lib().vmonarch_set_cr_min(c_float(x)))


def get_cr_min() -> float:
    return float(lib().vmonarch_get_cr_min())


def set_manual_control(cr_control: int = 0, cl_control: int = 0, cl_value: float = float("nan")) -> None:
    _check(lib().vmonarch_set_manual_control(cr_control, cl_control, cl_value))


def get_manual_control():
    a, b, c = ctypes.c_int(), ctypes.c_int(), ctypes.c_float()
    _check(lib().vmonarch_get_manual_control(ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)))
    return a.value, b.value, c.value


def set_fused_apply(enable: bool) -> None:
    _check(lib().vmonarch_set_fused_apply(int(enable)))


def get_fused_apply() -> bool:
    return bool(lib().vmonarch_get_fused_apply())


def set_entropy_mode(mode: int) -> None:
    _check(lib().vmonarch_set_entropy_mode(mode))


def set_phase_timing(enable: bool) -> None:
    _check(lib().vmonarch_set_phase_timing(int(bool(enable))))


def get_phase_timing():
    """[(phase name, milliseconds)] of the last attention call made while timing was enabled."""
    cap = 32
    n = c_int(0)
    ms = (c_float * cap)()
    names = ctypes.create_string_buffer(cap * 32)
    _check(lib().vmonarch_get_phase_timing(ctypes.byref(n), ms, names, cap))
    return [(names.raw[32 * i:32 * i + 32].split(b"\0")[0].decode(), float(ms[i])) for i in range(n.value)]


def workspace_bytes(B, heads, T, Hs, Ws, d, iters, recompute, elem_bytes) -> int:
    return int(lib().vmonarch_workspace_bytes(B, heads, T, Hs, Ws, d, iters, int(bool(recompute)), elem_bytes))


def set_workspace(t) -> None:
    """Hand a uint8 CUDA tensor to the library as scratch (None returns to the internal arena)."""
    if t is None:
        _check(lib().vmonarch_set_workspace(None, 0))
    else:
        _check(lib().vmonarch_set_workspace(_ptr(t), t.numel() * t.element_size()))


def shutdown() -> None:
    _check(lib().vmonarch_shutdown())


def attention(q, k, v, T, Hs, Ws, iters=2, recompute=True, out=None):
    """q, k, v: [B, heads, N, d] bf16 or f32 CUDA tensors -> out of the same shape.
    recompute: False / 0 none, True / 1 first-frame recomputation, 2 sink averaging."""
    B, heads, N, d = q.shape
    assert N == T * Hs * Ws and k.shape == q.shape and v.shape == q.shape
    if out is None:
        out = torch.empty_like(q)
    fn = getattr(lib(), "vmonarch_attention" + _suffix(q))
    _check(fn(_ptr(q), _ptr(k), _ptr(v), _ptr(out), B, heads, T, Hs, Ws, d, iters, int(recompute), _stream()))
    return out


def default_options() -> Options:
    """A vmonarch_options filled with the library's defaults."""
    o = Options()
    _check(lib().vmonarch_options_init(ctypes.byref(o)))
    return o


def attention_ex(q, k, v, T, Hs, Ws, iters, recompute, options: Options, out=None, workspace=None):
    """attention() with the settings (and optionally the workspace tensor) carried by this call."""
    B, heads, N, d = q.shape
    assert N == T * Hs * Ws and k.shape == q.shape and v.shape == q.shape
    if out is None:
        out = torch.empty_like(q)
    if workspace is not None:
        options.workspace = workspace.data_ptr()
        options.workspace_bytes = workspace.numel() * workspace.element_size()
    fn = getattr(lib(), "vmonarch_attention_ex" + _suffix(q))
    _check(fn(_ptr(q), _ptr(k), _ptr(v), _ptr(out), B, heads, T, Hs, Ws, d, iters, int(recompute),
              ctypes.byref(options), _stream()))
    return out


def r_update(aR, cR, k, v, T, Hs, Ws, row_scale, cr_min):
    """Returns (aL, cL, y or None); layouts [B, heads, T*b, d] and [B, heads, T*b]."""
    B, heads, N, d = aR.shape
    aL = torch.empty_like(aR)
    cL = torch.empty((B, heads, N), dtype=torch.float32, device=aR.device)
    y = torch.empty_like(aR) if v is not None else None
    fn = getattr(lib(), "vmonarch_r_update" + _suffix(aR))
    _check(fn(_ptr(aR), _ptr(cR), _ptr(k), _ptr(v), _ptr(aL), _ptr(cL), _ptr(y), B, heads, T, Hs, Ws, d,
              c_float(row_scale), c_float(cr_min), _stream()))
    return aL, cL, y


def r_update_lse(aR, cR, k, v, T, Hs, Ws, row_scale, cr_min):
    """Like r_update; returns (aL, cL, y or None, lse) with lse [B, heads, T*b] float32."""
    B, heads, N, d = aR.shape
    aL = torch.empty_like(aR)
    cL = torch.empty((B, heads, N), dtype=torch.float32, device=aR.device)
    lse = torch.empty((B, heads, N), dtype=torch.float32, device=aR.device)
    y = torch.empty_like(aR) if v is not None else None
    fn = getattr(lib(), "vmonarch_r_update_lse" + _suffix(aR))
    _check(fn(_ptr(aR), _ptr(cR), _ptr(k), _ptr(v), _ptr(aL), _ptr(cL), _ptr(y), _ptr(lse), B, heads, T, Hs, Ws, d,
              c_float(row_scale), c_float(cr_min), _stream()))
    return aL, cL, y, lse


def l_update(q, aL, cL, y, T, Hs, Ws, q_scale):
    """Fitting sweep (y None): returns (aR, cR).  Last sweep (y given): returns out."""
    B, heads, N, d = q.shape
    fn = getattr(lib(), "vmonarch_l_update" + _suffix(q))
    if y is None:
        aR = torch.empty_like(q)
        cR = torch.empty((B, heads, N), dtype=torch.float32, device=q.device)
        _check(fn(_ptr(q), _ptr(aL), _ptr(cL), None, _ptr(aR), _ptr(cR), None, B, heads, T, Hs, Ws, d,
                  c_float(q_scale), _stream()))
        return aR, cR
    out = torch.empty_like(q)
    _check(fn(_ptr(q), _ptr(aL), _ptr(cL), _ptr(y), None, None, _ptr(out), B, heads, T, Hs, Ws, d,
              c_float(q_scale), _stream()))
    return out


def first_frame_attention(q, k, v, T, Hs, Ws, out):
    """Overwrites rows 0..b-1 of every head of `out` with exact attention over all keys."""
    B, heads, N, d = q.shape
    fn = getattr(lib(), "vmonarch_first_frame_attention" + _suffix(q))
    _check(fn(_ptr(q), _ptr(k), _ptr(v), _ptr(out), B, heads, T, Hs, Ws, d, _stream()))
    return out


def recompute_rows(q, k, v, T, Hs, Ws, out, row_begin, row_count):
    """Overwrites rows [row_begin, row_begin + row_count) of every head of `out` with exact attention over all keys."""
    B, heads, N, d = q.shape
    fn = getattr(lib(), "vmonarch_recompute_rows" + _suffix(q))
    _check(fn(_ptr(q), _ptr(k), _ptr(v), _ptr(out), B, heads, T, Hs, Ws, d, row_begin, row_count, _stream()))
    return out


def set_flash_variant(variant: int):
    _check(lib().vmonarch_set_flash_variant(int(variant)))


def get_flash_variant() -> int:
    return int(lib().vmonarch_get_flash_variant())


def recompute_tokens(q, k, v, T, Hs, Ws, out, rows):
    """Overwrites the rows listed in `rows` (int32 CUDA tensor, row numbers within a head) of every head of `out`
    with exact attention over all keys."""
    B, heads, N, d = q.shape
    assert rows.dtype == torch.int32 and rows.is_cuda and rows.is_contiguous()
    fn = getattr(lib(), "vmonarch_recompute_tokens" + _suffix(q))
    _check(fn(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(rows), rows.numel(), B, heads, T, Hs, Ws, d, _stream()))
    return out


def recompute_rows_noalloc(q, k, v, T, Hs, Ws, out, row_begin, row_count):
    """recompute_rows (bf16) through the entry point that allocates no device memory."""
    B, heads, N, d = q.shape
    assert q.dtype == torch.bfloat16
    _check(lib().vmonarch_recompute_rows_noalloc(_ptr(q), _ptr(k), _ptr(v), _ptr(out), B, heads, T, Hs, Ws, d,
                                                 row_begin, row_count, _stream()))
    return out


def sink_average(q, k, v, T, Hs, Ws, out):
    """out <- (out + softmax(q K_F1^T / sqrt(d)) V_F1) / 2 in place."""
    B, heads, N, d = q.shape
    fn = getattr(lib(), "vmonarch_sink_average" + _suffix(q))
    _check(fn(_ptr(q), _ptr(k), _ptr(v), _ptr(out), B, heads, T, Hs, Ws, d, _stream()))
    return out


def first_frame_attention_lse(q, k, v, T, Hs, Ws, out):
    """Like first_frame_attention; also returns lse [B, heads, T*b] float32 (frame-0 entries written)."""
    B, heads, N, d = q.shape
    lse = torch.zeros((B, heads, N), dtype=torch.float32, device=q.device)
    fn = getattr(lib(), "vmonarch_first_frame_attention_lse" + _suffix(q))
    _check(fn(_ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(lse), B, heads, T, Hs, Ws, d, _stream()))
    return out, lse


def entropy_attention_bwd(q, cR, k, v, o, dO, lse, H, dH, T, Hs, Ws, row_scale, cr_min):
    """Alg. 2: returns (dq, dk, dv) for the batch of per-frame softmax blocks; dH may be None."""
    B, heads, N, d = q.shape
    dq, dk, dv = torch.empty_like(q), torch.empty_like(q), torch.empty_like(q)
    fn = getattr(lib(), "vmonarch_entropy_attention_bwd" + _suffix(q))
    _check(fn(_ptr(q), _ptr(cR), _ptr(k), _ptr(v), _ptr(o), _ptr(dO), _ptr(lse), _ptr(H), _ptr(dH), _ptr(dq), _ptr(dk),
              _ptr(dv), B, heads, T, Hs, Ws, d, c_float(row_scale), c_float(cr_min), _stream()))
    return dq, dk, dv


def mfma_probe(operands, blocks, iters):
    """Launches the matrix-instruction probe on `operands` (uint8/bf16 device tensor of blocks*512*128 bytes);
    returns (out tensor, floating-point operations of the launch)."""
    assert operands.numel() * operands.element_size() >= blocks * 512 * 128
    out = torch.empty(blocks * 512, dtype=torch.float32, device=operands.device)
    fl = ctypes.c_double(0.0)
    _check(lib().vmonarch_mfma_probe(_ptr(operands), _ptr(out), blocks, iters, ctypes.byref(fl), _stream()))
    return out, fl.value


def index_maps(T, Hs, Ws):
    """(perm, inv) as int32 CPU tensors."""
    N = T * Hs * Ws
    perm = torch.empty(N, dtype=torch.int32)
    inv = torch.empty(N, dtype=torch.int32)
    _check(lib().vmonarch_index_maps(T, Hs, Ws, c_void_p(perm.data_ptr()), c_void_p(inv.data_ptr())))
    return perm, inv


def permute_tokens(x, T, Hs, Ws, to_position_major=True, out=None):
    B, heads, N, d = x.shape
    if out is None:
        out = torch.empty_like(x)
    _check(lib().vmonarch_permute_tokens(_ptr(x), _ptr(out), B, heads, T, Hs, Ws, d * x.element_size(),
                                         int(bool(to_position_major)), _stream()))
    return out

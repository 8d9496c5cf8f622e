"""The C-ABI library loads and exports every symbol the public header declares (no GPU needed)."""
import ctypes
import os
import re

import numpy as np

from oracle import vmonarch_oracle as O

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    names = set()
    inc = os.path.join(ROOT, "include")
    for f in sorted(os.listdir(inc)):
        if not f.endswith(".h"):
            continue
        text = open(os.path.join(inc, f)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(vmonarch_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    from paper_2601_22275_amd import binding
    lib = binding.lib()
    names = _declared()
    assert len(names) >= 19
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names
    assert binding.version() >= 100


def test_host_only_entry_points():
    from paper_2601_22275_amd import binding
    perm, inv = binding.index_maps(21, 3, 5)
    operm, oinv = O.index_maps(21, 15)
    assert np.array_equal(perm.numpy(), operm) and np.array_equal(inv.numpy(), oinv)
    lib = binding.lib()
    assert lib.vmonarch_index_maps(0, 3, 5, None, None) == -1
    assert binding.workspace_bytes(1, 12, 81, 28, 52, 128, 2, True, 2) > 3 * 12 * 117936 * 128 * 2
    assert binding.workspace_bytes(1, 12, 81, 28, 52, 128, 0, True, 2) == 0
    assert lib.vmonarch_set_cr_min(ctypes.c_float(-1.0)) == -1
    assert b"cr_min" in lib.vmonarch_last_error()
    # per-call options: defaults, and validation without a GPU (nothing is launched on a bad field)
    o = binding.default_options()
    assert o.struct_bytes == ctypes.sizeof(binding.Options) and abs(o.cr_min - 0.1) < 1e-7
    assert (o.entropy_mode, o.fused_apply, o.flash_variant, o.cr_control, o.cl_control) == (0, 1, 2, 0, 0)
    assert o.cl_value != o.cl_value and not o.workspace and o.workspace_bytes == 0
    one = ctypes.c_void_p(256)   # never dereferenced: validation fails first
    o.entropy_mode = 7
    assert lib.vmonarch_attention_ex(one, one, one, ctypes.c_void_p(512), 1, 1, 2, 2, 2, 64, 1, 0, ctypes.byref(o), None) == -1
    assert b"entropy_mode" in lib.vmonarch_last_error()
    o = binding.default_options()
    o.struct_bytes = 8
    assert lib.vmonarch_attention_ex(one, one, one, ctypes.c_void_p(512), 1, 1, 2, 2, 2, 64, 1, 0, ctypes.byref(o), None) == -1
    assert lib.vmonarch_attention_ex(one, one, one, ctypes.c_void_p(512), 1, 1, 2, 2, 2, 64, 1, 0, None, None) == -1


def test_workspace_size_follows_the_documented_layout():
    """alpha_L, y and c_L always; alpha_R and c_R from the second sweep on; first-frame partials when the MFMA path
    recomputes; 256-byte granules; monotone in every argument that adds a buffer."""
    from paper_2601_22275_amd import binding
    B, heads, T, Hs, Ws, d = 1, 12, 81, 28, 52, 128
    N = T * Hs * Ws
    up = lambda x: (x + 255) // 256 * 256
    tok, sca = up(B * heads * N * d * 2), up(B * heads * N * 4)
    one = binding.workspace_bytes(B, heads, T, Hs, Ws, d, 1, False, 2)
    two = binding.workspace_bytes(B, heads, T, Hs, Ws, d, 2, False, 2)
    three = binding.workspace_bytes(B, heads, T, Hs, Ws, d, 3, False, 2)
    rec = binding.workspace_bytes(B, heads, T, Hs, Ws, d, 2, True, 2)
    assert one == 2 * tok + sca                       # alpha_L, y, c_L
    assert two == 3 * tok + 2 * sca                   # + alpha_R, c_R
    assert three == two                               # further sweeps reuse them
    assert rec > two and (rec - two) % 256 == 0       # + partial outputs and log-sum-exps of the key ranges
    assert rec - two >= heads * Hs * Ws * (4 * d + 4) * 2   # at least two key ranges at this length
    # fp32 tensors are twice as large; the plain-ALU recomputation needs no partials
    f32 = binding.workspace_bytes(B, heads, T, Hs, Ws, d, 2, True, 4)
    assert f32 == 3 * up(B * heads * N * d * 4) + 2 * sca
    # more than 128 frames: the temporal factor's fitting form takes two passes and keeps one float per token
    long_t = binding.workspace_bytes(1, 2, 260, 4, 8, 64, 2, False, 2)
    n2 = 260 * 32
    assert long_t == 3 * up(2 * n2 * 64 * 2) + 3 * up(2 * n2 * 4)
    assert binding.workspace_bytes(1, 2, 260, 4, 8, 64, 1, False, 2) == 2 * up(2 * n2 * 64 * 2) + up(2 * n2 * 4)


def test_size_limits_and_setters_are_validated_on_the_host():
    from paper_2601_22275_amd import binding
    lib = binding.lib()
    wb = binding.workspace_bytes
    assert wb(1, 1, 1, 1, 1, 256, 1, False, 2) > 0 and wb(1, 1, 1, 1, 1, 257, 1, False, 2) == 0      # d <= 256
    assert wb(1, 65535, 1, 1, 1, 8, 1, False, 2) > 0 and wb(2, 32768, 1, 1, 1, 8, 1, False, 2) == 0  # B * heads <= 65535
    assert wb(1, 1, 65535, 1, 1, 8, 1, False, 2) > 0 and wb(1, 1, 65536, 1, 1, 8, 1, False, 2) == 0  # T <= 65535
    assert wb(1, 1, 2, 32768, 32767, 8, 1, False, 2) > 0                                             # N = 2^31 - 65536
    assert wb(1, 1, 2, 32768, 32768, 8, 1, False, 2) == 0                                            # N = 2^31
    assert wb(1, 1, 4, 4, 4, 8, 1, False, 3) == 0 and wb(0, 1, 4, 4, 4, 8, 1, False, 2) == 0
    for bad in (-1, 3):
        assert lib.vmonarch_set_flash_variant(bad) == -1 and b"flash variant" in lib.vmonarch_last_error()
    assert binding.get_flash_variant() == 2
    for v in (0, 1, 2):
        binding.set_flash_variant(v)
        assert binding.get_flash_variant() == v
    assert lib.vmonarch_set_entropy_mode(5) == -1
    assert lib.vmonarch_set_manual_control(3, 0, ctypes.c_float(0.0)) == -1
    assert lib.vmonarch_set_workspace(ctypes.c_void_p(256), 0) == -1          # pointer without size
    assert lib.vmonarch_set_workspace(ctypes.c_void_p(100), 1024) == -1       # not 256-byte aligned
    assert b"aligned" in lib.vmonarch_last_error()
    assert lib.vmonarch_set_workspace(None, 0) == 0
    o = binding.default_options()
    o.flash_variant = 3
    one = ctypes.c_void_p(256)
    assert lib.vmonarch_attention_ex(one, one, one, ctypes.c_void_p(512), 1, 1, 2, 2, 2, 64, 1, 0, ctypes.byref(o), None) == -1
    assert b"flash_variant" in lib.vmonarch_last_error()

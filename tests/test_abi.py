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

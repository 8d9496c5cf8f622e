"""GPU parity of the ablation variants (sink averaging, Sec. 4.4; manual control of c_R / c_L, App. "Manual Control
of Monarch Parameters") against the CPU oracle, through the C ABI."""
import math

import numpy as np
import pytest

from oracle import vmonarch_oracle as O
from tests import util as U

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    from paper_2601_22275_amd import binding
    assert torch.cuda.is_available()
    binding.lib()
    return torch, binding, torch.device("cuda:0")


def _tol(bf16):
    return (U.BF16_REL_L2, U.BF16_MAX_ABS) if bf16 else (1e-4, 1e-4)


SHAPES = [
    # T, Hs, Ws, d, dtype
    (4, 4, 4, 32, "f32"),
    (5, 4, 6, 96, "bf16"),       # plain-ALU bf16
    (7, 9, 11, 64, "bf16"),      # MFMA d = 64, b = 99
    (21, 12, 13, 128, "bf16"),   # MFMA d = 128, b = 156, N = 3276: ragged last query block
    (3, 17, 19, 128, "bf16"),    # b = 323: several key tiles with a ragged tail
]


@pytest.mark.parametrize("T,Hs,Ws,d,dt", SHAPES)
def test_sink_average_variant_matches_oracle(env, T, Hs, Ws, d, dt):
    torch, binding, dev = env
    bf16 = dt == "bf16"
    b, heads = Hs * Ws, 2
    data = U.structured_heads(T, Hs, Ws, d, 31, heads, bf16)
    tq, tk, tv = (U.to_device([h[i] for h in data], torch, dev) for i in range(3))
    got = U.from_device(binding.attention(tq, tk, tv, T, Hs, Ws, 2, binding_mode(binding, "sink")))
    # the two-call form gives the same bytes: plain path, then the in-place averaging pass
    two = binding.attention(tq, tk, tv, T, Hs, Ws, 2, False)
    binding.sink_average(tq, tk, tv, T, Hs, Ws, two)
    assert np.array_equal(got, U.from_device(two))
    rel_tol, abs_tol = _tol(bf16)
    for h in range(heads):
        q64, k64, v64 = (U.to_f64(x) for x in data[h])
        ref = O.monarch_attention(q64, k64, v64, T, b, 2, sink_average=True)["O"].reshape(T * b, d)
        print(f"sink T={T} b={b} d={d} {dt}: rel {U.rel_l2(got[h], ref):.2e} max {U.max_abs(got[h], ref):.2e}")
        assert U.rel_l2(got[h], ref) <= rel_tol and U.max_abs(got[h], ref) <= abs_tol


def binding_mode(binding, name):
    return {"none": 0, "first_frame": 1, "sink": 2}[name]


@pytest.mark.parametrize("T,Hs,Ws,d,dt", [(4, 4, 4, 32, "f32"), (6, 9, 11, 128, "bf16"), (5, 4, 6, 96, "bf16")])
def test_sink_average_pass_alone(env, T, Hs, Ws, d, dt):
    """The averaging pass on a known `out`: (out + softmax(Q K_F1^T / sqrt(d)) V_F1) / 2, every row."""
    torch, binding, dev = env
    bf16 = dt == "bf16"
    b, heads = Hs * Ws, 2
    data = U.structured_heads(T, Hs, Ws, d, 32, heads, bf16)
    tq, tk, tv = (U.to_device([h[i] for h in data], torch, dev) for i in range(3))
    rng = np.random.default_rng(7)
    prior = [U.random_bits(rng, (T * b, d), 1.0, bf16) for _ in range(heads)]
    out = U.to_device(prior, torch, dev)
    binding.sink_average(tq, tk, tv, T, Hs, Ws, out)
    got = U.from_device(out)
    rel_tol, abs_tol = _tol(bf16)
    for h in range(heads):
        q64, k64, v64 = (U.to_f64(x) for x in data[h])
        ref = 0.5 * (U.to_f64(prior[h]) + O.softmax_attention(q64, k64[:b], v64[:b], 1.0 / math.sqrt(d)))
        assert U.rel_l2(got[h], ref) <= rel_tol and U.max_abs(got[h], ref) <= abs_tol


CONTROL = [
    # iters, cr_control, cl_control, cl_value (None: the default -log b)
    (1, 0, 1, None),
    (1, 2, 2, None),
    (2, 1, 0, None),
    (2, 2, 0, None),
    (2, 0, 1, None),
    (2, 1, 1, -2.5),
    (2, 2, 2, 0.7),
    (3, 1, 1, None),
]


@pytest.mark.parametrize("iters,cr_control,cl_control,cl_value", CONTROL)
@pytest.mark.parametrize("T,Hs,Ws,d,dt", [(4, 4, 4, 32, "f32"), (9, 9, 11, 128, "bf16"), (5, 5, 7, 64, "bf16")])
def test_manual_control_matches_oracle(env, T, Hs, Ws, d, dt, iters, cr_control, cl_control, cl_value):
    torch, binding, dev = env
    bf16 = dt == "bf16"
    b, heads = Hs * Ws, 2
    data = U.structured_heads(T, Hs, Ws, d, 33, heads, bf16)
    tq, tk, tv = (U.to_device([h[i] for h in data], torch, dev) for i in range(3))
    assert binding.get_manual_control()[:2] == (0, 0)
    binding.set_manual_control(cr_control, cl_control, float("nan") if cl_value is None else cl_value)
    try:
        got = U.from_device(binding.attention(tq, tk, tv, T, Hs, Ws, iters, True))
    finally:
        binding.set_manual_control()
    plain = U.from_device(binding.attention(tq, tk, tv, T, Hs, Ws, iters, True))
    rel_tol, abs_tol = _tol(bf16)
    for h in range(heads):
        q64, k64, v64 = (U.to_f64(x) for x in data[h])
        res = O.monarch_attention(q64, k64, v64, T, b, iters, recompute=True, cr_control=cr_control,
                                  cl_control=cl_control, cl_value=cl_value, keep_factors=True)
        ref = res["O"].reshape(T * b, d)
        free = O.monarch_attention(q64, k64, v64, T, b, iters, recompute=True)["O"].reshape(T * b, d)
        ok, ratio = U.within_end_to_end_bound(got[h], res, abs_tol, bf16, (q64 / math.sqrt(d)).reshape(T, b, d))
        print(f"control T={T} b={b} d={d} {dt} t={iters} cR{cr_control} cL{cl_control}: rel {U.rel_l2(got[h], ref):.2e} "
              f"max {U.max_abs(got[h], ref):.2e} worst/bound {ratio:.2f}; variant vs plain {U.rel_l2(ref, free):.2e}")
        assert U.rel_l2(got[h], ref) <= rel_tol and ok
        # the setting is off again: the plain call matches the plain oracle
        assert U.rel_l2(plain[h], free) <= rel_tol


def test_variant_arguments_are_validated(env):
    torch, binding, dev = env
    x = torch.zeros(1, 1, 8, 16, device=dev)
    with pytest.raises(binding.VMonarchError):
        binding.attention(x, x, x, 2, 2, 2, 1, 3)
    with pytest.raises(binding.VMonarchError):
        binding.set_manual_control(3, 0)
    with pytest.raises(binding.VMonarchError):
        binding.set_manual_control(0, 1, float("inf"))
    with pytest.raises(binding.VMonarchError):
        binding.sink_average(x, x, x, 2, 2, 2, x)
    assert binding.get_manual_control()[:2] == (0, 0)


def test_per_call_options_on_two_streams(env):
    """vmonarch_attention_ex: two calls with different settings and their own workspaces, enqueued back to back on
    two streams (several rounds, so that they overlap in time), each against its own variant of the oracle; the
    process-wide settings stay untouched."""
    torch, binding, dev = env
    T, Hs, Ws, d, heads, iters = 9, 9, 11, 128, 2, 2
    b = Hs * Ws
    data = U.structured_heads(T, Hs, Ws, d, 35, heads, True)
    tq, tk, tv = (U.to_device([h[i] for h in data], torch, dev) for i in range(3))
    opt_a = binding.default_options()                      # plain: clamp 0.1, online entropy, first-frame recomputation
    opt_b = binding.default_options()                      # manual control of both terms, no clamp, other kernels
    opt_b.cr_control, opt_b.cl_control, opt_b.cl_value = 1, 1, -2.5
    opt_b.cr_min = 0.0
    opt_b.entropy_mode = binding.ENTROPY_IDENTITY
    opt_b.flash_variant = 1
    nbytes = binding.workspace_bytes(1, heads, T, Hs, Ws, d, iters, True, 2)
    ws_a = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    ws_b = torch.empty(nbytes, dtype=torch.uint8, device=dev)
    out_a, out_b = torch.empty_like(tq), torch.empty_like(tq)
    s_a, s_b = torch.cuda.Stream(), torch.cuda.Stream()
    torch.cuda.synchronize()
    for _ in range(4):
        with torch.cuda.stream(s_a):
            binding.attention_ex(tq, tk, tv, T, Hs, Ws, iters, True, opt_a, out=out_a, workspace=ws_a)
        with torch.cuda.stream(s_b):
            binding.attention_ex(tq, tk, tv, T, Hs, Ws, iters, False, opt_b, out=out_b, workspace=ws_b)
    torch.cuda.synchronize()
    assert binding.get_manual_control()[:2] == (0, 0) and binding.get_cr_min() == pytest.approx(0.1)
    got_a, got_b = U.from_device(out_a), U.from_device(out_b)
    for h in range(heads):
        q64, k64, v64 = (U.to_f64(x) for x in data[h])
        res_a = O.monarch_attention(q64, k64, v64, T, b, iters, recompute=True, keep_factors=True)
        res_b = O.monarch_attention(q64, k64, v64, T, b, iters, recompute=False, cr_min=0.0, cr_control=1, cl_control=1,
                                    cl_value=-2.5, keep_factors=True)
        qs = (q64 / math.sqrt(d)).reshape(T, b, d)
        for tag, got, res, rec in (("plain", got_a[h], res_a, True), ("controlled", got_b[h], res_b, False)):
            ref = res["O"].reshape(T * b, d)
            ok, ratio = U.within_end_to_end_bound(got, res, U.BF16_MAX_ABS, True, qs, recomputed_frame=rec)
            print(f"options {tag} head {h}: rel {U.rel_l2(got, ref):.2e} max {U.max_abs(got, ref):.2e} worst/bound {ratio:.2f}")
            assert U.rel_l2(got, ref) <= U.BF16_REL_L2 and ok
        assert U.rel_l2(res_a["O"], res_b["O"]) > 5e-2      # the two settings really differ
    # a workspace that is too small is refused before anything is launched
    opt_a.workspace_bytes = 256
    with pytest.raises(binding.VMonarchError):
        binding.attention_ex(tq, tk, tv, T, Hs, Ws, iters, True, opt_a)

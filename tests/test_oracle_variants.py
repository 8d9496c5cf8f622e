"""Pins of the oracle's ablation variants: sink averaging (Sec. 4.4) and manual control of c_R / c_L
(App. "Manual Control of Monarch Parameters").  Each is a property the paper's table or the mathematics
fixes, not a restatement of the oracle's code."""
import math

import numpy as np
import pytest

from oracle import vmonarch_oracle as O


def _qkv(m, b, d, seed, gain=1.5):
    rng = np.random.default_rng(seed)
    return tuple(gain * rng.normal(size=(m * b, d)) for _ in range(2)) + (rng.normal(size=(m * b, d)),)


@pytest.mark.parametrize("cl_control", [0, 1, 2])
def test_one_sweep_ignores_cr_control(cl_control):
    # the paper's control table: with one iteration the rows that differ only in the c_R strategy are identical
    Q, K, V = _qkv(5, 6, 8, 1)
    base = O.monarch_attention(Q, K, V, 5, 6, 1, cl_control=cl_control)["O"]
    for cr_control in (1, 2):
        got = O.monarch_attention(Q, K, V, 5, 6, 1, cr_control=cr_control, cl_control=cl_control)["O"]
        assert np.array_equal(got, base)


def test_two_sweeps_do_depend_on_cr_control():
    Q, K, V = _qkv(5, 6, 8, 2)
    base = O.monarch_attention(Q, K, V, 5, 6, 2)["O"]
    for cr_control in (1, 2):
        assert np.abs(O.monarch_attention(Q, K, V, 5, 6, 2, cr_control=cr_control)["O"] - base).max() > 1e-4


@pytest.mark.parametrize("iters", [1, 2, 3])
def test_cl_fixed_everywhere_is_independent_of_the_constant(iters):
    # the temporal softmax runs over key frames: a shift common to all of them cancels
    Q, K, V = _qkv(4, 7, 8, 3)
    a = O.monarch_attention(Q, K, V, 4, 7, iters, cl_control=2, cl_value=-1.3)["O"]
    c = O.monarch_attention(Q, K, V, 4, 7, iters, cl_control=2, cl_value=+4.0)["O"]
    dflt = O.monarch_attention(Q, K, V, 4, 7, iters, cl_control=2)["O"]
    assert np.allclose(a, c, atol=1e-12) and np.allclose(a, dflt, atol=1e-12)
    assert np.abs(a - O.monarch_attention(Q, K, V, 4, 7, iters)["O"]).max() > 1e-4


def test_default_cl_constant_is_the_uniform_row_value():
    m, b, d = 3, 5, 4
    Q, K, V = _qkv(m, b, d, 4)
    K0 = np.zeros_like(K)          # zero keys: every R row is uniform, c_L = -log b on its own
    free = O.monarch_attention(Q, K0, V, m, b, 1)
    assert np.allclose(free["cL"], -math.log(b), atol=1e-12)
    fixed = O.monarch_attention(Q, K0, V, m, b, 1, cl_control=1)
    assert np.allclose(fixed["O"], free["O"], atol=1e-12)


def test_very_negative_first_frame_cl_collapses_to_frame0_spatial_attention():
    # -c_L enters the temporal logits: c_L[., k=0] -> -inf puts all temporal mass on key frame 0, so every query
    # (j, i) returns y[0, i] = softmax(Q[0, i] K_F1^T / sqrt(d)) V_F1 (one sweep: alpha_R is still Q / sqrt(d))
    m, b, d = 4, 6, 8
    Q, K, V = _qkv(m, b, d, 5)
    got = O.monarch_attention(Q, K, V, m, b, 1, cl_control=1, cl_value=-1e4)["O"]
    z = Q[:b] @ K[:b].T / math.sqrt(d)
    p = np.exp(z - z.max(axis=1, keepdims=True))
    ref = (p / p.sum(axis=1, keepdims=True)) @ V[:b]
    for j in range(m):
        assert np.allclose(got[j], ref, atol=1e-10)
    # and a very positive one removes frame 0 from every temporal row: V of frame 0 no longer matters
    V2 = V.copy()
    V2[:b] += 3.0
    a = O.monarch_attention(Q, K, V, m, b, 2, cl_control=1, cl_value=1e4)["O"]
    c = O.monarch_attention(Q, K, V2, m, b, 2, cl_control=1, cl_value=1e4)["O"]
    assert np.allclose(a, c, atol=1e-10)


def test_cr_first_frame_control_leaves_other_frames_alone():
    m, b, d = 4, 6, 8
    Q, K, V = _qkv(m, b, d, 6)
    free = O.monarch_attention(Q, K, V, m, b, 2, keep_factors=True)
    ctl = O.monarch_attention(Q, K, V, m, b, 2, cr_control=1, keep_factors=True)
    assert np.array_equal(ctl["trace"][0]["aR"], free["trace"][0]["aR"])
    assert np.all(ctl["trace"][0]["cR"][0] == 1.0)
    assert np.array_equal(ctl["trace"][0]["cR"][1:], free["trace"][0]["cR"][1:])
    assert np.array_equal(ctl["R"][1:], free["R"][1:])            # R_k depends on alpha_R[k], c_R[k] only
    assert np.abs(ctl["R"][0] - free["R"][0]).max() > 1e-6
    # frame 0's factor is the untempered softmax of alpha_R[0] K_0^T
    z = ctl["trace"][0]["aR"][0] @ K[:b].T
    p = np.exp(z - z.max(axis=1, keepdims=True))
    assert np.allclose(ctl["R"][0], p / p.sum(axis=1, keepdims=True), atol=1e-12)
    allc = O.monarch_attention(Q, K, V, m, b, 3, cr_control=2)
    assert all(np.all(t["cR"] == 1.0) for t in allc["trace"])


def test_sink_average_single_frame_is_textbook_attention():
    b, d = 9, 8
    Q, K, V = _qkv(1, b, d, 7)
    got = O.monarch_attention(Q, K, V, 1, b, 2, sink_average=True)["O"][0]
    z = Q @ K.T / math.sqrt(d)
    p = np.exp(z - z.max(axis=1, keepdims=True))
    assert np.allclose(got, (p / p.sum(axis=1, keepdims=True)) @ V, atol=1e-12)


def test_sink_average_is_half_monarch_plus_half_first_frame_term():
    m, b, d = 4, 5, 8
    Q, K, V = _qkv(m, b, d, 8)
    rng = np.random.default_rng(9)
    dV = rng.normal(size=V.shape)
    dV[:b] = 0.0                                       # the sink term sees V_F1 only
    mon = lambda v: O.monarch_attention(Q, K, v, m, b, 2)["O"]
    snk = lambda v: O.monarch_attention(Q, K, v, m, b, 2, sink_average=True)["O"]
    assert np.allclose(snk(V + dV) - snk(V), 0.5 * (mon(V + dV) - mon(V)), atol=1e-12)
    # constant values stay constant, and V_F1 = const c with V = 0 elsewhere bounds the sink share from below by c/2
    assert np.allclose(snk(np.ones_like(V)), 1.0, atol=1e-12)
    V0 = np.zeros_like(V); V0[:b] = 2.0
    assert np.all(snk(V0) >= 1.0 - 1e-12) and np.all(snk(V0) <= 2.0 + 1e-12)
    # keys of later frames do not enter the sink term
    V1 = np.zeros_like(V); V1[:b] = rng.normal(size=(b, d))
    K2 = K.copy(); K2[b:] = rng.normal(size=K2[b:].shape)
    s1 = snk(V1) - 0.5 * mon(V1)
    s2 = O.monarch_attention(Q, K2, V1, m, b, 2, sink_average=True)["O"] - 0.5 * O.monarch_attention(Q, K2, V1, m, b, 2)["O"]
    assert np.allclose(s1, s2, atol=1e-12)

"""GPU parity of the Alg. 2 backward (through the C ABI) against the CPU oracle."""
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


CASES = [
    # T, Hs, Ws, d, dtype, with_dH, with_cR
    (2, 3, 5, 8, "f32", True, True),
    (3, 4, 4, 32, "f32", False, False),
    (1, 9, 11, 20, "f32", True, False),     # b = 99: two key chunks, ragged
    (2, 1, 1, 16, "f32", True, True),       # one key: no logit gradient
    (2, 8, 9, 96, "bf16", True, True),      # plain-ALU bf16 (d not 64 or 128)
    (2, 8, 9, 64, "bf16", True, True),      # MFMA, d = 64
    (1, 13, 10, 128, "bf16", False, True),  # MFMA, b = 130
    (2, 10, 30, 128, "bf16", True, True),   # b = 300: two owner blocks, ragged last stream tile
    (1, 23, 29, 64, "bf16", True, False),   # b = 667
    (2, 1, 1, 128, "bf16", True, True),     # one key
    (1, 4, 8, 128, "bf16", True, True),     # b = 32: exactly one sub-tile
]


@pytest.mark.parametrize("T,Hs,Ws,d,dt,with_dh,with_cr", CASES)
def test_entropy_attention_backward_matches_oracle(env, T, Hs, Ws, d, dt, with_dh, with_cr):
    torch, binding, dev = env
    bf16 = dt == "bf16"
    b, heads = Hs * Ws, 2
    N = T * b
    rng = np.random.default_rng(500 + T * 31 + b)
    data = U.structured_heads(T, Hs, Ws, d, 21, heads, bf16)
    Q = [h[0] for h in data]; K = [h[1] for h in data]; V = [h[2] for h in data]
    dO = [U.random_bits(rng, (N, d), 1.0, bf16) for _ in range(heads)]
    cR = (0.3 + 1.5 * rng.random((heads, N))).astype(np.float32) if with_cr else None
    dH = rng.normal(size=(heads, N)).astype(np.float32) if with_dh else None
    row_scale, cr_min = 1.0 / math.sqrt(d), 0.1
    tq, tk, tv, tdo = (U.to_device(x, torch, dev) for x in (Q, K, V, dO))
    tcr = torch.from_numpy(cR).to(dev).view(1, heads, N) if with_cr else None
    tdh = torch.from_numpy(dH).to(dev).view(1, heads, N) if with_dh else None
    # forward results from the library itself: O = y (values V), lse, H = -cL
    _, cL, y, lse = binding.r_update_lse(tq, tcr, tk, tv, T, Hs, Ws, row_scale, cr_min)
    Hent = (-cL).contiguous()
    dq, dk, dv = binding.entropy_attention_bwd(tq, tcr, tk, tv, y, tdo, lse, Hent, tdh, T, Hs, Ws, row_scale, cr_min)
    again = binding.entropy_attention_bwd(tq, tcr, tk, tv, y, tdo, lse, Hent, tdh, T, Hs, Ws, row_scale, cr_min)
    assert all(torch.equal(a, c) for a, c in zip((dq, dk, dv), again))     # bit-reproducible
    gdq, gdk, gdv = (U.from_device(x) for x in (dq, dk, dv))
    # Alg. 2 takes O, L and H as inputs: the oracle gets the very values the kernel was given
    # (the forward pass's rounded outputs), so that the comparison isolates the backward arithmetic
    gy, glse, gH = U.from_device(y), U.from_device(lse), U.from_device(Hent)
    rel_tol = 1e-2 if bf16 else 2e-4
    for h in range(heads):
        q64, k64, v64, do64 = (U.to_f64(x[h]).reshape(T, b, d) for x in (Q, K, V, dO))
        for kf in range(T):
            c = np.maximum(cR[h].reshape(T, b)[kf].astype(np.float64), cr_min) if with_cr else np.ones(b)
            sc = row_scale / c
            Oo = gy[h].reshape(T, b, d)[kf].astype(np.float64)
            l64 = glse[h].reshape(T, b)[kf].astype(np.float64)
            H64 = gH[h].reshape(T, b)[kf].astype(np.float64)
            dh64 = dH[h].reshape(T, b)[kf].astype(np.float64) if with_dh else None
            rdq, rdk, rdv = O.entropy_attention_backward(q64[kf], k64[kf], v64[kf], Oo, do64[kf], l64, H64, dh64, sc)
            for name, got, ref in (("dq", gdq, rdq), ("dk", gdk, rdk), ("dv", gdv, rdv)):
                g = got[h].reshape(T, b, d)[kf]
                # one-key blocks have no logit gradient: both sides hold rounding noise only
                err = U.rel_l2(g, ref) if np.abs(ref).max() > 1e-4 else float(np.abs(g - ref).max()) * (rel_tol / 1e-5)
                if kf == 0:
                    print(f"bwd T={T} b={b} d={d} {dt} dH={with_dh} head {h} {name}: rel {err:.2e} |ref| {np.abs(ref).max():.2e}")
                assert err <= rel_tol, (name, err)


CHAIN_CASES = [
    # T, Hs, Ws, d, dtype, with_dH, with_cR
    (2, 5, 7, 24, "f32", True, True),
    (2, 12, 13, 64, "bf16", True, True),     # MFMA, b = 156
    (1, 20, 33, 128, "bf16", True, False),   # MFMA, b = 660: several owner blocks, ragged tail
    (2, 7, 9, 128, "bf16", False, True),
]


@pytest.mark.parametrize("T,Hs,Ws,d,dt,with_dh,with_cr", CHAIN_CASES)
def test_forward_then_backward_against_the_oracles_own_forward(env, T, Hs, Ws, d, dt, with_dh, with_cr):
    """The whole chain on each side: the library's forward feeds the library's backward, and the oracle's
    forward (the definitions, fp64) feeds the oracle's backward; no value crosses from one side to the other
    except Q, K, V, dO, dH and c_R.  With bf16 the backward sees a forward output rounded to bf16, which moves
    D = rowsum(dO o O); the tolerance is the usual 1e-2 plus the first-order effect of that rounding."""
    torch, binding, dev = env
    bf16 = dt == "bf16"
    b, heads = Hs * Ws, 2
    N = T * b
    rng = np.random.default_rng(900 + T * 17 + b)
    data = U.structured_heads(T, Hs, Ws, d, 33, heads, bf16)
    Q = [h[0] for h in data]; K = [h[1] for h in data]; V = [h[2] for h in data]
    dO = [U.random_bits(rng, (N, d), 1.0, bf16) for _ in range(heads)]
    cR = (0.3 + 1.5 * rng.random((heads, N))).astype(np.float32) if with_cr else None
    dH = rng.normal(size=(heads, N)).astype(np.float32) if with_dh else None
    row_scale, cr_min = 1.0 / math.sqrt(d), 0.1
    tq, tk, tv, tdo = (U.to_device(x, torch, dev) for x in (Q, K, V, dO))
    tcr = torch.from_numpy(cR).to(dev).view(1, heads, N) if with_cr else None
    tdh = torch.from_numpy(dH).to(dev).view(1, heads, N) if with_dh else None
    _, cL, y, lse = binding.r_update_lse(tq, tcr, tk, tv, T, Hs, Ws, row_scale, cr_min)
    dq, dk, dv = binding.entropy_attention_bwd(tq, tcr, tk, tv, y, tdo, lse, (-cL).contiguous(), tdh,
                                               T, Hs, Ws, row_scale, cr_min)
    gdq, gdk, gdv = (U.from_device(x) for x in (dq, dk, dv))
    gy, glse, gH = U.from_device(y), U.from_device(lse), -U.from_device(cL)
    rel_tol = 1e-2 if bf16 else 2e-4
    for h in range(heads):
        q64, k64, v64, do64 = (U.to_f64(x[h]).reshape(T, b, d) for x in (Q, K, V, dO))
        for kf in range(T):
            c = np.maximum(cR[h].reshape(T, b)[kf].astype(np.float64), cr_min) if with_cr else np.ones(b)
            sc = row_scale / c
            Oo, l64, H64 = O.entropy_attention(q64[kf], k64[kf], v64[kf], sc)
            # the forward halves agree first, so that a backward mismatch is the backward's
            assert U.rel_l2(gy[h].reshape(T, b, d)[kf], Oo) <= (U.BF16_REL_L2 if bf16 else 1e-5)
            assert np.abs(glse[h].reshape(T, b)[kf] - l64).max() <= (2e-2 if bf16 else 1e-4)
            assert np.abs(gH[h].reshape(T, b)[kf] - H64).max() <= (2e-2 if bf16 else 1e-4)
            dh64 = dH[h].reshape(T, b)[kf].astype(np.float64) if with_dh else None
            ref = O.entropy_attention_backward(q64[kf], k64[kf], v64[kf], Oo, do64[kf], l64, H64, dh64, sc)
            # What storing O in bf16 between the passes costs: every O_ic moves by up to 2^-9 |O_ic|, independently
            # and about uniformly, so D_i = sum_c dO_ic O_ic moves by a sum of d independent terms of standard
            # deviation <= 2^-9 |dO_ic O_ic| / sqrt(3); dD_i below is twice that sum's standard deviation.
            # dS_il = P_il (dP_il - D_i - ...) then moves by P_il dD_i, hence
            # dQ_i by sc_i dD_i (P K)_i and dK_l by sum_i sc_i dD_i P_il Q_i.  On sharp rows (small c_R) the exact
            # dS is a small difference of large terms and this is the leading error; dV does not see D.
            extra = {"dq": 0.0, "dk": 0.0, "dv": 0.0}
            if bf16:
                dD = 2.0 * 2.0 ** -9 / math.sqrt(3.0) * np.sqrt(((do64[kf] * Oo) ** 2).sum(axis=1))
                P = np.exp((q64[kf] @ k64[kf].T) * sc[:, None] - l64[:, None])
                extra["dq"] = np.linalg.norm((sc * dD)[:, None] * (P @ k64[kf])) / np.linalg.norm(ref[0])
                extra["dk"] = np.linalg.norm((P * (sc * dD)[:, None]).T @ np.abs(q64[kf])) / np.linalg.norm(ref[1])
            for name, got, r in zip(("dq", "dk", "dv"), (gdq, gdk, gdv), ref):
                err = U.rel_l2(got[h].reshape(T, b, d)[kf], r)
                tol = rel_tol + extra[name]
                if kf == 0:
                    print(f"chain T={T} b={b} d={d} {dt} head {h} {name}: rel {err:.2e} of {tol:.2e} allowed")
                assert err <= tol, (name, err, tol)


def test_backward_rejects_bad_arguments(env):
    torch, binding, dev = env
    x = torch.zeros(1, 1, 4, 8, device=dev)
    s = torch.zeros(1, 1, 4, device=dev)
    with pytest.raises(binding.VMonarchError):
        binding.entropy_attention_bwd(x, None, x, x, x, x, s, s, None, 2, 1, 2, -1.0, 0.1)

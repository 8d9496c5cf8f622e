"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element."""
import ctypes
import math

import numpy as np
import pytest

from oracle import vmonarch_oracle as O
from paper_2601_22275_amd import synth
from tests import util as U

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def env():
    import torch
    from paper_2601_22275_amd import binding
    assert torch.cuda.is_available()
    binding.lib()  # fails loudly if the HIP library is missing
    return torch, binding, torch.device("cuda:0")


def _tol(bf16):
    return (U.BF16_REL_L2, U.BF16_MAX_ABS) if bf16 else (U.F32_REL_L2, 1e-4)


# ------------------------------------------------------------------ index maps (bit exact)
@pytest.mark.parametrize("T,Hs,Ws", [(1, 1, 1), (4, 4, 4), (21, 5, 7), (81, 28, 52)])
def test_index_maps_bit_exact(env, T, Hs, Ws):
    torch, binding, dev = env
    perm, inv = binding.index_maps(T, Hs, Ws)
    operm, oinv = O.index_maps(T, Hs * Ws)
    assert np.array_equal(perm.numpy(), operm) and np.array_equal(inv.numpy(), oinv)


@pytest.mark.parametrize("T,Hs,Ws,d,dt", [(4, 3, 5, 8, "f32"), (21, 6, 7, 128, "bf16"), (5, 1, 9, 6, "bf16")])
def test_permute_tokens_bit_exact(env, T, Hs, Ws, d, dt):
    torch, binding, dev = env
    rng = np.random.default_rng(3)
    N = T * Hs * Ws
    x = U.random_bits(rng, (2, N, d), 1.0, dt == "bf16")
    tx = U.to_device(list(x), torch, dev)
    perm, inv = O.index_maps(T, Hs * Ws)
    got = binding.permute_tokens(tx, T, Hs, Ws, True)
    back = binding.permute_tokens(got, T, Hs, Ws, False)
    g = got.view(torch.int16 if dt == "bf16" else torch.int32).cpu().numpy()[0]
    ref = x.view(np.int16 if dt == "bf16" else np.int32)[:, perm, :]
    assert np.array_equal(g, ref)
    assert torch.equal(back.view(torch.uint8), tx.view(torch.uint8))


# ------------------------------------------------------------------ R-update per factor
R_CASES = [
    # T, Hs, Ws, d, dtype, with_v, with_cR
    (4, 4, 4, 32, "f32", True, True),
    (3, 5, 7, 20, "f32", False, False),
    (2, 9, 9, 96, "bf16", True, True),       # plain-ALU bf16 (d not 64 or 128)
    (3, 10, 30, 64, "bf16", True, True),     # MFMA, d = 64: ragged query block and key tile
    (2, 3, 11, 64, "bf16", False, True),     # d = 64, b = 33
    (1, 23, 29, 64, "bf16", True, False),    # d = 64, b = 667
    (1, 1, 1, 64, "bf16", True, True),       # d = 64, one key
    (3, 10, 30, 128, "bf16", True, True),    # MFMA: b = 300 = 256 + 44 (ragged query block and key tile)
    (2, 8, 8, 128, "bf16", False, False),    # MFMA: exactly one key tile
    (1, 1, 1, 128, "bf16", True, True),      # degenerate: one key
    (2, 3, 11, 128, "bf16", False, True),    # b = 33: a 32-key sub-tile plus one key
    (1, 23, 29, 128, "bf16", True, False),   # b = 667: three query blocks, 11 key tiles
]


@pytest.mark.parametrize("mode", [0, 1])
@pytest.mark.parametrize("T,Hs,Ws,d,dt,with_v,with_cr", R_CASES)
def test_r_update_matches_oracle(env, T, Hs, Ws, d, dt, with_v, with_cr, mode):
    torch, binding, dev = env
    if mode == 1 and not (dt == "bf16" and d in (64, 128)):
        pytest.skip("entropy modes differ only on the MFMA path")
    bf16 = dt == "bf16"
    b, heads = Hs * Ws, 2
    rng = np.random.default_rng(1000 + T * 7 + b)
    data = U.structured_heads(T, Hs, Ws, d, 11, heads, bf16)
    aR = [h[0] for h in data]; K = [h[1] for h in data]; V = [h[2] for h in data]
    cR = (0.03 + 2.5 * rng.random((heads, T * b))).astype(np.float32) if with_cr else None
    row_scale, cr_min = 1.0 / math.sqrt(d), 0.1
    binding.set_entropy_mode(mode)
    try:
        aL, cL, y = binding.r_update(U.to_device(aR, torch, dev), None if cR is None else torch.from_numpy(cR).to(dev).view(1, heads, -1),
                                     U.to_device(K, torch, dev), U.to_device(V, torch, dev) if with_v else None,
                                     T, Hs, Ws, row_scale, cr_min)
    finally:
        binding.set_entropy_mode(0)
    aL, cL = U.from_device(aL), U.from_device(cL)
    rel_tol, abs_tol = _tol(bf16)
    for h in range(heads):
        c = np.ones((T, b)) if cR is None else cR[h].reshape(T, b).astype(np.float64)
        oaL, ocL, R = O.r_update(U.to_f64(aR[h]).reshape(T, b, d) * row_scale, c, U.to_f64(K[h]).reshape(T, b, d), cr_min)
        ref_aL = oaL.transpose(1, 0, 2).reshape(T * b, d)
        assert U.rel_l2(aL[h], ref_aL) <= rel_tol and U.max_abs(aL[h], ref_aL) <= abs_tol
        ref_cL = ocL.T.reshape(T * b)
        # Online accumulator (mode 0) errors are ~1e-6; the identity form c_L = scale * (aR . alpha_L) - logsumexp
        # (mode 1) inherits the bf16 rounding of the weights through alpha_L and lands at a few 1e-3.
        cl_tol = 1e-4 if not bf16 else 2e-2
        print(f"r_update T={T} b={b} d={d} {dt} mode={mode}: aL rel {U.rel_l2(aL[h], ref_aL):.2e} max {U.max_abs(aL[h], ref_aL):.2e} cL max {U.max_abs(cL[h], ref_cL):.2e}")
        assert U.max_abs(cL[h], ref_cL) <= cl_tol, U.max_abs(cL[h], ref_cL)
        if with_v:
            ref_y = np.matmul(R, U.to_f64(V[h]).reshape(T, b, d)).reshape(T * b, d)
            gy = U.from_device(y)[h]
            assert U.rel_l2(gy, ref_y) <= rel_tol and U.max_abs(gy, ref_y) <= abs_tol


@pytest.fixture(params=["one-wave", "wave-pair", "two-pass"])
def fused(request, env):
    """The three forms of the bf16 MFMA R-update: one wave per SIMD with two query tiles (alpha_L, c_L and, with values,
    y from one softmax); two waves per SIMD, alpha_L, c_L and y from one pass shared by a wave pair; two waves per
    SIMD, a pass for alpha_L / c_L and a second one for y."""
    binding = env[1]
    binding.set_flash_variant(1 if request.param == "one-wave" else 0)
    binding.set_fused_apply(request.param != "two-pass")
    yield request.param
    binding.set_fused_apply(True)
    binding.set_flash_variant(2)     # the library's default: each update on the kernel measured faster for it


@pytest.mark.parametrize("d", [64, 128])
@pytest.mark.parametrize("b", [31, 32, 33, 63, 64, 65, 95, 96, 97, 127, 128, 129, 191, 192, 193, 255, 256, 257, 320, 511, 513])
def test_r_update_at_every_tile_boundary(env, b, d, fused):
    """One frame of b tokens around every boundary of the blocked kernels: 32-key sub-tiles, 64-key tiles (1 to 9
    of them: every start-up and wind-down path of the step pipelines), 32-row waves, 128- and 256-row query
    blocks, the four-tile LDS rotation."""
    torch, binding, dev = env
    rng = np.random.default_rng(9000 + 7 * b + d)
    q = U.random_bits(rng, (b, d), 1.2, True)
    k = U.random_bits(rng, (b, d), 1.2, True)
    v = U.random_bits(rng, (b, d), 1.0, True)
    cR = (0.2 + 2.0 * rng.random((1, b))).astype(np.float32)
    row_scale, cr_min = 1.0 / math.sqrt(d), 0.1
    tq, tk, tv = (U.to_device([x], torch, dev) for x in (q, k, v))
    aL, cL, y = binding.r_update(tq, torch.from_numpy(cR).to(dev).view(1, 1, -1), tk, tv, 1, 1, b, row_scale, cr_min)
    z = (U.to_f64(q) @ U.to_f64(k).T) * row_scale / np.maximum(cR[0].astype(np.float64), cr_min).reshape(-1, 1)
    R = O.softmax_rows(z)
    for name, got, ref in (("aL", aL, R @ U.to_f64(k)), ("y", y, R @ U.to_f64(v))):
        g = U.from_device(got)[0]
        assert U.rel_l2(g, ref) <= U.BF16_REL_L2 and U.max_abs(g, ref) <= U.BF16_MAX_ABS, (name, b, d)
    assert U.max_abs(U.from_device(cL)[0], O.neg_entropy_rows(R)) <= 2e-2
    if fused != "two-pass":
        # the same update without values (the fitting sweeps' form of the kernel)
        aL2, cL2, _ = binding.r_update(tq, torch.from_numpy(cR).to(dev).view(1, 1, -1), tk, None, 1, 1, b, row_scale, cr_min)
        g = U.from_device(aL2)[0]
        ref = R @ U.to_f64(k)
        assert U.rel_l2(g, ref) <= U.BF16_REL_L2 and U.max_abs(g, ref) <= U.BF16_MAX_ABS, ("aL without values", b, d)
        assert U.max_abs(U.from_device(cL2)[0], O.neg_entropy_rows(R)) <= 2e-2


@pytest.mark.parametrize("seed", range(12))
def test_r_update_random_shapes_both_forms(env, seed, fused):
    """Seeded random (T, b, d, c_R) problems: both forms of the R-update with values against the oracle."""
    torch, binding, dev = env
    rng = np.random.default_rng(4242 + seed)
    T = int(rng.integers(1, 6))
    b = int(rng.integers(1, 700))
    d = int(rng.choice([64, 128]))
    heads = 2
    with_cr = bool(rng.integers(0, 2))
    q = [U.random_bits(rng, (T * b, d), 1.3, True) for _ in range(heads)]
    k = [U.random_bits(rng, (T * b, d), 1.3, True) for _ in range(heads)]
    v = [U.random_bits(rng, (T * b, d), 1.0, True) for _ in range(heads)]
    cR = (0.05 + 2.5 * rng.random((heads, T * b))).astype(np.float32) if with_cr else None
    row_scale, cr_min = 1.0 / math.sqrt(d), 0.1
    tq, tk, tv = (U.to_device(x, torch, dev) for x in (q, k, v))
    tcr = torch.from_numpy(cR).to(dev).view(1, heads, -1) if with_cr else None
    aL, cL, y = binding.r_update(tq, tcr, tk, tv, T, 1, b, row_scale, cr_min)
    gaL, gcL, gy = U.from_device(aL), U.from_device(cL), U.from_device(y)
    for h in range(heads):
        c = cR[h].reshape(T, b).astype(np.float64) if with_cr else np.ones((T, b))
        raL, rcL, R = O.r_update(U.to_f64(q[h]).reshape(T, b, d) * row_scale, c, U.to_f64(k[h]).reshape(T, b, d), cr_min)
        k3, v3 = U.to_f64(k[h]).reshape(T, b, d), U.to_f64(v[h]).reshape(T, b, d)
        ry = np.matmul(R, v3)
        for name, g, ref, mag in (("aL", gaL[h].reshape(T, b, d), raL.transpose(1, 0, 2), np.matmul(R, np.abs(k3))),
                                  ("y", gy[h].reshape(T, b, d), ry, np.matmul(R, np.abs(v3)))):
            ratio = float((np.abs(g - ref) / U.weighted_sum_bound(ref, mag)).max())
            assert U.rel_l2(g, ref) <= U.BF16_REL_L2 and ratio <= 1.0, (name, T, b, d, with_cr, ratio)
        assert U.max_abs(gcL[h].reshape(T, b), rcL.T) <= 2e-2, (T, b, d, with_cr)


@pytest.mark.parametrize("spike", [7.0, 72.0])
@pytest.mark.parametrize("d", [64, 128])
def test_r_update_when_the_reference_max_moves_in_every_tile(env, d, fused, spike):
    """Keys with ever larger logits in later tiles, one spike key per tile, and queries that respond to the
    spikes with different strength: the kernels' reference maxima move in almost every tile, in the wave that
    produces the probabilities and in the one that adopts them, while the mass below the spikes still matters for
    many rows.  Spikes of 7 per tile raise the strongest rows' maxima by 2^8 per tile (the margin of the kernels
    with two waves per SIMD), spikes of 72 by more than 2^56 (margin plus headroom of the kernel with one)."""
    torch, binding, dev = env
    b = 600                                           # 10 key tiles, ragged; 5 query blocks of 128
    rng = np.random.default_rng(77 + d)
    qf = rng.normal(size=(b, d)) * 0.8
    kf = rng.normal(size=(b, d)) * 0.8
    qf[:, 0] = np.linspace(0.0, 9.0, b)[rng.permutation(b)]   # response of a query to the spikes
    kf[:, 0] = 0.0
    for t, l in enumerate(range(17, b, 61)):                   # one spike every 61 keys, growing
        kf[l, 0] = spike * (t + 1)
    vf = rng.normal(size=(b, d))
    q, k, v = (synth.f32_to_bf16_bits(x.astype(np.float32)) for x in (qf, kf, vf))
    row_scale, cr_min = 1.0 / math.sqrt(d), 0.1
    tq, tk, tv = (U.to_device([x], torch, dev) for x in (q, k, v))
    aL, cL, y, lse = binding.r_update_lse(tq, None, tk, tv, 1, 1, b, row_scale, cr_min)
    z = (U.to_f64(q) @ U.to_f64(k).T) * row_scale
    assert (z.max(axis=1) - np.median(z, axis=1)).max() > 40  # far more than the 2^8 threshold, for some rows
    R = O.softmax_rows(z)
    for name, got, x in (("aL", aL, U.to_f64(k)), ("y", y, U.to_f64(v))):
        g = U.from_device(got)[0]
        ref = R @ x
        # entries reach 70 here: the bound is the first-order rounding analysis of a bf16 weighted sum (one rounding
        # per weight, one of the result), the flat 2e-2 wherever that is smaller
        bound = U.weighted_sum_bound(ref, R @ np.abs(x))
        ratio = float((np.abs(g - ref) / bound).max())
        w = np.unravel_index(np.argmax(np.abs(g - ref) / bound), ref.shape)
        print(f"moving reference d={d} {name}: rel {U.rel_l2(g, ref):.2e} worst/bound {ratio:.2f} at row {w[0]} channel {w[1]}: "
              f"got {g[w]:.5f} ref {ref[w]:.5f} bound {bound[w]:.4f}")
        assert U.rel_l2(g, ref) <= U.BF16_REL_L2 and ratio <= 1.0, (name, d, ratio)
    assert U.max_abs(U.from_device(cL)[0], O.neg_entropy_rows(R)) <= 2e-2
    ref_lse = np.log(np.exp(z - z.max(axis=1, keepdims=True)).sum(axis=1)) + z.max(axis=1)
    np.testing.assert_allclose(U.from_device(lse)[0], ref_lse, rtol=2.0 ** -7, atol=2e-2)


@pytest.mark.parametrize("T,Hs,Ws,d,dt", [(4, 4, 4, 32, "f32"), (3, 10, 30, 128, "bf16"), (2, 3, 11, 64, "bf16"),
                                           (2, 9, 9, 96, "bf16")])
def test_r_update_log_sum_exp_output(env, T, Hs, Ws, d, dt):
    """lse = log sum_l exp z from the definition; the entropy identity c_L = sum_l R z - lse ties it
    to the other two outputs."""
    torch, binding, dev = env
    bf16 = dt == "bf16"
    b, heads = Hs * Ws, 2
    rng = np.random.default_rng(77)
    data = U.structured_heads(T, Hs, Ws, d, 15, heads, bf16)
    aR = [h[0] for h in data]; K = [h[1] for h in data]
    cR = (0.05 + 2.0 * rng.random((heads, T * b))).astype(np.float32)
    row_scale, cr_min = 1.0 / math.sqrt(d), 0.1
    taR, tK = U.to_device(aR, torch, dev), U.to_device(K, torch, dev)
    tcR = torch.from_numpy(cR).to(dev).view(1, heads, -1)
    aL, cL, _, lse = binding.r_update_lse(taR, tcR, tK, None, T, Hs, Ws, row_scale, cr_min)
    aL2, cL2, _ = binding.r_update(taR, tcR, tK, None, T, Hs, Ws, row_scale, cr_min)
    assert torch.equal(aL, aL2) and torch.equal(cL, cL2)      # the extra output changes nothing else
    glse, gcL, gaL = U.from_device(lse), U.from_device(cL), U.from_device(aL)
    for h in range(heads):
        a = U.to_f64(aR[h]).reshape(T, b, d)
        kk = U.to_f64(K[h]).reshape(T, b, d)
        z = np.einsum("kid,kld->kil", a, kk) * row_scale / np.maximum(cR[h].reshape(T, b, 1).astype(np.float64), cr_min)
        zmax = z.max(axis=2, keepdims=True)
        ref = (zmax[..., 0] + np.log(np.exp(z - zmax).sum(axis=2))).reshape(T * b)
        err = U.max_abs(glse[h], ref)
        print(f"r_update_lse T={T} b={b} d={d} {dt}: lse max err {err:.2e}")
        assert err <= (5e-3 if bf16 else 1e-4)
        # sum_l R_l z_l = scale / c * aR . alpha_L  (z is linear in K): c_L + lse equals it
        mean_z = (a * gaL[h].reshape(T, b, d)).sum(axis=2).reshape(T * b) * row_scale / np.maximum(cR[h], cr_min)
        # (alpha_L carries a relative bf16 rounding error, and |z| grows like 1 / c_R)
        np.testing.assert_allclose(gcL[h] + glse[h], mean_z, rtol=2.0 ** -7 if bf16 else 1e-4, atol=2e-2 if bf16 else 1e-3)


# ------------------------------------------------------------------ L-update per factor
L_CASES = [
    (4, 4, 4, 32, "f32"), (7, 1, 5, 20, "f32"), (5, 2, 3, 96, "bf16"),
    (5, 2, 3, 64, "bf16"), (21, 1, 7, 64, "bf16"), (32, 1, 5, 64, "bf16"), (81, 1, 5, 64, "bf16"), (128, 1, 2, 64, "bf16"),
    (1, 2, 3, 128, "bf16"), (21, 1, 7, 128, "bf16"), (33, 1, 3, 128, "bf16"),
    (81, 1, 5, 128, "bf16"), (128, 1, 2, 128, "bf16"),
    # more than 128 frames: the temporal factor runs through the blocked-softmax kernel (strided rows, additive key terms)
    (129, 1, 3, 128, "bf16"), (130, 1, 2, 128, "bf16"), (200, 1, 3, 64, "bf16"), (256, 1, 2, 128, "bf16"),
    (257, 1, 3, 64, "bf16"), (300, 2, 2, 128, "bf16"), (513, 1, 2, 128, "bf16"), (520, 1, 3, 64, "bf16"),
    # plain-ALU kernels beyond the 200 frames whose T x T block fits LDS: one wave per row, logits recomputed
    (200, 1, 2, 16, "f32"), (201, 1, 3, 24, "f32"), (333, 2, 1, 96, "bf16"), (700, 1, 1, 8, "f32"),
]


@pytest.mark.parametrize("final", [False, True])
@pytest.mark.parametrize("T,Hs,Ws,d,dt", L_CASES)
def test_l_update_matches_oracle(env, T, Hs, Ws, d, dt, final):
    torch, binding, dev = env
    bf16 = dt == "bf16"
    b, heads = Hs * Ws, 2
    rng = np.random.default_rng(2000 + T)
    data = U.structured_heads(T, Hs, Ws, d, 12, heads, bf16)
    Q = [h[0] for h in data]
    aL = [U.random_bits(rng, (T * b, d), 1.0, bf16) for _ in range(heads)]
    Y = [h[2] for h in data]
    cL = (-3.0 * rng.random((heads, T * b))).astype(np.float32)
    qs = 1.0 / math.sqrt(d)
    tq, taL, tcL = U.to_device(Q, torch, dev), U.to_device(aL, torch, dev), torch.from_numpy(cL).to(dev).view(1, heads, -1)
    rel_tol, abs_tol = _tol(bf16)
    if final:
        out = U.from_device(binding.l_update(tq, taL, tcL, U.to_device(Y, torch, dev), T, Hs, Ws, qs))
    else:
        gaR, gcR = binding.l_update(tq, taL, tcL, None, T, Hs, Ws, qs)
        gaR, gcR = U.from_device(gaR), U.from_device(gcR)
    for h in range(heads):
        Qb = (U.to_f64(Q[h]) * qs).reshape(T, b, d).transpose(1, 0, 2)
        oaR, ocR, L = O.l_update(U.to_f64(aL[h]).reshape(T, b, d).transpose(1, 0, 2), cL[h].reshape(T, b).T.astype(np.float64), Qb)
        if final:
            yb = U.to_f64(Y[h]).reshape(T, b, d).transpose(1, 0, 2)
            ref = np.matmul(L, yb).transpose(1, 0, 2).reshape(T * b, d)
            print(f"l_update final T={T} b={b} d={d} {dt}: rel {U.rel_l2(out[h], ref):.2e} max {U.max_abs(out[h], ref):.2e}")
            assert U.rel_l2(out[h], ref) <= rel_tol and U.max_abs(out[h], ref) <= abs_tol
        else:
            ref_aR = oaR.reshape(T * b, d)
            got = gaR[h] * qs       # the library sums unscaled Q
            # alpha_R is an unnormalised sum (rows reach c_R |Q|, far above 1) stored in bf16: its
            # rounding error is relative, one ulp = 2^-8 of the magnitude
            ratio = U.worst_ratio(got, ref_aR, 2.0 ** -8, abs_tol) if bf16 else U.max_abs(got, ref_aR) / abs_tol
            print(f"l_update fit T={T} b={b} d={d} {dt}: aR rel {U.rel_l2(got, ref_aR):.2e} max {U.max_abs(got, ref_aR):.2e} "
                  f"(|aR| max {np.abs(ref_aR).max():.2f}) worst/bound {ratio:.2f} cR max {U.max_abs(gcR[h], ocR.reshape(T * b)):.2e}")
            assert U.rel_l2(got, ref_aR) <= rel_tol and ratio <= 1.0
            assert U.max_abs(gcR[h], ocR.reshape(T * b)) <= (2e-2 if bf16 else 1e-4)
            np.testing.assert_allclose(gcR[h].reshape(T, b).sum(axis=0), T, rtol=5e-3 if bf16 else 1e-5)


# ------------------------------------------------------------------ first-frame recomputation
@pytest.fixture(params=["two-tile", "one-tile"])
def first_frame_kernel(request, env):
    """Exact attention of contiguous rows runs on the kernel with two query tiles per wave by default and on the
    one-tile kernel when flash variant 0 is selected (bf16, d = 64 or 128; other cases take neither)."""
    binding = env[1]
    default = binding.get_flash_variant()
    binding.set_flash_variant(0 if request.param == "one-tile" else default)
    yield request.param
    binding.set_flash_variant(default)


@pytest.mark.parametrize("T,Hs,Ws,d,dt", [(4, 4, 4, 32, "f32"), (3, 5, 5, 96, "bf16"), (1, 3, 3, 128, "bf16"),
                                           (4, 10, 30, 128, "bf16"), (9, 7, 9, 128, "bf16"),
                                           (3, 5, 5, 64, "bf16"), (4, 10, 30, 64, "bf16"), (9, 7, 9, 64, "bf16")])
def test_first_frame_attention_matches_oracle(env, T, Hs, Ws, d, dt, first_frame_kernel):
    torch, binding, dev = env
    bf16 = dt == "bf16"
    b, heads = Hs * Ws, 2
    data = U.structured_heads(T, Hs, Ws, d, 13, heads, bf16)
    tq, tk, tv = (U.to_device([h[i] for h in data], torch, dev) for i in range(3))
    out = torch.full_like(tq, 7.0)
    binding.first_frame_attention(tq, tk, tv, T, Hs, Ws, out)
    got = U.from_device(out)
    rel_tol, abs_tol = _tol(bf16)
    for h in range(heads):
        ref = O.first_frame_attention(*(U.to_f64(x) for x in data[h]), b)
        print(f"first_frame T={T} b={b} d={d} {dt}: rel {U.rel_l2(got[h][:b], ref):.2e} max {U.max_abs(got[h][:b], ref):.2e}")
        assert U.rel_l2(got[h][:b], ref) <= rel_tol and U.max_abs(got[h][:b], ref) <= abs_tol
        assert (got[h][b:] == 7.0).all()          # nothing beyond frame 0 is written


@pytest.mark.parametrize("T,b", [(15, 64), (16, 64), (17, 64), (33, 40), (64, 33), (130, 31), (9, 300)])
def test_first_frame_key_range_splits(env, T, b, first_frame_kernel):
    """N = T b keys around the points where the pass starts splitting the key range (at least 8 tiles per
    range) and where ranges end in ragged tiles."""
    torch, binding, dev = env
    d = 128
    rng = np.random.default_rng(700 + T * b)
    q, k, v = (U.random_bits(rng, (T * b, d), s, True) for s in (1.2, 1.2, 1.0))
    tq, tk, tv = (U.to_device([x], torch, dev) for x in (q, k, v))
    out = torch.zeros_like(tq)
    binding.first_frame_attention(tq, tk, tv, T, 1, b, out)
    ref = O.first_frame_attention(U.to_f64(q), U.to_f64(k), U.to_f64(v), b)
    g = U.from_device(out)[0][:b]
    assert U.rel_l2(g, ref) <= U.BF16_REL_L2 and U.max_abs(g, ref) <= U.BF16_MAX_ABS


@pytest.mark.parametrize("T,Hs,Ws,d,dt,begin,count", [(4, 4, 4, 32, "f32", 5, 20), (6, 9, 11, 128, "bf16", 300, 270),
                                                       (6, 9, 11, 64, "bf16", 593, 1), (3, 5, 5, 96, "bf16", 0, 75),
                                                       (20, 16, 16, 128, "bf16", 1000, 700)])
def test_recompute_rows_any_range(env, T, Hs, Ws, d, dt, begin, count):
    """Exact attention for an arbitrary contiguous token range (ranges that straddle frames, a single row, a
    whole head, a range long enough for the key ranges to be split); nothing outside the range is touched."""
    torch, binding, dev = env
    bf16 = dt == "bf16"
    b, heads = Hs * Ws, 2
    data = U.structured_heads(T, Hs, Ws, d, 23, heads, bf16)
    tq, tk, tv = (U.to_device([h[i] for h in data], torch, dev) for i in range(3))
    out = torch.full_like(tq, 7.0)
    binding.recompute_rows(tq, tk, tv, T, Hs, Ws, out, begin, count)
    got = U.from_device(out)
    rel_tol, abs_tol = _tol(bf16)
    for h in range(heads):
        q64, k64, v64 = (U.to_f64(x) for x in data[h])
        ref = O.softmax_attention(q64[begin:begin + count], k64, v64, 1.0 / math.sqrt(d))
        g = got[h][begin:begin + count]
        assert U.rel_l2(g, ref) <= rel_tol and U.max_abs(g, ref) <= abs_tol
        assert (got[h][:begin] == 7.0).all() and (got[h][begin + count:] == 7.0).all()
    with pytest.raises(binding.VMonarchError, match="rows"):
        binding.recompute_rows(tq, tk, tv, T, Hs, Ws, out, T * b - 3, 4)


TOKEN_CASES = [
    # T, Hs, Ws, d, dtype, kind of row list
    (4, 4, 4, 32, "f32", "random"),
    (3, 5, 5, 96, "bf16", "random"),          # plain-ALU bf16
    (6, 9, 11, 128, "bf16", "sorted"),
    (6, 9, 11, 128, "bf16", "unsorted"),
    (6, 9, 11, 64, "bf16", "one"),
    (5, 8, 8, 128, "bf16", "all"),
    (5, 8, 8, 64, "bf16", "all-reversed"),
    (20, 16, 16, 128, "bf16", "many"),        # several query blocks and key ranges, merged partial results
    (6, 9, 11, 128, "bf16", "with-strays"),   # entries outside [0, N) are skipped on the device
]


@pytest.mark.parametrize("T,Hs,Ws,d,dt,kind", TOKEN_CASES)
def test_recompute_tokens_any_subset(env, T, Hs, Ws, d, dt, kind):
    """Exact attention for an arbitrary list of rows (gathered on load, scattered on store): sorted and unsorted
    lists, one row, every row, a list long enough for several query blocks and key ranges; rows that are not
    listed stay bit-identical; the range form of the same rows gives the same bits."""
    torch, binding, dev = env
    bf16 = dt == "bf16"
    b, heads = Hs * Ws, 2
    N = T * b
    rng = np.random.default_rng(100 + T + d)
    if kind == "one":
        rows = np.array([N - 2])
    elif kind == "all":
        rows = np.arange(N)
    elif kind == "all-reversed":
        rows = np.arange(N)[::-1].copy()
    elif kind == "many":
        rows = rng.permutation(N)[:1500]
    else:
        rows = rng.permutation(N)[:max(3, N // 7)]
        if kind == "sorted":
            rows = np.sort(rows)
    listed = rows.copy()
    if kind == "with-strays":
        listed = np.concatenate([rows[:5], [-1, N, 2 ** 31 - 1, -2 ** 31], rows[5:]])
    data = U.structured_heads(T, Hs, Ws, d, 29, heads, bf16)
    tq, tk, tv = (U.to_device([h[i] for h in data], torch, dev) for i in range(3))
    torch.manual_seed(3)
    base = torch.randn((1, heads, N, d), device=dev).to(tq.dtype)
    out = base.clone()
    trows = torch.from_numpy(listed.astype(np.int32)).to(dev)
    binding.recompute_tokens(tq, tk, tv, T, Hs, Ws, out, trows)
    got, base_np = U.from_device(out), U.from_device(base)
    rel_tol, abs_tol = _tol(bf16)
    untouched = np.setdiff1d(np.arange(N), rows)
    for h in range(heads):
        q64, k64, v64 = (U.to_f64(x) for x in data[h])
        ref = O.softmax_attention(q64[rows], k64, v64, 1.0 / math.sqrt(d))
        assert U.rel_l2(got[h][rows], ref) <= rel_tol and U.max_abs(got[h][rows], ref) <= abs_tol
        assert np.array_equal(got[h][untouched], base_np[h][untouched])
    if kind in ("all", "all-reversed"):
        # the same rows as one contiguous range: identical arithmetic per row, identical bits, when the range runs on
        # the kernel that gathers a list (the contiguous range may otherwise take the kernel with two query tiles
        # per wave, whose sums associate differently: then the two agree to rounding)
        default = binding.get_flash_variant()
        binding.set_flash_variant(0)
        try:
            ranged = binding.recompute_rows(tq, tk, tv, T, Hs, Ws, base.clone(), 0, N)
        finally:
            binding.set_flash_variant(default)
        assert torch.equal(ranged.view(torch.uint8), out.view(torch.uint8))
        ranged2 = binding.recompute_rows(tq, tk, tv, T, Hs, Ws, base.clone(), 0, N)
        assert U.max_abs(U.from_device(ranged2), U.from_device(out)) <= (2 * abs_tol if dt == "bf16" else 1e-5)
    with pytest.raises(binding.VMonarchError):
        binding.recompute_tokens(tq, tk, tv, T, Hs, Ws, out, trows[:0])


@pytest.mark.parametrize("T,Hs,Ws,d,dt", [(4, 4, 4, 32, "f32"), (1, 3, 3, 128, "bf16"), (9, 7, 9, 128, "bf16"),
                                           (40, 16, 16, 64, "bf16")])
def test_first_frame_log_sum_exp_output(env, T, Hs, Ws, d, dt):
    """(1, 3, 3): one key range, written by the kernel; (40, 16, 16): several ranges, written by the merge."""
    torch, binding, dev = env
    bf16 = dt == "bf16"
    b, heads = Hs * Ws, 2
    data = U.structured_heads(T, Hs, Ws, d, 16, heads, bf16)
    tq, tk, tv = (U.to_device([h[i] for h in data], torch, dev) for i in range(3))
    out, out2 = torch.zeros_like(tq), torch.zeros_like(tq)
    _, lse = binding.first_frame_attention_lse(tq, tk, tv, T, Hs, Ws, out)
    binding.first_frame_attention(tq, tk, tv, T, Hs, Ws, out2)
    assert torch.equal(out, out2)
    glse = U.from_device(lse)
    for h in range(heads):
        q, k = U.to_f64(data[h][0])[:b], U.to_f64(data[h][1])
        z = q @ k.T / math.sqrt(d)
        zmax = z.max(axis=1, keepdims=True)
        ref = zmax[:, 0] + np.log(np.exp(z - zmax).sum(axis=1))
        err = U.max_abs(glse[h][:b], ref)
        print(f"first_frame_lse T={T} b={b} d={d} {dt}: lse max err {err:.2e}")
        assert err <= (5e-3 if bf16 else 1e-4)
        assert (glse[h][b:] == 0.0).all()


# ------------------------------------------------------------------ whole path
E2E = [
    # T, Hs, Ws, d, dtype, iters, recompute
    (4, 4, 4, 32, "f32", 2, True),            # the tiny plumbing config
    (3, 5, 7, 24, "f32", 3, False),
    (5, 4, 6, 96, "bf16", 2, True),           # plain-ALU bf16
    (5, 4, 6, 64, "bf16", 2, True),           # MFMA, d = 64
    (32, 1, 300, 64, "bf16", 2, False),       # d = 64, m = 32 blocks of b = 300 (a general (m, b) split, no video shape)
    (21, 12, 13, 64, "bf16", 2, True),
    (6, 17, 19, 64, "bf16", 3, True),
    (21, 12, 13, 128, "bf16", 2, True),       # MFMA: T = 21 (one wave per position), b = 156
    (21, 12, 13, 128, "bf16", 1, False),
    (6, 17, 19, 128, "bf16", 3, True),        # b = 323: ragged second query block
    (81, 3, 5, 128, "bf16", 2, True),         # T = 81: three waves per position
    (1, 9, 11, 128, "bf16", 2, False),        # single frame: exact attention
    (40, 1, 1, 128, "bf16", 2, False),        # single position: exact attention over frames
    (260, 3, 5, 128, "bf16", 2, True),        # more frames than positions: temporal factor on the blocked-softmax kernel
    (512, 1, 8, 64, "bf16", 2, False),        # m = 512 blocks of b = 8
    (300, 1, 1, 64, "bf16", 3, False),        # single position, 300 frames: exact attention over frames
    (230, 2, 3, 16, "f32", 2, True),          # plain-ALU kernels with more than 200 frames
    (260, 1, 4, 96, "bf16", 2, False),
]


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_attention_random_configurations(env, seed):
    """Seeded random (T, Hs, Ws, d, sweeps, recomputation mode, kernel family) through the whole path, every output
    element against the oracle: 12 configurations per seed, frames up to 300 (so that all three forms of the temporal
    factor occur), ragged everything."""
    torch, binding, dev = env
    rng = np.random.default_rng(seed)
    default = binding.get_flash_variant()
    done = 0
    try:
        while done < 12:
            d = int(rng.choice([64, 128]))
            T = int(rng.integers(1, 40)) if rng.random() < 0.85 else int(rng.integers(129, 300))
            Hs, Ws = int(rng.integers(1, 24)), int(rng.integers(1, 40))
            b = Hs * Ws
            if T * b > 40000 or T * b * b > 2e7:
                continue
            iters, rec, variant = int(rng.integers(1, 4)), int(rng.choice([0, 1, 1, 2])), int(rng.choice([0, 1, 2, 2]))
            data = U.structured_heads(T, Hs, Ws, d, 60 + done, 2, True)
            tq, tk, tv = (U.to_device([h[i] for h in data], torch, dev) for i in range(3))
            binding.set_flash_variant(variant)
            got = U.from_device(binding.attention(tq, tk, tv, T, Hs, Ws, iters, rec))
            for h in range(2):
                q64, k64, v64 = (U.to_f64(x) for x in data[h])
                res = O.monarch_attention(q64, k64, v64, T, b, iters, recompute=(rec == 1), sink_average=(rec == 2),
                                          keep_factors=True)
                ref = res["O"].reshape(T * b, d)
                rel, mx = U.rel_l2(got[h], ref), U.max_abs(got[h], ref)
                what = f"T={T} Hs={Hs} Ws={Ws} d={d} sweeps={iters} recompute={rec} variant={variant}"
                print(f"random configuration {what}: rel {rel:.2e} max {mx:.2e}")
                assert np.isfinite(got[h]).all() and rel <= U.BF16_REL_L2, what
                if rec == 2:
                    # averaged with exact attention over the first frame: half of each part's error
                    assert mx <= U.BF16_MAX_ABS, what
                else:
                    # element-wise: the flat 2e-2 where the first-order bound of the three bf16 roundings of an output
                    # (y stored, L as an operand, O stored) and of alpha_L's own storage is smaller, that bound elsewhere
                    ok, ratio = U.within_end_to_end_bound(got[h], res, U.BF16_MAX_ABS, True,
                                                          (q64 / math.sqrt(d)).reshape(T, b, d), recomputed_frame=(rec == 1))
                    assert ok, (what, ratio)
            done += 1
    finally:
        binding.set_flash_variant(default)


@pytest.mark.parametrize("T,Hs,Ws,d,dt,iters,rec", E2E)
def test_attention_matches_oracle(env, T, Hs, Ws, d, dt, iters, rec):
    torch, binding, dev = env
    bf16 = dt == "bf16"
    b, heads = Hs * Ws, 2
    data = U.structured_heads(T, Hs, Ws, d, 14, heads, bf16)
    tq, tk, tv = (U.to_device([h[i] for h in data], torch, dev) for i in range(3))
    got = U.from_device(binding.attention(tq, tk, tv, T, Hs, Ws, iters, rec))
    again = U.from_device(binding.attention(tq, tk, tv, T, Hs, Ws, iters, rec))
    assert np.array_equal(got, again)          # no atomics anywhere: runs are bit-identical
    rel_tol, abs_tol = _tol(bf16)
    for h in range(heads):
        ref = O.monarch_attention(*(U.to_f64(x) for x in data[h]), T, b, iters, recompute=rec, cr_min=0.1)["O"].reshape(T * b, d)
        assert np.isfinite(got[h]).all()
        print(f"attention T={T} b={b} d={d} {dt} iters={iters} rec={rec}: rel {U.rel_l2(got[h], ref):.2e} max {U.max_abs(got[h], ref):.2e}")
        assert U.rel_l2(got[h], ref) <= rel_tol, U.rel_l2(got[h], ref)
        assert U.max_abs(got[h], ref) <= abs_tol, U.max_abs(got[h], ref)


def test_single_frame_equals_textbook_attention(env):
    torch, binding, dev = env
    Hs, Ws, d = 14, 15, 128
    data = U.structured_heads(1, Hs, Ws, d, 15, 1, True)
    tq, tk, tv = (U.to_device([data[0][i]], torch, dev) for i in range(3))
    got = U.from_device(binding.attention(tq, tk, tv, 1, Hs, Ws, 2, False))[0]
    q, k, v = (U.to_f64(x) for x in data[0])
    ref = O.softmax_attention(q, k, v, 1.0 / math.sqrt(d))
    assert U.rel_l2(got, ref) <= U.BF16_REL_L2 and U.max_abs(got, ref) <= U.BF16_MAX_ABS


def test_cr_min_setting_and_sink_regime(env):
    torch, binding, dev = env
    T, Hs, Ws, d, heads = 9, 6, 7, 128, 1
    data = U.structured_heads(T, Hs, Ws, d, 16, heads, True, sink=3.0)
    tq, tk, tv = (U.to_device([h[i] for h in data], torch, dev) for i in range(3))
    assert abs(binding.get_cr_min() - 0.1) < 1e-7
    for cr_min in (0.1, 0.5):
        binding.set_cr_min(cr_min)
        try:
            got = U.from_device(binding.attention(tq, tk, tv, T, Hs, Ws, 2, True))[0]
        finally:
            binding.set_cr_min(0.1)
        ref = O.monarch_attention(*(U.to_f64(x) for x in data[0]), T, Hs * Ws, 2, recompute=True, cr_min=cr_min)["O"].reshape(-1, d)
        assert U.rel_l2(got, ref) <= U.BF16_REL_L2 and U.max_abs(got, ref) <= U.BF16_MAX_ABS


def test_constant_values_give_constant_output(env):
    torch, binding, dev = env
    T, Hs, Ws, d = 21, 8, 9, 128
    data = U.structured_heads(T, Hs, Ws, d, 17, 1, True)
    tq, tk = (U.to_device([data[0][i]], torch, dev) for i in range(2))
    tv = torch.ones_like(tq)
    out = binding.attention(tq, tk, tv, T, Hs, Ws, 2, True).float()
    assert float((out - 1.0).abs().max()) <= 1e-2


def test_user_workspace_is_used_and_checked(env):
    torch, binding, dev = env
    T, Hs, Ws, d = 5, 6, 6, 128
    data = U.structured_heads(T, Hs, Ws, d, 18, 1, True)
    tq, tk, tv = (U.to_device([data[0][i]], torch, dev) for i in range(3))
    ref = binding.attention(tq, tk, tv, T, Hs, Ws, 2, True)
    need = binding.workspace_bytes(1, 1, T, Hs, Ws, d, 2, True, 2)
    assert need > 0
    ws = torch.empty(need, dtype=torch.uint8, device=dev)
    binding.set_workspace(ws)
    try:
        assert torch.equal(binding.attention(tq, tk, tv, T, Hs, Ws, 2, True), ref)
        binding.set_workspace(ws[: need // 2 // 256 * 256])
        with pytest.raises(binding.VMonarchError, match="workspace"):
            binding.attention(tq, tk, tv, T, Hs, Ws, 2, True)
    finally:
        binding.set_workspace(None)


def test_batch_and_head_axes_are_independent(env):
    """[B][heads] is one flat axis of independent problems: a (2, 3) batch equals its six single runs."""
    torch, binding, dev = env
    T, Hs, Ws, d = 6, 9, 11, 128
    data = U.structured_heads(T, Hs, Ws, d, 19, 6, True)
    full = [torch.stack([torch.from_numpy(data[2 * bb + hh][i]).view(torch.bfloat16) for bb in range(3) for hh in range(2)])
            .view(3, 2, T * Hs * Ws, d).to(dev) for i in range(3)]
    got = binding.attention(full[0], full[1], full[2], T, Hs, Ws, 2, True)
    for bb in range(3):
        for hh in range(2):
            one = [x[bb:bb + 1, hh:hh + 1].contiguous() for x in full]
            assert torch.equal(binding.attention(one[0], one[1], one[2], T, Hs, Ws, 2, True)[0, 0], got[bb, hh])


def test_whole_path_replays_from_a_hip_graph(env):
    """With a caller workspace the call only enqueues kernels (no allocation, no synchronisation), so it
    can be captured once and replayed; every replay, with fresh inputs in the same buffers and eager work
    in between, must equal the eager result bit for bit."""
    torch, binding, dev = env
    T, Hs, Ws, d, heads = 8, 10, 13, 128, 2
    N = T * Hs * Ws
    sets = [U.structured_heads(T, Hs, Ws, d, 30 + r, heads, True) for r in range(3)]
    def dev_inputs(r):
        return [U.to_device([h[i] for h in sets[r]], torch, dev) for i in range(3)]
    need = binding.workspace_bytes(1, heads, T, Hs, Ws, d, 2, True, 2)
    ws = torch.empty(need, dtype=torch.uint8, device=dev)
    binding.set_workspace(ws)
    try:
        sq, sk, sv = dev_inputs(0)
        sout = torch.empty_like(sq)
        eager = [binding.attention(*dev_inputs(r), T, Hs, Ws, 2, True).clone() for r in range(3)]  # also warms up
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            binding.attention(sq, sk, sv, T, Hs, Ws, 2, True, out=sout)
        torch.cuda.current_stream().wait_stream(side)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            binding.attention(sq, sk, sv, T, Hs, Ws, 2, True, out=sout)
        for r in (1, 2, 0, 1):
            nq, nk, nv = dev_inputs(r)
            sq.copy_(nq); sk.copy_(nk); sv.copy_(nv)
            sout.fill_(float("nan"))
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(sout, eager[r])
            # eager work of the same library between replays
            assert torch.equal(binding.attention(nq, nk, nv, T, Hs, Ws, 2, True), eager[r])
    finally:
        torch.cuda.synchronize()
        binding.set_workspace(None)


def test_mfma_probe_runs_and_counts_its_work(env):
    torch, binding, dev = env
    blocks, iters = 4, 3
    ops = torch.ones(blocks * 512 * 64, dtype=torch.bfloat16, device=dev)
    out, fl = binding.mfma_probe(ops, blocks, iters)
    assert fl == blocks * 8 * iters * 8 * 2 * 32 * 32 * 16
    # all-ones operands: every accumulator element is 16 per MFMA; 8 * iters MFMAs over 4 accumulators of 16
    # registers, summed per lane
    assert torch.equal(out.cpu(), torch.full((blocks * 512,), float(16 * 8 * iters * 16)))


def test_invalid_arguments_are_rejected_without_launching(env):
    torch, binding, dev = env
    L = binding.lib()
    t = torch.zeros(1, 1, 16, 128, dtype=torch.bfloat16, device=dev)
    p = ctypes.c_void_p(t.data_ptr())
    assert L.vmonarch_attention(None, p, p, p, 1, 1, 4, 2, 2, 128, 2, 1, None) == -1
    assert L.vmonarch_attention(p, p, p, p, 1, 1, 4, 2, 2, 128, 2, 1, None) == -1            # out aliases q
    o = torch.zeros_like(t); po = ctypes.c_void_p(o.data_ptr())
    assert L.vmonarch_attention(p, p, p, po, 1, 1, 4, 2, 2, 128, 0, 1, None) == -1           # iters < 1
    assert L.vmonarch_attention(p, p, p, po, 1, 1, 0, 2, 2, 128, 2, 1, None) == -1           # T = 0
    assert L.vmonarch_attention(p, p, p, po, 1, 1, 4, 2, 2, 512, 2, 1, None) == -2           # d too large
    assert b"exceeds" in L.vmonarch_last_error()
    assert L.vmonarch_set_entropy_mode(7) == -1
    torch.cuda.synchronize()
    assert float(o.float().abs().max()) == 0.0

"""GPU parity at the benchmark's full sizes and launch configuration, on sampled outputs.

The oracle follows a subset of query positions exactly (each position's iteration depends
only on its own T queries and on all of K, V), so full-size runs are checked on sampled
positions over all frames, plus properties that need no oracle.
"""
import dataclasses
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
    binding.lib()
    return torch, binding, torch.device("cuda:0")


def _run_workload(env, name, heads, n_pos, seed, iters=None, wl=None):
    torch, binding, dev = env
    wl = synth.WORKLOADS[name] if wl is None else wl
    if iters is not None:
        wl = dataclasses.replace(wl, iters=iters)
    q, k, v = synth.make_inputs(wl, heads=heads)
    tq, tk, tv = (torch.from_numpy(x).to(dev).view(torch.bfloat16).view(1, len(heads), wl.N, wl.d) for x in (q, k, v))
    out = binding.attention(tq, tk, tv, wl.T, wl.Hs, wl.Ws, wl.iters, wl.recompute)
    got = out.float().cpu().numpy()[0].reshape(len(heads), wl.T, wl.b, wl.d)
    assert np.isfinite(got).all()
    rng = np.random.default_rng(seed)
    worst = (0.0, 0.0)
    for hi in range(len(heads)):
        # always include the edges of the last (ragged) query block and key tile and both sides of the
        # interior query-block boundaries
        forced = U.boundary_positions(wl.b)
        free = np.setdiff1d(np.arange(wl.b), forced)
        pos = np.sort(np.concatenate([forced, rng.choice(free, size=max(n_pos - len(forced), 4), replace=False)]))
        ref = O.monarch_attention(O.widen_bf16(q[hi]), O.widen_bf16(k[hi]), O.widen_bf16(v[hi]), wl.T, wl.b, wl.iters,
                                  recompute=wl.recompute, positions=pos)["O"]
        g = got[hi][:, pos, :]
        rel, mx = U.rel_l2(g, ref), U.max_abs(g, ref)
        w = np.unravel_index(np.argmax(np.abs(g - ref)), ref.shape)
        print(f"{name} head {heads[hi]}: {len(pos)} positions x {wl.T} frames: rel {rel:.2e} max {mx:.2e} "
              f"(max / 2e-2 = {mx / U.BF16_MAX_ABS:.2f}; worst at frame {w[0]} position {pos[w[1]]} channel {w[2]}: "
              f"got {g[w]:.5f} ref {ref[w]:.5f})")
        worst = (max(worst[0], rel), max(worst[1], mx))
        assert rel <= U.BF16_REL_L2 and mx <= U.BF16_MAX_ABS
    return tq, tk, tv, out, wl


def test_wan_480p_clip_sampled_positions(env):
    _run_workload(env, "wan1.3b-480p", [0, 7], 48, 1)


def test_wan_720p_clip_sampled_positions(env):
    """b = 3600 (15 query blocks, ragged), T = 21 padded to 32 in the temporal pass; 3 of the 40 heads."""
    _run_workload(env, "wan14b-720p", [0, 21, 39], 24, 3)


@pytest.mark.parametrize("iters", [1, 3])
def test_wan_720p_clip_one_and_three_sweeps(env, iters):
    """The 720p workload with 1 and 3 sweeps (the pair that separates the cost of one sweep in the benchmark)."""
    _run_workload(env, "wan14b-720p", [17], 16, 30 + iters, iters=iters)


@pytest.mark.parametrize("m,b", synth.BUDGET_SPLITS)
def test_computation_budget_splits_of_32k_tokens(env, m, b):
    """N = 2^15 tokens as m blocks of b, every power-of-two split from (8, 4096) to (512, 64), d = 64: from four
    query blocks per R-update problem and one wave per temporal block to one tile per R-update problem and the
    temporal factor on the blocked-softmax kernel (m = 256, 512)."""
    _run_workload(env, f"budget-{m}x{b}", [0, 11], 20, 40 + m.bit_length())


def test_blocks_of_two_frames(env):
    """Block size b = 2 H W (two frames per spatial block, half as many temporal blocks), the paper's block-size
    ablation: the same call with T / 2 frames of 2 H x W tokens.  20 frames of 28 x 52 tokens -> m = 10, b = 2912."""
    wl = synth.Workload("two-frame-blocks-20x28x52", 7, 1, 12, 10, 56, 52, 128, "bf16", 2, True)
    _run_workload(env, wl.name, [0, 7], 24, 9, wl=wl)


def test_permutation_copy_at_headline_shape(env):
    """The stride permutation of 12 x 117,936 rows of 256 bytes (the benchmark's copy calibration) and of rows of
    12 bytes (the 4-byte-word form), bit-exact against the oracle's index map, and back."""
    torch, binding, dev = env
    wl = synth.WORKLOADS["long-81x28x52"]
    perm, _ = O.index_maps(wl.T, wl.b)
    tperm = torch.from_numpy(perm.astype(np.int64)).to(dev)
    for d, dt in ((128, torch.int16), (3, torch.int32)):
        g = torch.Generator(device=dev).manual_seed(d)
        x = torch.randint(-30000, 30000, (1, 3, wl.N, d), device=dev, generator=g, dtype=torch.int32).to(dt)
        got = binding.permute_tokens(x, wl.T, wl.Hs, wl.Ws, True)
        assert torch.equal(got, x[:, :, tperm, :])
        assert torch.equal(binding.permute_tokens(got, wl.T, wl.Hs, wl.Ws, False), x)


def test_million_token_stress_two_heads(env):
    """N = 991,440 tokens: b = 12,240 keys per frame (192 key tiles, ragged), one sweep, no
    recomputation; two of the 12 heads (row offsets beyond 2^31 bytes within the head)."""
    _run_workload(env, "stress-1m", [5, 11], 16, 4)


def test_paper_kernel_benchmark_shape_sampled_positions(env):
    """d = 64, m = 32 blocks of b = 2048 tokens (N = 2^16), 2 sweeps: the largest shape of the
    paper's own kernel benchmark; 2 of the 12 heads."""
    _run_workload(env, "kernel-bench-64k", [0, 11], 24, 5)


def test_headline_long_video_sampled_positions_and_invariants(env):
    torch, binding, dev = env
    tq, tk, tv, out, wl = _run_workload(env, "long-81x28x52", [0, 5, 11], 24, 2)
    # recomputation touches only frame 0
    out_norec = binding.attention(tq, tk, tv, wl.T, wl.Hs, wl.Ws, wl.iters, False)
    assert torch.equal(out[:, :, wl.b:], out_norec[:, :, wl.b:])
    assert not torch.equal(out[:, :, :wl.b], out_norec[:, :, :wl.b])
    # constant values come back unchanged; outputs stay inside the hull of the values
    ones = torch.ones_like(tv)
    o1 = binding.attention(tq, tk, ones, wl.T, wl.Hs, wl.Ws, wl.iters, wl.recompute).float()
    assert float((o1 - 1.0).abs().max()) <= 1e-2
    vf = tv.float()
    lo, hi = vf.amin(dim=2, keepdim=True), vf.amax(dim=2, keepdim=True)
    of = out.float()
    assert bool(((of >= lo - 2e-2) & (of <= hi + 2e-2)).all())
    # bit-identical on a second run
    assert torch.equal(out, binding.attention(tq, tk, tv, wl.T, wl.Hs, wl.Ws, wl.iters, wl.recompute))


@pytest.mark.parametrize("variant", [0, 1])
def test_headline_shape_with_one_kernel_family_for_both_updates(env, variant):
    """The default gives each R-update the kernel measured faster for it; here both updates run on the kernels
    with two waves per SIMD (0), then both on the kernel with one wave per SIMD and two query tiles per wave (1)."""
    torch, binding, dev = env
    default = binding.get_flash_variant()
    binding.set_flash_variant(variant)
    try:
        _run_workload(env, "long-81x28x52", [2, 9], 24, 6)
        _run_workload(env, "wan1.3b-480p", [0], 48, 1)
    finally:
        binding.set_flash_variant(default)


def test_headline_unclamped_cr_sums_to_frame_count(env):
    """sum_k c_R[k, i] = T for every position (each query frame spreads one unit of mass)."""
    torch, binding, dev = env
    wl = synth.WORKLOADS["long-81x28x52"]
    q, k, v = synth.make_inputs(wl, heads=[3])
    tq, tk = (torch.from_numpy(x).to(dev).view(torch.bfloat16).view(1, 1, wl.N, wl.d) for x in (q, k))
    s = 1.0 / math.sqrt(wl.d)
    aL, cL, _ = binding.r_update(tq, None, tk, None, wl.T, wl.Hs, wl.Ws, s, 0.1)
    aR, cR = binding.l_update(tq, aL, cL, None, wl.T, wl.Hs, wl.Ws, s)
    tot = cR.view(wl.T, wl.b).sum(dim=0)
    assert float((tot - wl.T).abs().max()) <= 5e-3 * wl.T
    assert float(cL.max()) <= 1e-4          # c_L = -entropy <= 0
    assert float(cL.min()) >= -math.log(wl.b) - 1e-3


def test_backward_at_headline_shape_sampled_frames(env):
    """Alg. 2 backward on the 81 x 28 x 52 shape (one head, all 81 frames computed); three frames are checked
    entirely against the oracle, which is fed the kernel's own forward inputs."""
    torch, binding, dev = env
    wl = synth.WORKLOADS["long-81x28x52"]
    q, k, v = synth.make_inputs(wl, heads=[4])
    rng = np.random.default_rng(11)
    dO = U.random_bits(rng, (wl.N, wl.d), 1.0, True)
    dH = rng.normal(size=wl.N).astype(np.float32)
    tq, tk, tv = (torch.from_numpy(x).to(dev).view(torch.bfloat16).view(1, 1, wl.N, wl.d) for x in (q, k, v))
    tdo = U.to_device([dO], torch, dev)
    tdh = torch.from_numpy(dH).to(dev).view(1, 1, -1)
    s = 1.0 / math.sqrt(wl.d)
    _, cL, y, lse = binding.r_update_lse(tq, None, tk, tv, wl.T, wl.Hs, wl.Ws, s, 0.1)
    Hent = (-cL).contiguous()
    dq, dk, dv = binding.entropy_attention_bwd(tq, None, tk, tv, y, tdo, lse, Hent, tdh, wl.T, wl.Hs, wl.Ws, s, 0.1)
    assert all(bool(torch.isfinite(x.float()).all()) for x in (dq, dk, dv))
    got = [U.from_device(x)[0].reshape(wl.T, wl.b, wl.d) for x in (dq, dk, dv)]
    gy, glse, gH = (U.from_device(x)[0] for x in (y, lse, Hent))
    q64, k64, v64 = (O.widen_bf16(x[0]).reshape(wl.T, wl.b, wl.d) for x in (q, k, v))
    do64 = U.to_f64(dO).reshape(wl.T, wl.b, wl.d)
    for kf in (0, 37, 80):
        ref = O.entropy_attention_backward(q64[kf], k64[kf], v64[kf], gy.reshape(wl.T, wl.b, wl.d)[kf].astype(np.float64),
                                           do64[kf], glse.reshape(wl.T, wl.b)[kf].astype(np.float64),
                                           gH.reshape(wl.T, wl.b)[kf].astype(np.float64),
                                           dH.reshape(wl.T, wl.b)[kf].astype(np.float64), np.full(wl.b, s))
        for name, g, r in zip(("dq", "dk", "dv"), got, ref):
            err = U.rel_l2(g[kf], r)
            print(f"backward frame {kf} {name}: rel {err:.2e}")
            assert err <= 1e-2
        # and the whole chain: the oracle's own forward (fp64, from the definitions) feeding its backward
        Oo, l64, H64 = O.entropy_attention(q64[kf], k64[kf], v64[kf], np.full(wl.b, s))
        ref = O.entropy_attention_backward(q64[kf], k64[kf], v64[kf], Oo, do64[kf], l64, H64,
                                           dH.reshape(wl.T, wl.b)[kf].astype(np.float64), np.full(wl.b, s))
        # D = rowsum(dO o O) sees O rounded to bf16: first-order effect on dQ and dK (two standard deviations of the
        # sum of d independent roundings per row) added to the 1e-2
        dD = 2.0 * 2.0 ** -9 / math.sqrt(3.0) * np.sqrt(((do64[kf] * Oo) ** 2).sum(axis=1))
        P = np.exp((q64[kf] @ k64[kf].T) * s - l64[:, None])
        extra = (np.linalg.norm((s * dD)[:, None] * (P @ k64[kf])) / np.linalg.norm(ref[0]),
                 np.linalg.norm((P * (s * dD)[:, None]).T @ np.abs(q64[kf])) / np.linalg.norm(ref[1]), 0.0)
        for name, g, r, ex in zip(("dq", "dk", "dv"), got, ref, extra):
            err = U.rel_l2(g[kf], r)
            print(f"forward+backward frame {kf} {name}: rel {err:.2e} of {1e-2 + ex:.2e} allowed")
            assert err <= 1e-2 + ex


def test_headline_shape_ablation_variants_sampled_positions(env):
    """Sink averaging and manual c_R / c_L control at the headline shape (2 heads), sampled positions over all
    frames, plus arbitrary-row recomputation of a range that straddles two frames."""
    torch, binding, dev = env
    wl = synth.WORKLOADS["long-81x28x52"]
    heads = [3, 8]
    q, k, v = synth.make_inputs(wl, heads=heads)
    tq, tk, tv = (torch.from_numpy(x).to(dev).view(torch.bfloat16).view(1, len(heads), wl.N, wl.d) for x in (q, k, v))
    rng = np.random.default_rng(11)
    pos = np.sort(rng.choice(wl.b, size=12, replace=False))
    pos[0], pos[-1] = 0, wl.b - 1
    wide = [tuple(O.widen_bf16(x[hi]) for x in (q, k, v)) for hi in range(len(heads))]

    def check(tag, out, **kw):
        got = out.float().cpu().numpy()[0].reshape(len(heads), wl.T, wl.b, wl.d)
        for hi in range(len(heads)):
            ref = O.monarch_attention(*wide[hi], wl.T, wl.b, wl.iters, positions=pos, **kw)["O"]
            g = got[hi][:, pos, :]
            print(f"{tag} head {heads[hi]}: rel {U.rel_l2(g, ref):.2e} max {U.max_abs(g, ref):.2e}")
            assert U.rel_l2(g, ref) <= U.BF16_REL_L2 and U.max_abs(g, ref) <= U.BF16_MAX_ABS

    check("sink", binding.attention(tq, tk, tv, wl.T, wl.Hs, wl.Ws, wl.iters, 2), sink_average=True)
    binding.set_manual_control(1, 1)
    try:
        out = binding.attention(tq, tk, tv, wl.T, wl.Hs, wl.Ws, wl.iters, True)
    finally:
        binding.set_manual_control()
    check("control cR1 cL1", out, recompute=True, cr_control=1, cl_control=1)
    # rows [40*b - 700, 40*b + 900) recomputed exactly; everything else keeps the Monarch result
    base = binding.attention(tq, tk, tv, wl.T, wl.Hs, wl.Ws, wl.iters, False)
    mixed = base.clone()
    begin, count = 40 * wl.b - 700, 1600
    binding.recompute_rows(tq, tk, tv, wl.T, wl.Hs, wl.Ws, mixed, begin, count)
    assert torch.equal(mixed[:, :, :begin], base[:, :, :begin]) and torch.equal(mixed[:, :, begin + count:], base[:, :, begin + count:])
    rows = np.sort(rng.choice(count, size=40, replace=False)) + begin
    rows[0], rows[-1] = begin, begin + count - 1
    got = mixed.float().cpu().numpy()[0]
    for hi in range(len(heads)):
        ref = O.softmax_attention(wide[hi][0][rows], wide[hi][1], wide[hi][2], 1.0 / math.sqrt(wl.d))
        assert U.rel_l2(got[hi][rows], ref) <= U.BF16_REL_L2 and U.max_abs(got[hi][rows], ref) <= U.BF16_MAX_ABS
    # an arbitrary subset of 3000 tokens spread over all frames, unsorted; everything else keeps the Monarch result
    picked = rng.permutation(wl.N)[:3000]
    subset = base.clone()
    binding.recompute_tokens(tq, tk, tv, wl.T, wl.Hs, wl.Ws, subset, torch.from_numpy(picked.astype(np.int32)).to(dev))
    keep = torch.ones(wl.N, dtype=torch.bool, device=dev)
    keep[torch.from_numpy(picked).to(dev)] = False
    assert torch.equal(subset[:, :, keep], base[:, :, keep])
    check_rows = picked[:40]
    got = subset.float().cpu().numpy()[0]
    for hi in range(len(heads)):
        ref = O.softmax_attention(wide[hi][0][check_rows], wide[hi][1], wide[hi][2], 1.0 / math.sqrt(wl.d))
        assert U.rel_l2(got[hi][check_rows], ref) <= U.BF16_REL_L2 and U.max_abs(got[hi][check_rows], ref) <= U.BF16_MAX_ABS

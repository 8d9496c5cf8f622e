"""Shared helpers for the GPU parity tests: seeded inputs, torch marshalling, error norms."""
import math

import numpy as np

from oracle import vmonarch_oracle as O
from paper_2601_22275_amd import synth

# bf16 tensors with fp32 accumulation (tolerance stated by the task for the bf16 path)
BF16_REL_L2 = 1e-2
BF16_MAX_ABS = 2e-2
# fp32 path: accumulation-order noise only
F32_REL_L2 = 1e-4


def rel_l2(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-30))


def max_abs(a, b):
    return float(np.abs(np.asarray(a, dtype=np.float64) - np.asarray(b, dtype=np.float64)).max())


def worst_ratio(got, ref, rel, floor=BF16_MAX_ABS):
    """max over elements of |got - ref| / max(floor, rel * |ref|): the element-wise form of a bound that is
    the flat bf16 tolerance for small values and `rel` of the element's OWN magnitude for large ones
    (bf16 keeps 8 significant bits: one rounding is 2^-9 |x| at most, stored intermediates add theirs)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float((np.abs(got - ref) / np.maximum(floor, rel * np.abs(ref))).max())


def weighted_sum_bound(ref, abs_weighted, floor=BF16_MAX_ABS):
    """Element-wise bound for a bf16 weighted average sum_l w_l x_l that the kernels form with bf16-rounded weights
    and store in bf16: every weight carries one rounding (2^-9 relative, so at most 2^-9 sum_l w_l |x_l| in the sum:
    `abs_weighted` is that sum of magnitudes) and the result one more (half an ulp, at most 2^-8 |ref|).  Below the
    task's flat tolerance `floor` the flat tolerance applies."""
    return np.maximum(floor, 2.0 ** -9 * np.asarray(abs_weighted, dtype=np.float64) + 2.0 ** -8 * np.abs(ref))


def boundary_positions(b):
    """Query positions on both sides of the interior query-block boundaries of the MFMA kernels (128-row
    blocks of the one-pass R-update, 256-row blocks of the other passes), the last full block and the ends."""
    want = [0, 127, 128, 255, 256, 1407, 1408, b - 1]
    return sorted({p for p in want if 0 <= p < b})


def structured_heads(T, Hs, Ws, d, config, heads, bf16, gain=None, sink=0.0):
    """q, k, v as lists over heads of (N, d) arrays: float32, or uint16 bf16 bits."""
    phi = synth.positional_features(T, Hs, Ws)
    out = []
    for h in range(heads):
        qh, kh, vh, _ = synth.head_inputs(T, Hs, Ws, d, config, h, gain=gain if gain is not None else (None if bf16 else 1.0),
                                          sink=sink, phi=phi)
        if bf16:
            out.append(tuple(synth.f32_to_bf16_bits(x) for x in (qh, kh, vh)))
        else:
            out.append((qh, kh, vh))
    return out


def to_f64(x):
    return O.widen_bf16(x) if x.dtype == np.uint16 else x.astype(np.float64)


def to_device(arrs, torch, dev):
    """list over heads of (N, d) arrays -> [1, heads, N, d] device tensor (bf16 or f32)."""
    a = np.stack(arrs)
    t = torch.from_numpy(a).to(dev)
    if a.dtype == np.uint16:
        t = t.view(torch.bfloat16)
    return t.view(1, *a.shape)


def from_device(t):
    return t.float().cpu().numpy()[0]


def random_bits(rng, shape, scale, bf16):
    x = (scale * rng.standard_normal(shape)).astype(np.float32)
    return synth.f32_to_bf16_bits(x) if bf16 else x


def within_end_to_end_bound(got, res, abs_tol, bf16, q_scaled=None, recomputed_frame=True):
    """Element-wise bound against an oracle result `res` (kept factors).  In the bf16 path an output element
    O[j,i] = sum_k L[j,k] y[k] carries three roundings: of every y[k] when it is stored (half an ulp, at most
    2^-8 |y[k]|), of every weight L[j,k] as a matrix operand (2^-9 relative) and of the result (at most 2^-8 |O|):
    (2^-8 + 2^-9) sum_k L[j,k] |y[k]| + 2^-8 |O|.  The weights themselves inherit the bf16 storage of alpha_L:
    the temporal logit u[j,k] = Q[j] . alpha_L[k] moves by about 2^-9 (sum_v (Q[j,v] alpha_L[k,v])^2)^(1/2) (one
    independent rounding per channel, root sum of squares), a softmax weight by at most twice the largest such
    shift of its row, and the output by that times sum_k L[j,k] |y[k]|.  The control variants sharpen the
    temporal factor: rows of y reach the output undiluted and differences of large rows do not average out, so
    these terms exceed the flat 2e-2 in places.  Frame 0 is recomputed from all keys and stays under the flat
    tolerance."""
    T, s_, d = res["O"].shape
    ref = res["O"].reshape(T * s_, d)
    if not bf16:
        return max_abs(got, ref) <= abs_tol, max_abs(got, ref) / abs_tol
    spread = np.einsum("ijk,ikv->jiv", res["L"], np.abs(res["y"]))                       # [j, i, v]
    du = 2.0 ** -9 * np.sqrt(np.einsum("jiv,ikv->ijk", q_scaled ** 2, res["aL"] ** 2))     # [i, j, k]
    shift = 2.0 * du.max(axis=2).T                                                       # [j, i]
    bound = (2.0 ** -8 + 2.0 ** -9 + shift[:, :, None]) * spread + 2.0 ** -8 * np.abs(res["O"])
    bound = np.maximum(abs_tol, bound).reshape(T * s_, d)
    if recomputed_frame:
        bound[:s_] = abs_tol
    ratio = np.abs(got - ref) / bound
    w = np.unravel_index(np.argmax(ratio), ratio.shape)
    print(f"  worst element: token {w[0]} (frame {w[0] // s_}) channel {w[1]}: got {got[w]:.5f} ref {ref[w]:.5f} "
          f"sum L|y| {spread.reshape(T * s_, d)[w]:.4f} logit shift {shift.reshape(-1)[w[0]]:.4f} bound {bound[w]:.4f}")
    return float(ratio[w]) <= 1.0, float(ratio[w])

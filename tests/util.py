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

"""Seeded synthetic video-token workloads (inputs only; none of the method's arithmetic).

The paper evaluates on activations of Wan video diffusion transformers
(Sec. 4.1); those models are not available here, so q/k/v are synthetic
stand-ins with the same shapes and a comparable structure: logits that peak
for tokens at nearby (frame, row, column) coordinates, which is the
near-block-diagonal pattern Sec. 3.2 describes.

Recipe, per (batch*head) index ``h`` of workload ``config``:
  seed      = 20260122 + 1000*config + h                     (Philox stream)
  phi(t,y,x) in R^{6F}, F = 8: for each axis a in (t, y, x) and r = 1..F,
              sin(2 pi r c_a), cos(2 pi r c_a), c_a = coordinate / extent
  W_qk, W_v ~ N(0, 1/(6F)) of shape (6F, d); W_qk is shared by q and k
  q = g (0.5 e_q + phi W_qk),  k = g (0.5 e_k + phi W_qk),  v = 0.5 e_v + phi W_v
  e_* iid N(0, 1)
  g = 1 for the fp32 plumbing case; otherwise g is set so that the standard
  deviation of q_n . k_n' / sqrt(d) over 65,536 seeded random token pairs is 3.
  ``sink`` > 0 adds sink * u (u a seeded unit vector) to every query and to the
  keys of frame 0, which makes frame 0 attract attention from every frame (the
  regime Sec. 3.3 describes).
bf16 workloads are rounded to nearest-even and returned as uint16 bit patterns,
so every consumer reads the same bytes.
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import numpy as np

F_BANDS = 8
BASE_SEED = 20260122


@dataclass(frozen=True)
class Workload:
    name: str
    config: int          # index used in the seed
    B: int
    heads: int
    T: int
    Hs: int
    Ws: int
    d: int
    dtype: str           # "f32" or "bf16"
    iters: int
    recompute: bool

    @property
    def b(self) -> int:
        return self.Hs * self.Ws

    @property
    def N(self) -> int:
        return self.T * self.Hs * self.Ws


WORKLOADS = {
    "tiny": Workload("tiny", 0, 1, 2, 4, 4, 4, 32, "f32", 2, True),
    "wan1.3b-480p": Workload("wan1.3b-480p", 1, 1, 12, 21, 30, 52, 128, "bf16", 2, True),
    "wan14b-720p": Workload("wan14b-720p", 2, 1, 40, 21, 45, 80, 128, "bf16", 2, True),
    "long-81x28x52": Workload("long-81x28x52", 3, 1, 12, 81, 28, 52, 128, "bf16", 2, True),
    "stress-1m": Workload("stress-1m", 4, 1, 12, 81, 90, 136, 128, "bf16", 1, False),
}
# The paper's own kernel benchmark (App. "Kernel Optimization of VMonarch"): batch 1, 12 heads,
# d = 64, 2 sweeps, m = 32 blocks of b = N / 32 tokens, N = 2^10 .. 2^16; no video shape, no
# recomputation.  Expressed here as T = m, Hs = 1, Ws = b.
for _lg in range(10, 17):
    _n = f"kernel-bench-{1 << (_lg - 10)}k"
    WORKLOADS[_n] = Workload(_n, 10 + _lg, 1, 12, 32, 1, (1 << _lg) // 32, 64, "bf16", 2, False)


# The paper's study of computation budgets (App. "Various Monarch Computation Budgets"): one sequence of
# N = 2^15 tokens factored as m blocks of b tokens for every power-of-two split from (8, 4096) to (512, 64);
# the arithmetic is smallest near m = b = sqrt(N), the traffic falls as b grows.  d = 64, 12 heads, 2 sweeps as
# in the kernel benchmark above (the appendix gives figures only, no numbers).
BUDGET_SPLITS = [(8, 4096), (16, 2048), (32, 1024), (64, 512), (128, 256), (256, 128), (512, 64)]
for _m, _b in BUDGET_SPLITS:
    _n = f"budget-{_m}x{_b}"
    WORKLOADS[_n] = Workload(_n, 30 + _m.bit_length(), 1, 12, _m, 1, _b, 64, "bf16", 2, False)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bf16 bit patterns (uint16)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def positional_features(T: int, Hs: int, Ws: int) -> np.ndarray:
    """phi for every token in (t, y, x) order with x fastest: (N, 6F) float32."""
    t, y, x = np.meshgrid(np.arange(T), np.arange(Hs), np.arange(Ws), indexing="ij")
    cols = []
    for coord, extent in ((t, T), (y, Hs), (x, Ws)):
        c = coord.reshape(-1).astype(np.float64) / float(extent)
        for r in range(1, F_BANDS + 1):
            cols.append(np.sin(2.0 * math.pi * r * c))
            cols.append(np.cos(2.0 * math.pi * r * c))
    return np.stack(cols, axis=1).astype(np.float32)


def head_inputs(T, Hs, Ws, d, config, head, gain=None, sink=0.0, phi=None):
    """float32 q, k, v of shape (N, d) for one (batch*head) index, and the gain used."""
    rng = np.random.Generator(np.random.Philox(BASE_SEED + 1000 * config + head))
    if phi is None:
        phi = positional_features(T, Hs, Ws)
    N = phi.shape[0]
    nf = phi.shape[1]
    w_qk = rng.standard_normal((nf, d), dtype=np.float32) / np.float32(math.sqrt(nf))
    w_v = rng.standard_normal((nf, d), dtype=np.float32) / np.float32(math.sqrt(nf))
    base = phi @ w_qk
    q = np.float32(0.5) * rng.standard_normal((N, d), dtype=np.float32) + base
    k = np.float32(0.5) * rng.standard_normal((N, d), dtype=np.float32) + base
    v = np.float32(0.5) * rng.standard_normal((N, d), dtype=np.float32) + phi @ w_v
    if sink > 0.0:
        u = rng.standard_normal(d, dtype=np.float32)
        u /= np.linalg.norm(u)
        q += np.float32(sink) * u
        k[: Hs * Ws] += np.float32(sink) * u
    if gain is None:
        pa = rng.integers(0, N, size=65536)
        pb = rng.integers(0, N, size=65536)
        logits = np.einsum("nd,nd->n", q[pa].astype(np.float64), k[pb].astype(np.float64)) / math.sqrt(d)
        sd = float(logits.std())
        gain = math.sqrt(3.0 / sd) if sd > 1e-6 else 1.0   # a single token has no spread to normalise
    q *= np.float32(gain)
    k *= np.float32(gain)
    return q, k, v, float(gain)


def make_inputs(wl: Workload, heads=None, sink=0.0):
    """q, k, v for a workload, shape (B*heads_selected, N, d).

    dtype "f32": float32 arrays.  dtype "bf16": uint16 bit patterns.
    ``heads`` optionally restricts to a list of (batch*head) indices.
    """
    idx = list(range(wl.B * wl.heads)) if heads is None else list(heads)
    phi = positional_features(wl.T, wl.Hs, wl.Ws)
    bf16 = wl.dtype == "bf16"
    dt = np.uint16 if bf16 else np.float32
    q = np.empty((len(idx), wl.N, wl.d), dtype=dt)
    k = np.empty_like(q)
    v = np.empty_like(q)
    for o, h in enumerate(idx):
        qh, kh, vh, _ = head_inputs(wl.T, wl.Hs, wl.Ws, wl.d, wl.config, h,
                                    gain=None if bf16 else 1.0, sink=sink, phi=phi)
        if bf16:
            q[o], k[o], v[o] = f32_to_bf16_bits(qh), f32_to_bf16_bits(kh), f32_to_bf16_bits(vh)
        else:
            q[o], k[o], v[o] = qh, kh, vh
    return q, k, v


def algorithmic_flops(B, heads, T, b, d, iters, recompute):
    """Floating-point operations the method itself needs per call.

    R sweep = logits + R K (4 T b^2 d); the last R sweep also forms R V
    (6 T b^2 d); an L sweep = logits + L^T Q or L y (4 b T^2 d); the
    first-frame recomputation is b queries against all N keys (4 b N d).
    """
    N = T * b
    per = (iters - 1) * 4 * T * b * b * d + 6 * T * b * b * d + iters * 4 * b * T * T * d
    if recompute:
        per += 4 * b * N * d
    return B * heads * per

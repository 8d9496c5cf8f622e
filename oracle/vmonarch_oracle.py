"""Plain fp64 NumPy oracle for VMonarch's spatio-temporal Monarch attention.

TEST INFRASTRUCTURE ONLY.  This file is the slow, explicit statement of what
the method computes, written from the paper (Sec. 3.1 Eqs. R / alpha_R / c_R /
L / alpha_L / c_L, Sec. 3.2, Sec. 3.3 first-frame recomputation, Sec. 3.4
Alg. 1, App. A, App. B).  It shares no code with the HIP library and is never
imported by it.  Only tests, the smoke check and the benchmark's CPU-baseline
leg may call it.

Notation (the paper's): m = T frames, b = H*W spatial positions, N = m*b,
token n = j*b + i with j the frame and i the position (App. A reshape(m,b,d)).
Index letters: j query frame, i query position, k key frame, l key position,
v channel.  Factors: R = diag(R_0..R_{m-1}), R_k is b x b (spatial, one block
per frame); L = diag(L_0..L_{b-1}), L_i is m x m (temporal, one block per
position).  Monarch entry (Sec. 3.1): M[(j,i),(k,l)] = L[i][j,k] * R[k][i,l].

Readings taken where the paper is silent or inconsistent:
  * 1/sqrt(d): printed only in the recomputation formula (Sec. 3.3).  Here Q is
    replaced by Q/sqrt(d) everywhere it appears, so the fitted objective is
    <M, Q K^T / sqrt(d)> + H(M) and the T=1 / b=1 collapses give textbook
    scaled attention.
  * Eq. (L) prints softmax_j; App. A takes the softmax over the key-frame axis
    (dim=2).  The code's reading is used: L[i][j,:] is a distribution over k.
  * "clamp c_R to 0.1" (Sec. 4.1): a lower bound applied where c_R divides,
    c = max(c_R, cr_min).  The c_R the L-update emits is left unclamped.
  * 0*log(0) := 0 in c_L.
  * Recomputation overwrites only the output rows of frame 0; the fit is not
    changed by it.
  * Manual control: "first frame" is the key-frame index k = 0 of c_R[k, i] and
    c_L[i, k]; the overwrite happens right after the update that produces the
    term, in every sweep; the c_L constant is a parameter whose default is
    -log b (the paper's log M for the entropy of a uniform row, with this
    file's sign c_L = -H).

Pins (tests/test_oracle_*.py): NumPy reshape/transpose for the permutation;
row-stochastic R, L, M; O == M V with M formed densely; T=1 and b=1 collapse
to textbook softmax attention; separable logits give exact softmax attention
for every iteration count; brute-force entropy against c_L and against the
online accumulator; objective non-decreasing over half-steps and bounded by
the sum of row log-sum-exps; sum_k c_R[k,i] = T; V == 1 gives O == 1.
Variants (sink averaging, manual c_R / c_L): with one sweep c_R control changes
nothing (rows 2 = 3 = 7, 4 = 5 and 6 = 1 of the paper's control table); c_L
fixed for all frames is independent of the value; a very negative first-frame
c_L collapses every output to spatial attention within frame 0; frames whose
c_R is not overwritten keep their R; sink averaging at T = 1 is textbook
attention and is linear in V with half the Monarch response outside frame 0.
Backward (Alg. 2): central finite differences of <dO, O> + <dH, H> through
entropy_attention in every input, rows of dS summing to zero, one-key blocks.
No worked numeric example is printed in the paper, so no paper value pins it.
"""
from __future__ import annotations

import math

import numpy as np


# --------------------------------------------------------------------------
# input widening (the oracle's own; the HIP side never sees this)
# --------------------------------------------------------------------------
def widen_bf16(bits: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> float64, exactly."""
    u = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


# --------------------------------------------------------------------------
# Sec. 3.1 permutation P_(b,N): the footnote's definition
# --------------------------------------------------------------------------
def index_maps(m: int, b: int):
    """perm, inv as int32[N].

    Footnote of Sec. 3.1: reshape a length-N vector into an m x b row-major
    matrix, transpose, flatten.  Position-major slot p = i*m + j holds token
    perm[p] = j*b + i; inv is its inverse, inv[j*b + i] = i*m + j.
    (The printed sigma formula is the identity map and is not used.)
    """
    n = m * b
    perm = np.empty(n, dtype=np.int32)
    inv = np.empty(n, dtype=np.int32)
    for p in range(n):
        i, j = divmod(p, m)
        perm[p] = j * b + i
    for t in range(n):
        j, i = divmod(t, b)
        inv[t] = i * m + j
    return perm, inv


# --------------------------------------------------------------------------
# textbook pieces
# --------------------------------------------------------------------------
def softmax_rows(z: np.ndarray) -> np.ndarray:
    """softmax over the last axis."""
    e = np.exp(z - z.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def softmax_attention(Q, K, V, scale):
    """softmax(scale * Q K^T) V, the dense definition."""
    return softmax_rows(scale * (Q @ K.T)) @ V


def neg_entropy_rows(P: np.ndarray) -> np.ndarray:
    """sum over the last axis of P log P with 0 log 0 := 0."""
    safe = np.where(P > 0.0, P, 1.0)
    return (P * np.log(safe)).sum(axis=-1)


# --------------------------------------------------------------------------
# Sec. 3.1: the two closed-form half-steps, written from Eqs. (R), (alpha_L, c_L),
# (L), (alpha_R, c_R) with the paper's index letters: j query frame, i query
# position, k key frame, l key position, v channel.  One block at a time, every
# block formed explicitly.  Storage here is [k][i] for the spatial side and [i][k]
# for the temporal side, as the subscripts of the equations read.
# --------------------------------------------------------------------------
def r_update(alpha_R, c_R, K, cr_min=0.0):
    """Spatial half-step.  Eq. (R): R_k[i, l] = softmax_l(sum_v alpha_R[k,i,v] K[k,l,v] / c_R[k,i]);
    Eq. (alpha_L, c_L): alpha_L[i,k,v] = sum_l R_k[i,l] K[k,l,v], c_L[i,k] = sum_l R_k[i,l] log R_k[i,l].

    alpha_R (m, s, d), c_R (m, s), K (m, b, d); s query positions (s == b for the full
    problem, fewer when only some positions are followed).  c_R is bounded below by cr_min
    where it divides (Sec. 4.1).  Returns alpha_L (s, m, d), c_L (s, m), R (m, s, b).
    """
    m, s, d = alpha_R.shape
    b = K.shape[1]
    R = np.empty((m, s, b))
    alpha_L = np.empty((s, m, d))
    c_L = np.empty((s, m))
    for k in range(m):                                   # one b x b block per key frame
        temperature = np.maximum(c_R[k], cr_min)                         # (s,)
        logits_il = (alpha_R[k] @ K[k].T) / temperature[:, None]      # sum over v -> [i, l]
        R_k = softmax_rows(logits_il)                                    # over l
        R[k] = R_k
        alpha_L[:, k, :] = R_k @ K[k]                                    # sum over l -> [i, v]
        c_L[:, k] = neg_entropy_rows(R_k)
    return alpha_L, c_L, R


def l_update(alpha_L, c_L, Q):
    """Temporal half-step.  Eq. (L): L_i[j, k] = softmax over k of (sum_v alpha_L[i,k,v] Q[i,j,v] - c_L[i,k])
    (a distribution over key frames for every query frame: the reading that keeps M
    row-stochastic); Eq. (alpha_R, c_R): alpha_R[k,i,v] = sum_j L_i[j,k] Q[i,j,v],
    c_R[k,i] = sum_j L_i[j,k].

    alpha_L (s, m, d), c_L (s, m), Q (s, m, d) position-major (Q[i, j] is the query of
    frame j at position i, already carrying 1/sqrt(d)).
    Returns alpha_R (m, s, d), c_R (m, s), L (s, m, m) with L[i][j, k].
    """
    s, m, d = Q.shape
    L = np.empty((s, m, m))
    alpha_R = np.empty((m, s, d))
    c_R = np.empty((m, s))
    for i in range(s):                                   # one m x m block per position
        logits_jk = (Q[i] @ alpha_L[i].T) - c_L[i][None, :]              # sum over v -> [j, k]
        L_i = softmax_rows(logits_jk)                                    # over k
        L[i] = L_i
        alpha_R[:, i, :] = L_i.T @ Q[i]                                  # sum over j -> [k, v]
        c_R[:, i] = L_i.sum(axis=0)                                      # over j
    return alpha_R, c_R, L


def monarch_apply(L, R, V):
    """O = M V with M[(j,i),(k,l)] = L_i[j,k] R_k[i,l] (Sec. 3.1), without forming M:
    y[i,k,v] = sum_l R_k[i,l] V[k,l,v], then O[j,i,v] = sum_k L_i[j,k] y[i,k,v].

    L (s, m, m), R (m, s, b), V (m, b, d).  Returns O (m, s, d) and y (s, m, d).
    """
    s, m, _ = L.shape
    d = V.shape[2]
    y = np.empty((s, m, d))
    for k in range(m):
        y[:, k, :] = R[k] @ V[k]                        # sum over l -> [i, v]
    O = np.empty((m, s, d))
    for i in range(s):
        O[:, i, :] = L[i] @ y[i]                        # sum over k -> [j, v]
    return O, y


# --------------------------------------------------------------------------
# Sec. 3.1 alternating maximisation + Sec. 3.3 recomputation
# --------------------------------------------------------------------------
def monarch_attention(Q, K, V, m, b, iters, recompute=False, cr_min=0.1,
                      positions=None, keep_factors=False, sink_average=False,
                      cr_control=0, cl_control=0, cl_value=None):
    """Spatio-temporal Monarch attention for one (batch, head).

    Q, K, V: (N, d) float64, N = m*b, token n = j*b + i.
    positions: optional 1-D int array of query positions i to follow.  The
    whole iteration for a position depends only on Q[:, i, :] and on all of
    K, V, so a subset is followed exactly.  None means all b positions.

    Returns a dict:
      O      (m, s, d)   output rows for the followed positions, O[j, idx]
      aL,cL  (s, m, d), (s, m)  from the last R-update
      aR,cR  (m, s, d), (m, s)  from the last L-update (unclamped c_R)
      y      (s, m, d)   R V of the last sweep
      trace  list of per-sweep dicts (aL, cL, aR, cR [, R, L])
      R, L   last factors, only when keep_factors
    With recompute, O[0] is replaced by exact attention of the frame-0 queries
    over all N keys (Sec. 3.3); nothing else changes.

    Ablation variants (Sec. 4.4 and App. "Manual Control of Monarch Parameters"):
      sink_average  O <- (softmax(Q K_F1^T / sqrt(d)) V_F1 + O) / 2, every query
                    against the first frame's keys and values only.
      cr_control    after every L-update overwrite c_R with 1: 0 never, 1 for
                    the first frame (k = 0), 2 for all frames.
      cl_control    after every R-update overwrite c_L with cl_value: 0 never,
                    1 for the first frame (k = 0), 2 for all frames.  cl_value
                    defaults to the c_L of a uniform row of the b x b factor,
                    sum (1/b) log(1/b) = -log b in this file's sign convention.
    """
    N, d = Q.shape
    assert N == m * b and K.shape == (N, d) and V.shape == (N, d) and iters >= 1
    inv_sqrt_d = 1.0 / math.sqrt(d)
    pos = np.arange(b) if positions is None else np.asarray(positions, dtype=np.int64)
    s = len(pos)
    K_kl = K.reshape(m, b, d)                       # K[k, l, v]
    V_kl = V.reshape(m, b, d)
    Q_ji = (Q * inv_sqrt_d).reshape(m, b, d)[:, pos, :]   # scaled queries, [j, i, v]
    Q_ij = np.ascontiguousarray(Q_ji.transpose(1, 0, 2))  # the same rows position-major, [i, j, v]
    if cl_value is None:
        cl_value = -math.log(b)
    # L = identity to start with: Eq. (alpha_R, c_R) then gives alpha_R[k,i] = Q[i,k], c_R = 1
    alpha_R = Q_ji.copy()
    c_R = np.ones((m, s))
    trace = []
    for _ in range(iters):
        alpha_L, c_L, R = r_update(alpha_R, c_R, K_kl, cr_min)
        if cl_control == 1:
            c_L[:, 0] = cl_value
        elif cl_control == 2:
            c_L[:, :] = cl_value
        alpha_R, c_R, L = l_update(alpha_L, c_L, Q_ij)
        if cr_control == 1:
            c_R[0, :] = 1.0
        elif cr_control == 2:
            c_R[:, :] = 1.0
        step = dict(aL=alpha_L, cL=c_L, aR=alpha_R, cR=c_R)
        if keep_factors:
            step.update(R=R, L=L)
        trace.append(step)
    O, y = monarch_apply(L, R, V_kl)
    if recompute:
        O[0] = softmax_attention(Q.reshape(m, b, d)[0, pos, :], K, V, inv_sqrt_d)
    if sink_average:
        Qrows = Q.reshape(m, b, d)[:, pos, :].reshape(-1, d)
        sink = softmax_attention(Qrows, K[:b], V[:b], inv_sqrt_d).reshape(m, s, d)
        O = 0.5 * (sink + O)
    out = dict(O=O, aL=alpha_L, cL=c_L, aR=alpha_R, cR=c_R, y=y, trace=trace, positions=pos)
    if keep_factors:
        out.update(R=R, L=L)
    return out


def first_frame_attention(Q, K, V, b, rows=None):
    """Sec. 3.3: softmax(Q_0 K^T / sqrt(d)) V for frame-0 queries (tokens 0..b-1)."""
    d = Q.shape[1]
    r = np.arange(b) if rows is None else np.asarray(rows, dtype=np.int64)
    return softmax_attention(Q[r], K, V, 1.0 / math.sqrt(d))


# --------------------------------------------------------------------------
# Sec. 3.1: the dense Monarch matrix and the objective of Eq. 1 / Eq. 2
# --------------------------------------------------------------------------
def dense_monarch(L, R):
    """M[(j,i),(k,l)] = L[i][j,k] * R[k][i,l] as an (N, N) array, N = m*b.

    L (b, m, m), R (m, b, b): all positions present.
    """
    b, m, _ = L.shape
    M = np.empty((m, b, m, b))
    for j in range(m):
        for i in range(b):
            for k in range(m):
                M[j, i, k, :] = L[i, j, k] * R[k, i, :]
    return M.reshape(m * b, m * b)


def monarch_product(L, R, m, b):
    """P L P^T R with explicit block-diagonal and permutation matrices (Sec. 3.1)."""
    n = m * b
    perm, _ = index_maps(m, b)
    P = np.zeros((n, n))
    # P x = "reshape m x b, transpose, flatten": (P x)[p] = x[perm[p]]
    P[np.arange(n), perm] = 1.0
    Lbd = np.zeros((n, n))
    for i in range(b):
        Lbd[i * m:(i + 1) * m, i * m:(i + 1) * m] = L[i]
    Rbd = np.zeros((n, n))
    for k in range(m):
        Rbd[k * b:(k + 1) * b, k * b:(k + 1) * b] = R[k]
    # Rows of L_i are indexed by (i, j) = position-major, so the product that
    # acts on frame-major tokens is P^T L P R.  With the footnote's P this is
    # the paper's M up to which of P, P^T is named "the" permutation.
    return P.T @ Lbd @ P @ Rbd


def objective(M, Q, K):
    """Eq. 1: <M, Q K^T / sqrt(d)> + H(M), H the Shannon entropy summed over entries."""
    d = Q.shape[1]
    S = (Q @ K.T) / math.sqrt(d)
    return float((M * S).sum() - neg_entropy_rows(M).sum())


def objective_upper_bound(Q, K):
    """max over row-stochastic A of Eq. 1 = sum over rows of logsumexp(Q K^T / sqrt(d))."""
    d = Q.shape[1]
    S = (Q @ K.T) / math.sqrt(d)
    mx = S.max(axis=1)
    return float((mx + np.log(np.exp(S - mx[:, None]).sum(axis=1))).sum())


# --------------------------------------------------------------------------
# App. B online softmax / online entropy, and Alg. 1
# --------------------------------------------------------------------------
def online_entropy_state(x):
    """App. B: one pass over the vector x keeping (m_i, S_i, L_i).

    Returns (m, S, Lsum) with S = sum exp(x - m), Lsum = sum exp(x - m) (x - m).
    """
    m_run = -math.inf
    S = 0.0
    Lsum = 0.0
    for xi in x:
        m_new = max(m_run, xi)
        if m_new > m_run and S > 0.0:
            alpha = math.exp(m_run - m_new)
            # L <- L alpha + S alpha log(alpha);  S <- S alpha
            Lsum = Lsum * alpha + S * alpha * (m_run - m_new)
            S = S * alpha
        p = math.exp(xi - m_new)
        S = S + p
        Lsum = Lsum + p * (xi - m_new)
        m_run = m_new
    return m_run, S, Lsum


def online_entropy(x):
    """App. B final formula: H(p) = log S_N - L_N / S_N."""
    _, S, Lsum = online_entropy_state(x)
    return math.log(S) - Lsum / S


def merge_entropy_states(a, b_):
    """Combine the states of two disjoint parts of a vector (same rescale rule)."""
    (m1, S1, L1), (m2, S2, L2) = a, b_
    mm = max(m1, m2)
    a1 = math.exp(m1 - mm)
    a2 = math.exp(m2 - mm)
    S = S1 * a1 + S2 * a2
    Ls = L1 * a1 + S1 * a1 * (m1 - mm) + L2 * a2 + S2 * a2 * (m2 - mm)
    return mm, S, Ls


def flash_entropy_attention(Q, K, V, Br, Bc):
    """Alg. 1 (forward): blocked attention with running max, sum and entropy.

    Q (Nq, d), K, V (Nk, d) float64, logits S = Q K^T (the caller scales Q).
    Returns O (Nq, d), LSE (Nq,), H (Nq,).
    """
    Nq, d = Q.shape
    Nk = K.shape[0]
    O = np.zeros((Nq, V.shape[1]))
    LSE = np.zeros(Nq)
    H = np.zeros(Nq)
    for r0 in range(0, Nq, Br):
        Qi = Q[r0:r0 + Br]
        nr = Qi.shape[0]
        mi = np.full(nr, -np.inf)
        li = np.zeros(nr)
        hi = np.zeros(nr)
        Oi = np.zeros((nr, V.shape[1]))
        for c0 in range(0, Nk, Bc):
            Kj = K[c0:c0 + Bc]
            Vj = V[c0:c0 + Bc]
            Sij = Qi @ Kj.T
            m_new = np.maximum(mi, Sij.max(axis=1))
            Pij = np.exp(Sij - m_new[:, None])
            alpha = np.exp(mi - m_new)                      # 0 on the first tile
            # alpha log(alpha) -> 0 as alpha -> 0
            alogal = np.where(alpha > 0.0, alpha * np.log(np.where(alpha > 0.0, alpha, 1.0)), 0.0)
            Oi = alpha[:, None] * Oi + Pij @ Vj
            hi = alpha * hi + alogal * li + neg_entropy_rows(Pij)
            li = alpha * li + Pij.sum(axis=1)
            mi = m_new
        O[r0:r0 + Br] = Oi / li[:, None]
        LSE[r0:r0 + Br] = mi + np.log(li)
        H[r0:r0 + Br] = np.log(li) - hi / li
    return O, LSE, H


# --------------------------------------------------------------------------
# analytic counts (Sec. 3.2 complexity, Sec. 3.3 overhead, Sec. 4.1 sparsity)
# --------------------------------------------------------------------------
# --------------------------------------------------------------------------
# App. "Backward pass of Flash-Entropy-Attention", Alg. 2 (dense form)
# --------------------------------------------------------------------------
def entropy_attention(Q, K, V, row_scale):
    """One softmax block with its row entropy, from the definitions.

    z[i,l] = row_scale[i] * (Q[i] . K[l]);  P = softmax_l z;  O = P V;
    lse[i] = log sum_l exp z[i,l] (Alg. 1's L);  H[i] = -sum_l P log P.
    Returns (O, lse, H).
    """
    z = (Q @ K.T) * np.asarray(row_scale, dtype=np.float64).reshape(-1, 1)
    zmax = z.max(axis=1, keepdims=True)
    e = np.exp(z - zmax)
    ssum = e.sum(axis=1, keepdims=True)
    P = e / ssum
    lse = (zmax + np.log(ssum))[:, 0]
    return P @ V, lse, -neg_entropy_rows(P)


def entropy_attention_backward(Q, K, V, O, dO, lse, H, dH, row_scale):
    """Alg. 2 without the blocking: the steps of its inner loop on whole matrices.

    S is the scaled logit matrix z above.  D = rowsum(dO o O); P = exp(S - lse);
    dV = P^T dO; dP = dO V^T; dS = P o (dP - D) - dH o P o (S - lse + H);
    dQ = dS K and dK = dS^T Q, each carrying the row's logit scale (S = scale * Q K^T).
    dH = None stands for all zeros (no gradient through the entropy).
    Returns (dQ, dK, dV).
    """
    sc = np.asarray(row_scale, dtype=np.float64).reshape(-1, 1)
    S = (Q @ K.T) * sc
    D = (dO * O).sum(axis=1, keepdims=True)
    P = np.exp(S - lse.reshape(-1, 1))
    dV = P.T @ dO
    dP = dO @ V.T
    dS = P * (dP - D)
    if dH is not None:
        dS = dS - dH.reshape(-1, 1) * P * (S - lse.reshape(-1, 1) + H.reshape(-1, 1))
    dQ = (dS * sc) @ K
    dK = (dS * sc).T @ Q
    return dQ, dK, dV


def sparsity_estimate(T, HW, t):
    """Sec. 4.1: 1 - t (T + HW) / (T HW)."""
    return 1.0 - t * (T + HW) / (T * HW)


def recompute_cost_ratio(m, b, t):
    """Sec. 3.3: cost of the recomputation relative to the t sweeps, b / (t (m + b))."""
    return b / (t * (m + b))

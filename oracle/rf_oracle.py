"""CPU oracle for cascaded reductions (test infrastructure, NOT a product path).

This file is test infrastructure: only the tests, the smoke check and the
benchmark's cpu-baseline leg may import it.  It shares no code with the HIP
library and imports nothing from it.  Everything is float64 numpy, multi-pass
and unfused: each function evaluates the plain definition of a chain of
dependent reductions, one reduction after the other, each re-reading its
input, exactly the "chain of reduction trees" the paper starts from
(Section 3.1, Eq. (1)).  A matmul is used as a library step where the
definition contains one.

Two groups of functions:

* ``safe_softmax``, ``attention``, ``attention_partial_states``,
  ``merge_states``, ``rmsnorm_gemm``, ``variance``, ``moe_routing``: the
  definitions the GPU results are compared against; ``fp8_quant_gemm``: the
  tile-by-tile incremental algorithm of the quantised cascade (the one case
  here whose single-pass result is not that of the multi-pass definition,
  because rounding to FP8 sits between the two reductions).
* ``*_incremental`` and ``fused_*``: the paper's fused / incremental forms
  (Section 3.2 Eq. (6), (8), (11); Section 3.3 Eq. (15)-(16); Appendix A.2) written out
  step by step in the paper's order.  They exist so that the tests can check
  the paper's equivalence claim on tiny inputs; the GPU parity tests do not use
  them.

Readings of the paper taken here (each is also listed in the design notes):
  * the softmax scale 1/sqrt(d_k) multiplies Q K^T before the row max
    (Appendix A.2, definition of P); the code listings leave it out;
  * the level-1 fused / incremental attention equations of Appendix A.2 lose
    the factor V[l]; it is restored (the definition and the listings have it);
  * the combine step weights chunk c by t_c * exp(m_c - m) / t with the
    *unscaled* t_c (Appendix A.2, level-k equation); the printed combine
    listing applies the exponential twice;
  * a causal mask removes key j from all three reductions of query i unless
    j <= i + (Lk - Lq); grouped KV heads: query head h reads KV head
    h // (Hq // Hkv);
  * an empty index set gives the identity state (m=-inf, t=0, acc=0) and an
    output row of zeros (Appendix A.1: a non-invertible H is replaced by the
    identity of the combine operator);
  * RMSNorm + linear: H(ss) = (ss/K + eps)^(-1/2), eps added to the mean of
    squares; the clamp printed in the "Sum + Sum" example is garbled and is not
    used;
  * variance (Appendix, non-ML workloads) is the population variance (both
    reductions divide by L0).  Its second map (x - m)^2 is not of the form
    G(x) (x) H(m); the fused forms expand the square into decomposable terms,
    which gives the pairwise update of (count, mean, M2);
  * MoE routing (Appendix A.2): TopK acts on the raw scores (softmax keeps
    their order) and the final "s / t" is read as exp(s - m) / t, the softmax
    probability of each selected expert.  Equal scores are ordered by expert
    index, lowest first, and the k outputs are in descending order of score;
  * FP8 per-token quant + GEMM (Section 3.4): FP8 is OCP E4M3 (MAX = 448),
    rounding to nearest even, values beyond MAX saturate.  The scale MAX / m
    and the product a * scale are taken in float32 (they decide the FP8 code,
    so both sides of a comparison must use one precision); everything else is
    float64.  The weights arrive already in FP8.  The paper's c = sum (MAX a / m) w
    is the quantised-domain sum; the returned value undoes the scale,
    c * m / MAX, so that it approximates a @ w.  An all-zero token has m = 0: its
    scale is taken as 0 and its output row is 0.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64
NEG_INF = -np.inf


# --------------------------------------------------------------------------
# O1. safe softmax  (Section 2.2; Appendix A.2 first two reductions)
# --------------------------------------------------------------------------
def safe_softmax(x):
    """Row-wise safe softmax over the last axis, three passes per row.

    pass 1: m = max_j x[j];  pass 2: t = sum_j exp(x[j] - m);
    pass 3: y[j] = exp(x[j] - m) / t.   (Section 2.2, safe softmax.)
    """
    x = np.asarray(x, dtype=F64)
    m = np.max(x, axis=-1, keepdims=True)                     # reduction 1
    t = np.sum(np.exp(x - m), axis=-1, keepdims=True)         # reduction 2
    return np.exp(x - m) / t                                  # normalise


# --------------------------------------------------------------------------
# O2. attention  (Appendix A.2, Eq. "attention reductions"; unfused listing)
# --------------------------------------------------------------------------
def _visible(lq, lk, causal):
    """Boolean [lq, lk] mask: query i sees key j iff j <= i + (lk - lq)."""
    if not causal:
        return np.ones((lq, lk), dtype=bool)
    i = np.arange(lq)[:, None]
    j = np.arange(lk)[None, :]
    return j <= i + (lk - lq)


def attention(q, k, v, scale, causal=False):
    """O = softmax(scale * Q K^T) V, evaluated as four separate reductions.

    q [B,Hq,Lq,d]; k, v [B,Hkv,Lk,d]; Hq % Hkv == 0.  For each (b, h):
    reduction 1  P = scale * Q K^T            (over d)
    reduction 2  m = max_j P[., j]            (visible j only)
    reduction 3  t = sum_j exp(P[., j] - m)
    reduction 4  O = sum_j exp(P[., j] - m) / t * V[j]
    A row with no visible key yields zeros.
    """
    q = np.asarray(q, dtype=F64)
    k = np.asarray(k, dtype=F64)
    v = np.asarray(v, dtype=F64)
    B, Hq, Lq, d = q.shape
    _, Hkv, Lk, _ = k.shape
    assert Hq % Hkv == 0 and k.shape[:3] == v.shape[:3] and k.shape[0] == B and k.shape[3] == d
    grp = Hq // Hkv
    vis = _visible(Lq, Lk, causal)
    out = np.zeros((B, Hq, Lq, v.shape[3]), dtype=F64)
    for b in range(B):
        for h in range(Hq):
            kh = h // grp
            P = scale * (q[b, h] @ k[b, kh].T)                # reduction 1
            P = np.where(vis, P, NEG_INF)
            m = np.max(P, axis=1, keepdims=True)              # reduction 2
            m_safe = np.where(np.isfinite(m), m, 0.0)
            E = np.where(vis, np.exp(P - m_safe), 0.0)
            t = np.sum(E, axis=1, keepdims=True)              # reduction 3
            t_safe = np.where(t > 0.0, t, 1.0)
            out[b, h] = (E / t_safe) @ v[b, kh]               # reduction 4
    return out


def attention_rows(q, k, v, scale, causal, rows):
    """Same definition as ``attention`` for a list of (b, h, i) rows only.

    Used for sampled parity at sizes where the whole output is too slow on a
    CPU.  Returns an array [len(rows), d].
    """
    k = np.asarray(k)
    B, Hq, Lq, d = q.shape
    _, Hkv, Lk, _ = k.shape
    grp = Hq // Hkv
    out = np.zeros((len(rows), v.shape[3]), dtype=F64)
    for n, (b, h, i) in enumerate(rows):
        kh = h // grp
        nvis = min(Lk, i + (Lk - Lq) + 1) if causal else Lk
        if nvis <= 0:
            continue
        kk = np.asarray(k[b, kh, :nvis], dtype=F64)
        vv = np.asarray(v[b, kh, :nvis], dtype=F64)
        p = scale * (kk @ np.asarray(q[b, h, i], dtype=F64))
        m = np.max(p)
        e = np.exp(p - m)
        t = np.sum(e)
        out[n] = (e / t) @ vv
    return out


# --------------------------------------------------------------------------
# O3. split into segments + merge  (Section 4.3 multi-segment; Eq. (11);
#     Appendix A.2 level-k equations)
# --------------------------------------------------------------------------
def split_bounds(Lk, num_splits):
    """Chunk c covers keys [c*ceil(Lk/S), min(Lk, (c+1)*ceil(Lk/S)))."""
    step = -(-Lk // num_splits)
    return [(min(Lk, c * step), min(Lk, (c + 1) * step)) for c in range(num_splits)]


def attention_partial_states(q, k, v, scale, causal, num_splits):
    """Per-chunk states (m_c, t_c, acc_c) with acc_c = sum_j exp(P[j]-m_c) V[j].

    Each chunk runs reductions 2-4 of ``attention`` over its own keys only,
    without the final division (Eq. (8): the H-free partial reduction).
    Returns m, t of shape [B,Hq,Lq,S] and acc of shape [B,Hq,Lq,S,d].
    """
    q = np.asarray(q, dtype=F64)
    k = np.asarray(k, dtype=F64)
    v = np.asarray(v, dtype=F64)
    B, Hq, Lq, d = q.shape
    _, Hkv, Lk, _ = k.shape
    grp = Hq // Hkv
    S = num_splits
    vis = _visible(Lq, Lk, causal)
    pm = np.full((B, Hq, Lq, S), NEG_INF, dtype=F64)
    pt = np.zeros((B, Hq, Lq, S), dtype=F64)
    pacc = np.zeros((B, Hq, Lq, S, v.shape[3]), dtype=F64)
    for c, (lo, hi) in enumerate(split_bounds(Lk, S)):
        if hi <= lo:
            continue
        for b in range(B):
            for h in range(Hq):
                kh = h // grp
                P = scale * (q[b, h] @ k[b, kh, lo:hi].T)
                vz = vis[:, lo:hi]
                P = np.where(vz, P, NEG_INF)
                m = np.max(P, axis=1)
                m_safe = np.where(np.isfinite(m), m, 0.0)
                E = np.where(vz, np.exp(P - m_safe[:, None]), 0.0)
                pm[b, h, :, c] = m
                pt[b, h, :, c] = np.sum(E, axis=1)
                pacc[b, h, :, c, :] = E @ v[b, kh, lo:hi]
    return pm, pt, pacc


def merge_states(pm, pt, pacc):
    """Combine chunk states, multi-pass (Appendix A.2, level-k fused form).

    m = max_c m_c;  t = sum_c t_c exp(m_c - m);
    O = sum_c acc_c exp(m_c - m) / t.   Rows with t == 0 give zeros.
    """
    pm = np.asarray(pm, dtype=F64)
    pt = np.asarray(pt, dtype=F64)
    pacc = np.asarray(pacc, dtype=F64)
    m = np.max(pm, axis=-1, keepdims=True)
    m_safe = np.where(np.isfinite(m), m, 0.0)
    w = np.where(np.isfinite(pm), np.exp(pm - m_safe), 0.0)   # exp(m_c - m)
    t = np.sum(pt * w, axis=-1, keepdims=True)
    t_safe = np.where(t > 0.0, t, 1.0)
    return np.sum(pacc * (w / t_safe)[..., None], axis=-2)


# --------------------------------------------------------------------------
# O4. RMSNorm fused with a linear layer ("Sum + Sum" template, Appendix A.2)
# --------------------------------------------------------------------------
def rmsnorm_gemm(x, g, w, eps):
    """Y = (X / sqrt(mean(X^2) + eps) * g) W as two reductions over K.

    reduction 1: ss_i = sum_k X[i,k]^2
    reduction 2: Y[i,n] = sum_k X[i,k] g[k] W[k,n] * (ss_i/K + eps)^(-1/2)
    """
    x = np.asarray(x, dtype=F64)
    g = np.asarray(g, dtype=F64)
    w = np.asarray(w, dtype=F64)
    K = x.shape[1]
    ss = np.sum(x * x, axis=1, keepdims=True)                 # reduction 1
    r = 1.0 / np.sqrt(ss / K + eps)
    return ((x * r) * g[None, :]) @ w                         # reduction 2


# --------------------------------------------------------------------------
# O5. The paper's fused and incremental forms, step by step (tiny inputs only)
# --------------------------------------------------------------------------
def _corr(m_old, m_new):
    """exp(m_old - m_new) with the identity repair of Appendix A.1."""
    if m_new == NEG_INF:
        return 1.0
    return float(np.exp(m_old - m_new))


def softmax_incremental(x):
    """Level-1 incremental form of (m, t) for one row, then normalise.

    m[L] = max(m[L-1], x[L]);  t[L] = t[L-1] exp(m[L-1]-m[L]) + exp(x[L]-m[L]).
    """
    x = np.asarray(x, dtype=F64)
    m, t = NEG_INF, 0.0
    for xl in x:
        m_new = max(m, float(xl))
        t = t * _corr(m, m_new) + float(np.exp(xl - m_new))
        m = m_new
    return np.exp(x - m) / t


def attention_incremental_row(qrow, k, v, scale):
    """Level-1 incremental attention for one query, one key at a time, in the
    paper's own order: store previous, correct, reduce; the output is kept
    normalised by t at every step (Appendix A.2, level-1 incremental form,
    with the V[L] factor restored)."""
    qrow = np.asarray(qrow, dtype=F64)
    k = np.asarray(k, dtype=F64)
    v = np.asarray(v, dtype=F64)
    m, t = NEG_INF, 0.0
    o = np.zeros(v.shape[1], dtype=F64)
    for L in range(k.shape[0]):
        p = scale * float(qrow @ k[L])
        m_prev, t_prev = m, t
        m = max(m_prev, p)
        t = t_prev * _corr(m_prev, m) + float(np.exp(p - m))
        o = o * (_corr(m_prev, m) * (t_prev / t)) + (float(np.exp(p - m)) / t) * v[L]
    return o


def fused_segment_state(qrow, k, v, scale):
    """Level-1 fused state of one segment, normalised as the paper writes it:
    (m, t, O) with O = sum_l exp(P[l]-m)/t * V[l] over the segment."""
    qrow = np.asarray(qrow, dtype=F64)
    k = np.asarray(k, dtype=F64)
    v = np.asarray(v, dtype=F64)
    if k.shape[0] == 0:
        return NEG_INF, 0.0, np.zeros(v.shape[1], dtype=F64)
    p = scale * (k @ qrow)
    m = float(np.max(p))
    e = np.exp(p - m)
    t = float(np.sum(e))
    return m, t, (e / t) @ v


def fused_levelk(states):
    """Level-k fused form over a list of normalised (m, t, O) states:
    m = max m_c;  t = sum t_c exp(m_c-m);  O = sum O_c exp(m_c-m) t_c / t."""
    m = max(s[0] for s in states)
    t = sum(s[1] * _corr(s[0], m) for s in states)
    O = sum(s[2] * (_corr(s[0], m) * s[1] / t) for s in states)
    return m, t, O


def incremental_levelk(states):
    """Level-k incremental form: fold normalised (m, t, O) states one by one
    (Appendix A.2, last equation group)."""
    m, t = NEG_INF, 0.0
    O = np.zeros_like(states[0][2])
    for (mc, tc, Oc) in states:
        m_prev, t_prev = m, t
        m = max(m_prev, mc)
        t = t_prev * _corr(m_prev, m) + tc * _corr(mc, m)
        if t > 0.0:
            O = O * (_corr(m_prev, m) * t_prev / t) + Oc * (_corr(mc, m) * tc / t)
    return m, t, O


def attention_tiled_incremental(q, k, v, scale, tile, causal=False):
    """Single-segment strategy on a [Lq,d] x [Lk,d] problem: the running state
    carries the H-free accumulator acc = O*t (Eq. (8)), is rescaled as each
    tile of keys arrives, and is divided by t once at the end."""
    q = np.asarray(q, dtype=F64)
    k = np.asarray(k, dtype=F64)
    v = np.asarray(v, dtype=F64)
    Lq, d = q.shape
    Lk = k.shape[0]
    out = np.zeros((Lq, v.shape[1]), dtype=F64)
    for i in range(Lq):
        nvis = min(Lk, i + (Lk - Lq) + 1) if causal else Lk
        m, t = NEG_INF, 0.0
        acc = np.zeros(v.shape[1], dtype=F64)
        for lo in range(0, max(nvis, 0), tile):
            hi = min(nvis, lo + tile)
            p = scale * (k[lo:hi] @ q[i])
            m_new = max(m, float(np.max(p)))
            c = _corr(m, m_new)
            e = np.exp(p - m_new)
            t = t * c + float(np.sum(e))
            acc = acc * c + e @ v[lo:hi]
            m = m_new
        out[i] = acc / t if t > 0.0 else 0.0
    return out


def rmsnorm_gemm_incremental(x, g, w, eps):
    """Level-1 incremental form (Eq. (16)) of the sum-of-squares -> GEMM
    cascade, one k at a time, keeping y normalised at every step:
      ss[L] = ss[L-1] + x[L]^2
      y[L]  = y[L-1] * H(ss[L-1])^-1 * H(ss[L]) + x[L] g[L] W[L,:] * H(ss[L])
    with H(ss) = (ss/K + eps)^(-1/2)."""
    x = np.asarray(x, dtype=F64)
    g = np.asarray(g, dtype=F64)
    w = np.asarray(w, dtype=F64)
    M, K = x.shape
    H = lambda s: 1.0 / np.sqrt(s / K + eps)
    y = np.zeros((M, w.shape[1]), dtype=F64)
    for i in range(M):
        ss = 0.0
        yi = np.zeros(w.shape[1], dtype=F64)
        for L in range(K):
            ss_prev = ss
            ss = ss_prev + x[i, L] * x[i, L]
            yi = yi * (H(ss) / H(ss_prev)) + (x[i, L] * g[L] * H(ss)) * w[L]
        y[i] = yi
    return y


def rmsnorm_gemm_segments(x, g, w, eps, bounds):
    """Level-k fused form (Eq. (11)) for the same cascade: each K-segment gives
    (ss_c, y_c normalised with its own ss_c); the merge rescales every y_c by
    H(ss_c)^-1 H(ss) and adds."""
    x = np.asarray(x, dtype=F64)
    g = np.asarray(g, dtype=F64)
    w = np.asarray(w, dtype=F64)
    K = x.shape[1]
    H = lambda s: 1.0 / np.sqrt(s / K + eps)
    parts = []
    for lo, hi in bounds:
        ss_c = np.sum(x[:, lo:hi] ** 2, axis=1, keepdims=True)
        y_c = ((x[:, lo:hi] * g[None, lo:hi]) @ w[lo:hi]) * H(ss_c)
        parts.append((ss_c, y_c))
    ss = sum(p[0] for p in parts)
    return sum(p[1] * (H(ss) / H(p[0])) for p in parts)


# --------------------------------------------------------------------------
# Decomposability (Section 4.2, Eq. (23)-(25)): F, and G/H from a fixed point
# --------------------------------------------------------------------------
def F_sumexp(p, m):
    """Mapping function of reduction 3 of attention / 2 of softmax."""
    return np.exp(p - m)


def F_weighted(p, vj, m, t):
    """Mapping function of reduction 4 of attention."""
    return np.exp(p - m) / t * vj


def F_rms(xk, gk, wk, ss, K, eps):
    """Mapping function of reduction 2 of RMSNorm + linear."""
    return xk * gk * wk / np.sqrt(ss / K + eps)


# --------------------------------------------------------------------------
# O6. variance  (Appendix, evaluation on non-ML workloads)
# --------------------------------------------------------------------------
def variance(x):
    """Row-wise mean and population variance as two dependent reductions.

    reduction 1: m = (1/L) sum_l x[l];  reduction 2: var = (1/L) sum_l (x[l]-m)^2.
    Returns (m, var), each of shape x.shape[:-1].
    """
    x = np.asarray(x, dtype=F64)
    L = x.shape[-1]
    m = np.sum(x, axis=-1) / L                                # reduction 1
    d = x - m[..., None]
    var = np.sum(d * d, axis=-1) / L                          # reduction 2
    return m, var


def variance_segment_state(x):
    """Level-1 fused state of one segment: (n, mean, M2) with
    M2 = sum_l (x[l] - mean)^2 over the segment; the empty segment is (0, 0, 0)."""
    x = np.asarray(x, dtype=F64)
    n = x.shape[0]
    if n == 0:
        return 0, 0.0, 0.0
    mean = float(np.sum(x)) / n
    return n, mean, float(np.sum((x - mean) ** 2))


def variance_fused_levelk(states):
    """Level-k fused form over segment states: the mean of the union is the
    count-weighted mean; every segment's M2 is moved to the new mean with
    sum (x-c)^2 = sum (x-mean_s)^2 + n_s (mean_s - c)^2 (the cross term of the
    expanded square vanishes)."""
    n = sum(s[0] for s in states)
    if n == 0:
        return 0, 0.0, 0.0
    mean = sum(s[0] * s[1] for s in states) / n
    m2 = sum(s[2] + s[0] * (s[1] - mean) ** 2 for s in states)
    return n, mean, m2


def variance_incremental(states):
    """Level-k incremental form: fold segment states one by one.  A single
    element is the state (1, x, 0), which gives the level-1 incremental form."""
    n, mean, m2 = 0, 0.0, 0.0
    for (nc, meanc, m2c) in states:
        if nc == 0:
            continue
        n_new = n + nc
        delta = meanc - mean
        mean_new = mean + delta * nc / n_new
        m2 = m2 + m2c + delta * delta * n * nc / n_new
        n, mean = n_new, mean_new
    return n, mean, m2


# --------------------------------------------------------------------------
# O7. MoE routing: scores GEMM -> softmax -> top-k  (Appendix A.2, MoE routing)
# --------------------------------------------------------------------------
def topk_desc(values, k):
    """Indices of the k largest entries of a 1-D array, largest first; equal
    values in ascending index order."""
    values = np.asarray(values, dtype=F64)
    order = sorted(range(values.shape[0]), key=lambda j: (-values[j], j))
    return np.asarray(order[:k], dtype=np.int64)


def moe_routing(x, w, topk):
    """Router of a mixture-of-experts layer, as separate reductions per token.

    reduction 0: p[e] = sum_c x[c] w[c, e]          (the scores GEMM)
    reduction 1: m = max_e p[e]
    reduction 2: t = sum_e exp(p[e] - m)
    reduction 3: s = TopK_e p[e]                    (k largest scores, with their experts)
    output:      exp(s - m) / t                     (softmax probability of the selected experts)
    x [S, hd]; w [hd, E].  Returns (prob [S, topk] float64, idx [S, topk] int64, p [S, E]).
    """
    x = np.asarray(x, dtype=F64)
    w = np.asarray(w, dtype=F64)
    p = x @ w                                                 # reduction 0
    S, E = p.shape
    prob = np.empty((S, topk), dtype=F64)
    idx = np.empty((S, topk), dtype=np.int64)
    for i in range(S):
        m = np.max(p[i])                                      # reduction 1
        t = np.sum(np.exp(p[i] - m))                          # reduction 2
        sel = topk_desc(p[i], topk)                           # reduction 3
        idx[i] = sel
        prob[i] = np.exp(p[i, sel] - m) / t
    return prob, idx, p


def topk_merge(a, b, k):
    """TopK of the union of two (value, index) lists: the combine step of the
    mergeable TopK state (largest first, ties to the lower index)."""
    both = sorted(list(a) + list(b), key=lambda vi: (-vi[0], vi[1]))
    return both[:k]


def moe_routing_incremental_row(p, topk, seg):
    """Level-k incremental form for one token's scores p, fed in segments of
    `seg` experts: every segment yields the level-1 fused state (m, t, TopK),
    which is folded into the running state with
    m' = max(m, m_s);  t' = t exp(m-m') + t_s exp(m_s-m');  s' = TopK(s, s_s)."""
    p = np.asarray(p, dtype=F64)
    m, t, s = NEG_INF, 0.0, []
    for lo in range(0, p.shape[0], seg):
        chunk = p[lo:lo + seg]
        m_s = float(np.max(chunk))
        t_s = float(np.sum(np.exp(chunk - m_s)))
        s_s = [(float(chunk[j]), lo + int(j)) for j in topk_desc(chunk, min(topk, chunk.shape[0]))]
        m_new = max(m, m_s)
        t = t * _corr(m, m_new) + t_s * _corr(m_s, m_new)
        s = topk_merge(s, s_s, topk)
        m = m_new
    prob = np.asarray([np.exp(v - m) / t for v, _ in s], dtype=F64)
    idx = np.asarray([j for _, j in s], dtype=np.int64)
    return prob, idx


# --------------------------------------------------------------------------
# O8. FP8 per-token quantisation + GEMM  (Section 3.4, case study)
# --------------------------------------------------------------------------
E4M3_MAX = 448.0


def e4m3_round(x):
    """Round float32 values to the OCP E4M3 grid (4 exponent bits, bias 7, 3 mantissa bits,
    no infinities, largest finite value 448): nearest, ties to the even mantissa, finite
    values beyond 448 saturate.  Written from the format's definition: a value in
    [2^e, 2^(e+1)) with e >= -6 sits on a grid of step 2^(e-3); below 2^-6 the step is 2^-9."""
    x = np.asarray(x, dtype=np.float32).astype(F64)
    ax = np.abs(x)
    e = np.floor(np.log2(np.where(ax > 0, ax, 1.0)))
    e = np.maximum(e, -6.0)                    # subnormals share the exponent of 2^-6
    step = np.exp2(e - 3.0)
    q = np.rint(ax / step) * step              # rint: ties to even, exact here (powers of two)
    q = np.minimum(q, E4M3_MAX)
    return np.copysign(q, x)


def fp8_quant_gemm_twopass(a, w):
    """The multi-pass definition: m = max_l |a[l]|;  c = sum_l q(MAX a[l] / m) w[l], with q the
    rounding to FP8, one scale per token taken from the whole row.  a [M,K]; w [N,K] (FP8
    values, row n = output channel n).  Returns c * m / MAX, shape [M,N]."""
    a32 = np.asarray(a, dtype=np.float32)
    w = np.asarray(w, dtype=F64)
    m = np.max(np.abs(a32), axis=1)                                        # reduction 1
    with np.errstate(divide="ignore"):
        scale = np.where(m > 0, np.float32(E4M3_MAX) / m, np.float32(0.0)).astype(np.float32)
    q = e4m3_round(a32 * scale[:, None])
    c = q @ w.T                                                            # reduction 2
    return c * (m.astype(F64) / E4M3_MAX)[:, None]


def fp8_quant_gemm(a, w, tile):
    """Level-k incremental form over segments of `tile` elements of the contraction axis:
      m[L] = max(m[L-1], m_seg)
      c[L] = c[L-1] * m[L-1] / m[L] + sum_{l in seg} q(MAX a[l] / m[L]) w[l]
    Each segment is quantised with the running maximum that includes it; earlier
    segments keep the codes they were given and are only rescaled.  With one segment
    (tile >= K) this is the multi-pass definition."""
    a32 = np.asarray(a, dtype=np.float32)
    w = np.asarray(w, dtype=F64)
    M, K = a32.shape
    m = np.zeros(M, dtype=np.float32)
    c = np.zeros((M, w.shape[0]), dtype=F64)
    for lo in range(0, K, tile):
        seg = a32[:, lo:lo + tile]
        m_new = np.maximum(m, np.max(np.abs(seg), axis=1))
        with np.errstate(divide="ignore", invalid="ignore"):
            scale = np.where(m_new > 0, np.float32(E4M3_MAX) / m_new, np.float32(0.0)).astype(np.float32)
            corr = np.where(m_new > 0, m.astype(F64) / m_new.astype(F64), 1.0)
        q = e4m3_round(seg * scale[:, None])
        c = c * corr[:, None] + q @ w[:, lo:lo + tile].T
        m = m_new
    return c * (m.astype(F64) / E4M3_MAX)[:, None]

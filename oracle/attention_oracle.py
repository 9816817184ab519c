"""Plain fp64 oracle for parallel-pattern attention (test infrastructure only).

What it computes is the two-pass, fully materialised definition of the
operator that the paper's parallel pattern describes (Section 4.1, "Attention
Patterns and Templates": relevance scoring Q@K, a customizable function on the
scores, aggregation S@V):

    S  = Q K^T                                   relevance scoring
    S' = modification(S)                         elementwise, may carry a mask
    P  = row-wise normalization(S')              elementwise + row reduce
    O  = P V                                     aggregation

The instances follow Section 4.1, "Examples of Attention variants":
  * softmax attention: scale by 1/sqrt(d_k), P = exp(S' - rowmax) / rowsum;
  * RetNet parallel retention: S' = S x (decay mask),
    P = S' / clamp(sum_j |S'|, min=1)  (the reduceAbssum primitive);
  * ReLU attention: S' = max(S, 0), no normalization;
  * sigmoid attention is only named by the paper (Table 2); the formula
    P = sigmoid(S') with a constant bias folded into S' is the benchmark
    configuration's reading.
The full L_q x L_k score matrix is materialised in fp64.  There is no tiling,
no running maximum, no causal skipping and no reordering beyond the
definition.  numpy's matmul serves as the contraction step.

Readings taken where the paper is silent (all listed in the design notes):
  * the scale multiplies the scores (identical in exact arithmetic to
    scaling q, which is what the paper's q_mod does);
  * a masked entry contributes nothing: P = 0 and it is excluded from every
    row reduction, for every normalization;
  * a row with no visible key yields a zero output row;
  * causal alignment for L_q != L_k is bottom-right: key j is visible to
    query i iff j <= i + (L_k - L_q); a sliding window of W keeps, of those,
    the W keys nearest the diagonal: i + (L_k - L_q) - W < j;
  * grouped-query heads are contiguous groups: h_kv = h_q // (H_q // H_kv);
  * the decay mask entry is gamma[h_q] ** (i + (L_k - L_q) - j) on visible
    entries;
  * "abs_of_sum" (|sum_j S'|, clamp min 1) is the alternative reading of the
    retention normalizer and is provided beside the paper's "abssum".

Every function is pinned by tests/test_oracle_pins.py against closed forms,
invariants, a library routine for the softmax special case, a recurrent
formulation of retention and a pure-Python brute force.  No function here is
"parity unpinned".
"""
from __future__ import annotations

import math

import numpy as np

SCORE_MODS = ("none", "bias", "head_decay", "relu", "bias_tensor")
NORMS = ("softmax", "sigmoid", "abssum", "abs_of_sum", "none")
MASKS = ("none", "causal", "sliding_window")  # the last one is passed as ("sliding_window", W)


def _as_f64(x):
    # torch tensors (incl. bfloat16) and numpy arrays are both accepted;
    # widening bf16/fp32 to fp64 is exact.
    if hasattr(x, "detach"):
        x = x.detach().cpu().double().numpy()
    return np.asarray(x, dtype=np.float64)


def _visible(rows, L_q, L_k, mask):
    """Boolean [len(rows), L_k] visibility (Section 4.1: a modification
    annotated as a mask; causal = attend to prior tokens only)."""
    if mask == "none":
        return np.ones((len(rows), L_k), dtype=bool)
    off = L_k - L_q
    j = np.arange(L_k)[None, :]
    if mask == "causal":
        return j <= (rows[:, None] + off)
    # sliding window (Section 2, "Efficiency Innovations": the interaction is limited
    # to a local window): the W most recent keys up to and including the causal one
    if isinstance(mask, tuple) and len(mask) == 2 and mask[0] == "sliding_window" and int(mask[1]) >= 1:
        d = rows[:, None] + off - j
        return (d >= 0) & (d < int(mask[1]))
    raise ValueError(f"unknown mask {mask!r}")


def _modified_scores(q, k, *, scale, score_mod, bias, gamma_h, mask, rows, bias_t=None):
    """(S'[rows, :], visibility[rows, :]) for one head: relevance scoring and
    the elementwise modification, before any row-wise normalization."""
    q = _as_f64(q)
    k = _as_f64(k)
    L_q, L_k = q.shape[0], k.shape[0]
    rows = np.arange(L_q) if rows is None else np.asarray(rows, dtype=np.int64)
    vis = _visible(rows, L_q, L_k, mask)

    # relevance scoring
    s = q[rows] @ k.T
    # modification (elementwise)
    s = s * float(scale)
    if score_mod == "none":
        pass
    elif score_mod == "bias":
        s = s + float(bias)
    elif score_mod == "head_decay":
        if gamma_h is None:
            raise ValueError("head_decay needs gamma_h")
        dist = rows[:, None] + (L_k - L_q) - np.arange(L_k)[None, :]
        decay = np.power(float(gamma_h), np.where(vis, dist, 0).astype(np.float64))
        s = s * decay
    elif score_mod == "relu":
        s = np.maximum(s, 0.0)
    elif score_mod == "bias_tensor":
        # an additive bias per (query, key) pair (Section 4.1: a modification is any
        # elementwise function of the scores; relative-position and ALiBi biases are this)
        if bias_t is None:
            raise ValueError("bias_tensor needs bias_t [L_q, L_k]")
        s = s + _as_f64(bias_t)[rows]
    else:
        raise ValueError(f"unknown score_mod {score_mod!r}")
    return s, vis


def weights_head(q, k, *, scale, score_mod="none", bias=0.0, gamma_h=None,
                 norm="softmax", mask="none", rows=None, bias_t=None):
    """P[rows, :] for one head: q [L_q, D_qk], k [L_k, D_qk] -> [len(rows), L_k].

    `rows` selects query rows (default all); each row is independent, so a
    subset is the same definition evaluated on fewer rows.
    """
    s, vis = _modified_scores(q, k, scale=scale, score_mod=score_mod, bias=bias,
                              gamma_h=gamma_h, mask=mask, rows=rows, bias_t=bias_t)
    # row-wise normalization; masked entries take no part
    if norm == "softmax":
        sm = np.where(vis, s, -np.inf)
        m = sm.max(axis=1, keepdims=True)
        m = np.where(np.isfinite(m), m, 0.0)
        e = np.where(vis, np.exp(sm - m), 0.0)
        den = e.sum(axis=1, keepdims=True)
        p = np.divide(e, den, out=np.zeros_like(e), where=den > 0)
    elif norm == "sigmoid":
        p = np.where(vis, 1.0 / (1.0 + np.exp(-s)), 0.0)
    elif norm == "abssum":
        sv = np.where(vis, s, 0.0)
        den = np.maximum(np.abs(sv).sum(axis=1, keepdims=True), 1.0)
        p = sv / den
    elif norm == "abs_of_sum":
        sv = np.where(vis, s, 0.0)
        den = np.maximum(np.abs(sv.sum(axis=1, keepdims=True)), 1.0)
        p = sv / den
    elif norm == "none":
        p = np.where(vis, s, 0.0)
    else:
        raise ValueError(f"unknown norm {norm!r}")
    return p


def row_stats_head(q, k, *, scale, score_mod="none", bias=0.0, gamma_h=None,
                   norm="softmax", mask="none", rows=None, bias_t=None):
    """The final result of the row reduction that the normalization keeps per
    query row (Section 4.1, online row-norm interface: the final row scales),
    over the visible keys of each row:
      softmax     ln sum_j exp(S'_ij)   (-inf for a row with no visible key);
      abssum      sum_j |S'_ij|         (before the clamp at 1);
      abs_of_sum  sum_j S'_ij           (signed, before |.| and the clamp).
    The running maximum and running sum of the online form are not unique
    (they depend on the block order); their combination above is."""
    s, vis = _modified_scores(q, k, scale=scale, score_mod=score_mod, bias=bias,
                              gamma_h=gamma_h, mask=mask, rows=rows, bias_t=bias_t)
    if norm == "softmax":
        sm = np.where(vis, s, -np.inf)
        m = sm.max(axis=1)
        safe = np.where(np.isfinite(m), m, 0.0)
        tot = np.where(vis, np.exp(sm - safe[:, None]), 0.0).sum(axis=1)
        with np.errstate(divide="ignore"):
            return np.where(tot > 0, safe + np.log(tot), -np.inf)
    if norm == "abssum":
        return np.abs(np.where(vis, s, 0.0)).sum(axis=1)
    if norm == "abs_of_sum":
        return np.where(vis, s, 0.0).sum(axis=1)
    raise ValueError(f"normalization {norm!r} keeps no row statistic")


def attention_head(q, k, v, *, scale, score_mod="none", bias=0.0, gamma_h=None,
                   norm="softmax", mask="none", rows=None, bias_t=None):
    """O[rows, :] for one head: aggregation P @ V (Section 4.1)."""
    p = weights_head(q, k, scale=scale, score_mod=score_mod, bias=bias,
                     gamma_h=gamma_h, norm=norm, mask=mask, rows=rows, bias_t=bias_t)
    return p @ _as_f64(v)


def attention(Q, K, V, *, scale, score_mod="none", bias=0.0, gamma=None,
              norm="softmax", mask="none", bias_tensor=None):
    """Full operator.  Q [B,H_q,L_q,D_qk], K [B,H_kv,L_k,D_qk],
    V [B,H_kv,L_k,D_v] -> O [B,H_q,L_q,D_v] in fp64.  `gamma` is a length-H_q
    sequence of per-query-head decay rates (head_decay only); `bias_tensor`
    [B or 1, H_q or 1, L_q, L_k] the additive bias of score_mod "bias_tensor"."""
    Q, K, V = _as_f64(Q), _as_f64(K), _as_f64(V)
    B, H_q, L_q, _ = Q.shape
    H_kv = K.shape[1]
    if H_q % H_kv:
        raise ValueError("H_q must be a multiple of H_kv")
    g = H_q // H_kv
    O = np.zeros((B, H_q, L_q, V.shape[3]), dtype=np.float64)
    bt = None if bias_tensor is None else _as_f64(bias_tensor)
    for b in range(B):
        for h in range(H_q):
            O[b, h] = attention_head(
                Q[b, h], K[b, h // g], V[b, h // g], scale=scale,
                score_mod=score_mod, bias=bias,
                gamma_h=None if gamma is None else float(gamma[h]),
                norm=norm, mask=mask,
                bias_t=None if bt is None else bt[b if bt.shape[0] > 1 else 0, h if bt.shape[1] > 1 else 0])
    return O


def brute(Q, K, V, *, scale, score_mod="none", bias=0.0, gamma=None,
          norm="softmax", mask="none", bias_tensor=None):
    """The same definition as scalar Python loops (tiny shapes only).  Used to
    check the vectorised functions above; written separately, element by
    element, so an indexing or broadcasting slip in one does not repeat in the
    other."""
    Q, K, V = _as_f64(Q), _as_f64(K), _as_f64(V)
    B, H_q, L_q, D_qk = Q.shape
    _, H_kv, L_k, D_v = V.shape
    g = H_q // H_kv
    off = L_k - L_q
    O = np.zeros((B, H_q, L_q, D_v))
    for b in range(B):
        for h in range(H_q):
            hk = h // g
            for i in range(L_q):
                w = []
                for j in range(L_k):
                    if mask == "causal" and j > i + off:
                        w.append(None)
                        continue
                    if isinstance(mask, tuple) and not (i + off - mask[1] < j <= i + off):
                        w.append(None)
                        continue
                    s = 0.0
                    for d in range(D_qk):
                        s += Q[b, h, i, d] * K[b, hk, j, d]
                    s *= scale
                    if score_mod == "bias":
                        s += bias
                    elif score_mod == "head_decay":
                        s *= float(gamma[h]) ** (i + off - j)
                    elif score_mod == "relu":
                        s = max(s, 0.0)
                    elif score_mod == "bias_tensor":
                        bt = bias_tensor
                        s += float(bt[b if bt.shape[0] > 1 else 0][h if bt.shape[1] > 1 else 0][i][j])
                    w.append(s)
                live = [x for x in w if x is not None]
                if not live:
                    continue
                if norm == "softmax":
                    mx = max(live)
                    den = sum(math.exp(x - mx) for x in live)
                    p = [0.0 if x is None else math.exp(x - mx) / den for x in w]
                elif norm == "sigmoid":
                    p = [0.0 if x is None else 1.0 / (1.0 + math.exp(-x)) for x in w]
                elif norm == "abssum":
                    den = max(sum(abs(x) for x in live), 1.0)
                    p = [0.0 if x is None else x / den for x in w]
                elif norm == "abs_of_sum":
                    den = max(abs(sum(live)), 1.0)
                    p = [0.0 if x is None else x / den for x in w]
                elif norm == "none":
                    p = [0.0 if x is None else x for x in w]
                else:
                    raise ValueError(norm)
                for d in range(D_v):
                    acc = 0.0
                    for j in range(L_k):
                        acc += p[j] * V[b, hk, j, d]
                    O[b, h, i, d] = acc
    return O

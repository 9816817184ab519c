"""Plain fp64 oracle for the backward pass of parallel-pattern attention
(test infrastructure only).

The paper gives no formulas of its own for the backward pass: its backward
graph is the automatic differentiation of the forward one (Section 4.1,
online row-norm interface: forward and backward graphs built from the same
definition; Section 5.1: a gradient node per tensor).  What is computed here is
therefore the derivative of the forward definition

    S = Q K^T,  S' = modification(scale * S),  P = normalization(S'),  O = P V

with respect to Q, K and V, for a given upstream gradient dO (the gradient of
sum(O * dO)), by the chain rule on the fully materialised L_q x L_k matrices:

    dV  = P^T dO                       dP = dO V^T
    dS' = P * (dP - rowsum(P * dP))    softmax
        = dP * P * (1 - P)             sigmoid
        = dP on visible entries        no normalization
        = dP / n - g * rowsum(dP * S') / n^2     abs-sum family: P = S' / n, n = max(r, 1),
          r = rowsum |S'| with g = sign(S'), or r = |rowsum S'| with g = sign(rowsum S');
          the second term only where r > 1 (below the clamp n is the constant 1)
    dS  = dS' * d modification / dS    (1 for scale/bias, the decay factor,
                                        the step function for ReLU), times scale
    dQ  = dS K                         dK = dS^T Q

Masked entries take no part (their P is a constant 0), a row with no visible
key has zero gradient, and with grouped-query heads dK and dV of a k/v head are
the sums over the query heads that share it.  No tiling, no recomputation from
row statistics, no reordering.  The abs-sum normalizers are differentiated
piecewise (quotient rule above the clamp, identity below it; at the kinks r = 1
and S' = 0, a set of measure zero, the one-sided value of the branch taken).

Pinned by tests/test_oracle_backward_pins.py: central finite differences of
the (separately pinned) forward oracle, a library autograd for the softmax
special case, closed forms and invariants.  No function here is "parity
unpinned".
"""
from __future__ import annotations

import numpy as np

from .attention_oracle import _as_f64, _visible


def attention_backward_head(q, k, v, do, *, scale, score_mod="none", bias=0.0, gamma_h=None,
                            norm="softmax", mask="none", bias_t=None, with_dbias=False):
    """(dq, dk, dv) for one head: q [L_q, D_qk], k [L_k, D_qk], v [L_k, D_v],
    do [L_q, D_v].  with_dbias: also the gradient with respect to the additive
    bias tensor, [L_q, L_k] (it is dS': the bias enters S' with slope 1)."""
    q, k, v, do = _as_f64(q), _as_f64(k), _as_f64(v), _as_f64(do)
    L_q, L_k = q.shape[0], k.shape[0]
    rows = np.arange(L_q)
    vis = _visible(rows, L_q, L_k, mask)

    # forward, as the definition states it
    s0 = (q @ k.T) * float(scale)
    if score_mod == "none":
        s, dmod = s0, np.ones_like(s0)
    elif score_mod == "bias":
        s, dmod = s0 + float(bias), np.ones_like(s0)
    elif score_mod == "head_decay":
        dist = rows[:, None] + (L_k - L_q) - np.arange(L_k)[None, :]
        dmod = np.power(float(gamma_h), np.where(vis, dist, 0).astype(np.float64))
        s = s0 * dmod
    elif score_mod == "relu":
        s, dmod = np.maximum(s0, 0.0), (s0 > 0).astype(np.float64)
    elif score_mod == "bias_tensor":   # an additive constant per (query, key) pair: slope 1
        s, dmod = s0 + _as_f64(bias_t), np.ones_like(s0)
    else:
        raise ValueError(f"unknown score_mod {score_mod!r}")

    if norm == "softmax":
        sm = np.where(vis, s, -np.inf)
        m = sm.max(axis=1, keepdims=True)
        m = np.where(np.isfinite(m), m, 0.0)
        e = np.where(vis, np.exp(sm - m), 0.0)
        den = e.sum(axis=1, keepdims=True)
        p = np.divide(e, den, out=np.zeros_like(e), where=den > 0)
    elif norm == "sigmoid":
        p = np.where(vis, 1.0 / (1.0 + np.exp(-s)), 0.0)
    elif norm == "none":
        p = np.where(vis, s, 0.0)
    elif norm in ("abssum", "abs_of_sum"):
        sv = np.where(vis, s, 0.0)
        tot = sv.sum(axis=1, keepdims=True)
        r = np.abs(sv).sum(axis=1, keepdims=True) if norm == "abssum" else np.abs(tot)
        den = np.maximum(r, 1.0)
        p = sv / den
    else:
        raise ValueError(f"unknown norm {norm!r}")

    # aggregation O = P V
    dv = p.T @ do
    dp = do @ v.T
    # normalization
    if norm == "softmax":
        ds = p * (dp - (p * dp).sum(axis=1, keepdims=True))
    elif norm == "sigmoid":
        ds = dp * p * (1.0 - p)
    elif norm in ("abssum", "abs_of_sum"):
        # quotient rule for S' / n; d n / d S'_ij = g_ij where r > 1, 0 below the clamp
        grad_r = np.sign(sv) if norm == "abssum" else np.sign(tot) * np.ones_like(sv)
        ds = dp / den - np.where(r > 1.0, grad_r * (dp * sv).sum(axis=1, keepdims=True) / den ** 2, 0.0)
    else:
        ds = np.where(vis, dp, 0.0)
    # modification and scale
    dsp = np.where(vis, ds, 0.0)          # gradient of the modified scores S'
    ds = dsp * dmod * float(scale)
    # relevance scoring S = Q K^T
    if with_dbias:
        return ds @ k, ds.T @ q, dv, dsp
    return ds @ k, ds.T @ q, dv


def attention_backward(Q, K, V, dO, *, scale, score_mod="none", bias=0.0, gamma=None,
                       norm="softmax", mask="none", bias_tensor=None, with_dbias=False):
    """Full operator: Q [B,H_q,L_q,D_qk], K [B,H_kv,L_k,D_qk], V [B,H_kv,L_k,D_v],
    dO [B,H_q,L_q,D_v] -> (dQ, dK, dV) in fp64, shaped like Q, K, V."""
    Q, K, V, dO = _as_f64(Q), _as_f64(K), _as_f64(V), _as_f64(dO)
    B, H_q = Q.shape[:2]
    H_kv = K.shape[1]
    if H_q % H_kv:
        raise ValueError("H_q must be a multiple of H_kv")
    g = H_q // H_kv
    dQ, dK, dV = np.zeros_like(Q), np.zeros_like(K), np.zeros_like(V)
    dB = np.zeros((B, H_q, Q.shape[2], K.shape[2])) if with_dbias else None   # per batch and head, not summed
    bt = None if bias_tensor is None else _as_f64(bias_tensor)   # [B or 1, H_q or 1, L_q, L_k]
    for b in range(B):
        for h in range(H_q):
            res = attention_backward_head(
                Q[b, h], K[b, h // g], V[b, h // g], dO[b, h], scale=scale, score_mod=score_mod, bias=bias,
                gamma_h=None if gamma is None else float(gamma[h]), norm=norm, mask=mask,
                bias_t=None if bt is None else bt[b if bt.shape[0] > 1 else 0, h if bt.shape[1] > 1 else 0],
                with_dbias=with_dbias)
            dq, dk, dv = res[:3]
            if with_dbias:
                dB[b, h] = res[3]
            dQ[b, h] = dq
            dK[b, h // g] += dk
            dV[b, h // g] += dv
    if with_dbias:
        return dQ, dK, dV, dB
    return dQ, dK, dV

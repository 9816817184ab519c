"""Plain fp64 oracle for recurrent-pattern retention (test infrastructure only).

The paper's recurrent pattern (Section 4.1, "Attention Patterns and Templates")
forms the product of keys and values first and lets every query read a
compressed state: K@V, then Q@h, iterated along the sequence.  With the
identity as state modification except for a constant per-head decay (the
retention of RetNet, Table 2 "Retention Recurrent"; Section 4.1's h_mod:
h x decay) the recurrence is, for one batch entry and head,

    h_0 = 0                                  state, [d_qk x d_v]
    h_t = gamma * h_{t-1} + k_t^T v_t        state update (K@V, h_mod = decay)
    o_t = scale * q_t h_t                    read-out    (Q@h)

This file walks that recurrence token by token in fp64: no chunking, no
reordering.  The chunk-parallel form that the paper names as the kernel
template's way to reach the matrix units is an implementation matter of the
HIP path and is not used here.

Readings taken where the paper is silent: the state starts at zero; token t
reads the state that already includes token t (the recurrent form of the
causal parallel retention, whose diagonal weight is gamma^0 = 1); no
normalization follows the read-out (the paper's Table 2 row gives none for the
recurrent form); gamma is one constant per head.

Pinned by tests/test_oracle_recurrent_pins.py: equality with the parallel
retention oracle (decay mask gamma^(i-j) on the causal scores, no
normalization), the closed form for gamma = 1 (prefix sums), a hand-computed
two-token case, and a brute-force triple loop.

Only tests/, the smoke check and the benchmark's cpu_baseline leg may import
this module.  It shares no code with the HIP path.
"""
import numpy as np


def retention_recurrent_head(q, k, v, *, scale, gamma_h, return_state=False, h0=None):
    """q [L, d_qk], k [L, d_qk], v [L, d_v] (any float dtype) -> o [L, d_v] fp64
    (and the final state [d_qk, d_v] when asked).  h0: the state in front of the first token (default: zero)."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    L, d_qk = q.shape
    d_v = v.shape[1]
    h = np.zeros((d_qk, d_v), dtype=np.float64) if h0 is None else np.array(h0, dtype=np.float64)
    o = np.zeros((L, d_v), dtype=np.float64)
    for t in range(L):
        h = float(gamma_h) * h + np.outer(k[t], v[t])
        o[t] = float(scale) * (q[t] @ h)
    return (o, h) if return_state else o


def retention_recurrent(Q, K, V, *, scale, gamma):
    """Q, K [B, H, L, d_qk], V [B, H, L, d_v] -> O [B, H, L, d_v] fp64; gamma: one decay per head."""
    Q = np.asarray(Q, dtype=np.float64)
    B, H, L, _ = Q.shape
    O = np.zeros((B, H, L, np.asarray(V).shape[-1]), dtype=np.float64)
    for b in range(B):
        for h in range(H):
            O[b, h] = retention_recurrent_head(Q[b, h], K[b, h], V[b, h], scale=scale, gamma_h=gamma[h])
    return O

"""Plain fp64 oracle for the recurrent pattern with per-token gates (test infrastructure only).

The paper's recurrent pattern (Section 4.1, "Attention Patterns and Templates": K@V first, then Q@h, iterated
over a compressed state h) with the state and key modifications of its Mamba2 example (Section 4.1, "Examples of
Attention variants": k_mod = k x gate, h_mod = h x decay x gate) and of gated retention (Table 2, "Gated
Retention"; "Mamba2 SSM"): for one batch entry and value head,

    h_0 = given (default 0)                             state, [d_qk x d_v]
    h_t = a_t * h_{t-1} + (g_t * k_t)^T v_t             h_mod: the state times a per-token factor a_t in (0, 1];
                                                        k_mod: the key times a per-token gate g_t
    o_t = scale * q_t h_t                               read-out (Q@h)

walked token by token in fp64: no chunking, no reordering.  The instances:
  * retention with a constant decay: a_t = gamma, g_t = 1 (retention_recurrent_oracle.py);
  * gated retention: a_t data dependent (a sigmoid of the token raised to a power), g_t = 1;
  * Mamba2's state space module: q = C, k = B, v = x, a_t = exp(dt_t * A_head), g_t = dt_t; B and C are shared by
    the value heads of a group (heads // groups of them per q/k head).

Readings taken where the paper is silent or loose (listed in the design notes): the paper writes the state
modification as "h x decay x gate"; it is read as ONE per-token factor a_t = exp(log_decay_t) that the caller
supplies (for Mamba2 the product dt_t * A in the exponent), given as its natural logarithm so that products over
tokens are sums; token t reads the state that already includes token t; no normalization follows the read-out.

Pinned by tests/test_oracle_gated_pins.py.  Only tests/, the smoke check and the benchmark's cpu_baseline leg may
import this module.  It shares no code with the HIP path.
"""
import numpy as np


def gated_recurrent_head(q, k, v, log_decay, key_gate=None, *, scale, h0=None, return_state=False):
    """q, k [L, d_qk], v [L, d_v], log_decay [L] (ln a_t <= 0), key_gate [L] or None (ones) -> o [L, d_v] fp64
    (and the final state [d_qk, d_v] when asked).  h0: the state in front of the first token (default zero)."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    la = np.asarray(log_decay, dtype=np.float64)
    L, d_qk = q.shape
    g = np.ones(L) if key_gate is None else np.asarray(key_gate, dtype=np.float64)
    h = np.zeros((d_qk, v.shape[1])) if h0 is None else np.array(h0, dtype=np.float64)
    o = np.zeros((L, v.shape[1]))
    for t in range(L):
        h = np.exp(la[t]) * h + np.outer(g[t] * k[t], v[t])
        o[t] = float(scale) * (q[t] @ h)
    return (o, h) if return_state else o


def gated_recurrent(Q, K, V, log_decay, key_gate=None, *, scale, h0=None, return_state=False):
    """Q, K [B, H_qk, L, d_qk], V [B, H, L, d_v], log_decay / key_gate [B, H, L] -> O [B, H, L, d_v] fp64.
    Value head h reads q/k head h // (H // H_qk) (contiguous groups; H_qk = H: one q/k head per value head)."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    B, H, L, d_v = V.shape
    grp = H // Q.shape[1]
    O = np.zeros((B, H, L, d_v))
    S = np.zeros((B, H, Q.shape[3], d_v))
    for b in range(B):
        for h in range(H):
            O[b, h], S[b, h] = gated_recurrent_head(
                Q[b, h // grp], K[b, h // grp], V[b, h], np.asarray(log_decay)[b, h],
                None if key_gate is None else np.asarray(key_gate)[b, h], scale=scale,
                h0=None if h0 is None else np.asarray(h0)[b, h], return_state=True)
    return (O, S) if return_state else O

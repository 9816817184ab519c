"""Plain fp64 oracle for the backward pass of the recurrent pattern with per-token gates (test infrastructure only).

The paper evaluates the recurrent pattern forward and backward (Section 6.1; Table 2: "Mamba2 SSM", "Gated
Retention", "Retention Recurrent") and obtains its backward graphs by automatic differentiation of the forward
computation (Section 5.1: a gradient node per tensor); it prints no formulas for them.  This oracle is therefore the
chain rule applied to the forward definition of gated_recurrent_oracle.py,

    h_t = a_t * h_{t-1} + (g_t * k_t)^T v_t,    o_t = scale * q_t h_t,    a_t = exp(log_decay_t),

token by token in fp64, walking the tokens backwards with D_t, the gradient of the loss with respect to the state
h_t (everything that reads h_t: the read-out of token t, and h_{t+1} through the factor a_{t+1}):

    D_t        = scale * q_t^T dO_t  +  a_{t+1} * D_{t+1}          (tokens 1..L; for t = L the second term is dh_out,
                                                                     the gradient handed in for the final state, default 0)
    dq_t       = scale * h_t dO_t^T
    dk_t       = g_t * D_t v_t^T          dg_t = k_t . (D_t v_t^T)          dv_t = g_t * k_t D_t
    dlog_decay_t = a_t * <D_t, h_{t-1}>                           (sum over all entries of the state)
    dh0        = a_1 * D_1                                          (the gradient that reaches the initial state)

The states h_t the backward walk needs are recomputed from checkpoints kept every `ckpt` tokens by the same forward
step, so memory stays small at long sequences; that changes no arithmetic.  With grouped heads (Mamba2's B and C
shared by the value heads of a group) the gradients of a shared q/k head are the sums over its value heads.

Pinned by tests/test_oracle_gated_backward_pins.py (central finite differences of the pinned forward oracle, library
automatic differentiation of an independently written loop, closed forms, homogeneity identities, the attention
backward oracle on constant-decay retention, planted mistakes).  Only tests/, the smoke check and the benchmark's
cpu_baseline leg may import this module.  It shares no code with the HIP path.
"""
import numpy as np


def gated_recurrent_backward_head(q, k, v, log_decay, key_gate, dO, *, scale, h0=None, dh_out=None, ckpt=64):
    """q, k [L, d_qk], v, dO [L, d_v], log_decay [L], key_gate [L] or None (ones; its gradient is still returned).
    Returns a dict of fp64 arrays: dq, dk [L, d_qk], dv [L, d_v], dlog_decay, dkey_gate [L], dh0 [d_qk, d_v]."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    dO = np.asarray(dO, dtype=np.float64)
    la = np.asarray(log_decay, dtype=np.float64)
    L, d_qk = q.shape
    d_v = v.shape[1]
    g = np.ones(L) if key_gate is None else np.asarray(key_gate, dtype=np.float64)
    a = np.exp(la)
    s = float(scale)
    h_first = np.zeros((d_qk, d_v)) if h0 is None else np.array(h0, dtype=np.float64)

    def step(h, t):  # the forward definition, one token
        return a[t] * h + np.outer(g[t] * k[t], v[t])

    # forward walk: the state in front of every block of ckpt tokens
    front = []
    h = h_first
    for t in range(L):
        if t % ckpt == 0:
            front.append(h)
        h = step(h, t)

    dq, dk, dv = np.zeros((L, d_qk)), np.zeros((L, d_qk)), np.zeros((L, d_v))
    dla, dg = np.zeros(L), np.zeros(L)
    D = np.zeros((d_qk, d_v)) if dh_out is None else np.array(dh_out, dtype=np.float64)  # a_{t+1} D_{t+1}, carried
    for c in range(len(front) - 1, -1, -1):
        t0, t1 = c * ckpt, min(L, (c + 1) * ckpt)
        hs = [front[c]]                       # hs[i] = h_{t0 + i - 1}: the state in front of token t0 + i
        for t in range(t0, t1):
            hs.append(step(hs[-1], t))
        for t in range(t1 - 1, t0 - 1, -1):
            h_prev, h_t = hs[t - t0], hs[t - t0 + 1]
            D = D + s * np.outer(q[t], dO[t])           # now D_t
            dq[t] = s * (h_t @ dO[t])
            Dv = D @ v[t]                               # D_t v_t^T, [d_qk]
            dk[t] = g[t] * Dv
            dg[t] = k[t] @ Dv
            dv[t] = g[t] * (k[t] @ D)
            dla[t] = a[t] * np.sum(D * h_prev)
            D = a[t] * D                                # what reaches h_{t-1}
    return dict(dq=dq, dk=dk, dv=dv, dlog_decay=dla, dkey_gate=dg, dh0=D)


def gated_recurrent_backward(Q, K, V, log_decay, key_gate, dO, *, scale, h0=None, dh_out=None):
    """Q, K [B, H_qk, L, d_qk], V, dO [B, H, L, d_v], log_decay / key_gate [B, H, L] -> dict of fp64 arrays:
    dQ, dK [B, H_qk, L, d_qk] (summed over the value heads of each q/k head), dV [B, H, L, d_v], dlog_decay,
    dkey_gate [B, H, L], dh0 [B, H, d_qk, d_v]."""
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    B, H, L, d_v = V.shape
    H_qk, d_qk = Q.shape[1], Q.shape[3]
    grp = H // H_qk
    out = dict(dQ=np.zeros((B, H_qk, L, d_qk)), dK=np.zeros((B, H_qk, L, d_qk)), dV=np.zeros((B, H, L, d_v)),
               dlog_decay=np.zeros((B, H, L)), dkey_gate=np.zeros((B, H, L)), dh0=np.zeros((B, H, d_qk, d_v)))
    for b in range(B):
        for h in range(H):
            r = gated_recurrent_backward_head(
                Q[b, h // grp], K[b, h // grp], V[b, h], np.asarray(log_decay)[b, h],
                None if key_gate is None else np.asarray(key_gate)[b, h], np.asarray(dO)[b, h], scale=scale,
                h0=None if h0 is None else np.asarray(h0)[b, h], dh_out=None if dh_out is None else np.asarray(dh_out)[b, h])
            out["dQ"][b, h // grp] += r["dq"]
            out["dK"][b, h // grp] += r["dk"]
            out["dV"][b, h] = r["dv"]
            out["dlog_decay"][b, h] = r["dlog_decay"]
            out["dkey_gate"][b, h] = r["dkey_gate"]
            out["dh0"][b, h] = r["dh0"]
    return out

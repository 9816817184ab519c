"""GPU parity of the backward pass of the recurrent pattern with per-token gates (ae_gated_backward, through the C
ABI) against the fp64 token-by-token backward oracle on the same seeded inputs.

Bars.  dQ, dK, dV: as for the forward pass -- max-abs <= 1e-2 and mean-abs <= 1e-3 relative to max(1, the largest
|reference| of the row); each is one run of the forward kernel on other operands (bf16 operands, bf16 weights and
state into the MFMAs, fp32 accumulation).

dlog_decay and dkey_gate are one number per token, and a bar of their own is derived from the arithmetic.  With
G_ij = P_ij dP_ij (forward weight times its gradient), q_i . dq_i is the sum of row i of G, k_j . dk_j the sum of
column j, dkey_gate_j = k_j . dk_j / g_j, and dlog_decay_t = sum_{i >= t} (q_i . dq_i - k_i . dk_i).  Row sums and
column sums come out of different runs of the kernel, each of which rounds its weights (and the carried state, and
the weighted values that update it) to bf16: every term G_ij carries an independent relative error of up to 2^-9
per rounding, about 2^-9 in standard deviation for the three together.  A sum of such terms is off by 2^-9 times the
root of the sum of their squares, and for terms of random sign that root is about the size of the sum itself -- or,
where a sum happens to cancel, about the size such sums have elsewhere in the head.  With [x]_i = max(|x_i|, rms of
x over the head) standing in for that root,
    dkey_gate_j   is held to  6 x 2^-9 x [dkey_gate]_j,
    dlog_decay_t  is held to  6 x 2^-9 x sqrt(sum_{i >= t} ([q . dq]_i^2 + [k . dk]_i^2))   (+ 1e-3 absolute),
six standard deviations of that model (the stand-in for the root of the sum of squares is itself only right to a
factor of about 1.5), with the dot products taken from the oracle.  The errors of unrelated pairs (i, j >= t) do
not cancel in the suffix sum as their exact values do, which is why the bar grows with the root of the number of
later tokens; an implementation that forms both sums from one set of rounded weights would not need that.
"""
import math

import numpy as np
import pytest
import torch

from oracle.gated_recurrent_backward_oracle import gated_recurrent_backward as oracle_backward
from oracle.gated_recurrent_backward_oracle import gated_recurrent_backward_head
from paper_2502_15349_amd.workloads import Workload, make_gates, make_grad, make_inputs

pytestmark = pytest.mark.gpu
MAX_ABS, MEAN_ABS = 1e-2, 1e-3


@pytest.fixture(scope="module")
def A():
    from paper_2502_15349_amd import ae_attn
    return ae_attn


def check_rows(got, ref, what):
    assert np.isfinite(got).all(), what
    rs = np.maximum(np.abs(ref).max(axis=-1, keepdims=True), 1.0)
    err = np.abs(got - ref) / rs
    print(f"{what}: max_abs {err.max():.3e} mean_abs {err.mean():.3e} |ref|max {np.abs(ref).max():.3e}", flush=True)
    assert err.max() <= MAX_ABS and err.mean() <= MEAN_ABS, (what, err.max(), err.mean())


def inputs(cid, B, H, H_qk, L, dqk, dv, kind):
    Q, K, _ = make_inputs(Workload("gq", cid, B, H_qk, H_qk, L, L, dqk, dqk))
    wv = Workload("gv", cid, B, H, H, L, L, dv, dv)
    _, _, V = make_inputs(wv)
    dO = make_grad(wv)
    la, kg = make_gates(B, H, L, 1000 * cid + 5, kind)
    return Q, K, V, la, kg, dO


def run(A, Q, K, V, la, kg, dO, scale):
    dev = torch.device("cuda:0")
    r = A.gated_recurrent_backward(Q.to(dev), K.to(dev), V.to(dev), la.to(dev), None if kg is None else kg.to(dev), dO.to(dev),
                                   scale=scale)
    torch.cuda.synchronize()
    return [None if t is None else t.cpu().double().numpy() for t in r]


U = 2.0 ** -9


def check_tokens(got, bound, ref, what):
    """Per-token quantities [.., L] against the derived bound (same shape)."""
    assert np.isfinite(got).all(), what
    ratio = np.abs(got - ref) / bound
    print(f"{what}: worst error / bound {ratio.max():.3f}, mean {ratio.mean():.3f} |ref|max {np.abs(ref).max():.3e}", flush=True)
    assert ratio.max() <= 1.0, (what, ratio.max())


def token_bounds(qdq, kdk, dkg):
    """qdq, kdk: the oracle's q_i . dq_i and k_i . dk_i per value head [.., L]; dkg: its dkey_gate.  Returns the bars of
    dlog_decay and dkey_gate described at the top."""
    def floored(x):
        return np.maximum(np.abs(x), np.sqrt(np.mean(x ** 2, axis=-1, keepdims=True)))
    tail = np.sqrt(np.cumsum((floored(qdq) ** 2 + floored(kdk) ** 2)[..., ::-1], axis=-1)[..., ::-1])
    return 6 * U * tail + 1e-3, 6 * U * floored(dkg) + 1e-6


def head_dots(Q, K, V, la, kg, dO, scale):
    """q . dq and k . dk per VALUE head from the oracle (the grouped sums dQ, dK do not give them)."""
    B, H, L = la.shape
    grp = H // Q.shape[1]
    qdq, kdk = np.zeros((B, H, L)), np.zeros((B, H, L))
    for b in range(B):
        for h in range(H):
            r = gated_recurrent_backward_head(Q[b, h // grp], K[b, h // grp], V[b, h], la[b, h], None if kg is None else kg[b, h],
                                              dO[b, h], scale=scale)
            qdq[b, h] = np.sum(Q[b, h // grp] * r["dq"], axis=-1)
            kdk[b, h] = np.sum(K[b, h // grp] * r["dk"], axis=-1)
    return qdq, kdk


def compare(got, ref, what, with_gate, dots):
    dQ, dK, dV, dla, dkg = got
    check_rows(dQ, ref["dQ"], what + " dQ")
    check_rows(dK, ref["dK"], what + " dK")
    check_rows(dV, ref["dV"], what + " dV")
    b_dla, b_dkg = token_bounds(dots[0], dots[1], ref["dkey_gate"])
    check_tokens(dla, b_dla, ref["dlog_decay"], what + " dlog_decay")
    if with_gate:
        check_tokens(dkg, b_dkg, ref["dkey_gate"], what + " dkey_gate")
    else:
        assert dkg is None


def oracle_all(Q, K, V, la, kg, dO, scale):
    n = [Q.float().numpy().astype(np.float64), K.float().numpy().astype(np.float64), V.float().numpy().astype(np.float64),
         la.numpy().astype(np.float64), None if kg is None else kg.numpy().astype(np.float64), dO.float().numpy().astype(np.float64)]
    return oracle_backward(*n, scale=scale), head_dots(*n, scale)


@pytest.mark.parametrize("dqk,dv", [(64, 64), (128, 64), (64, 128), (128, 128)])
@pytest.mark.parametrize("kind", ["gated_retention", "mamba2"])
@pytest.mark.parametrize("L", [1, 63, 64, 65, 200, 513])
def test_matches_oracle(A, dqk, dv, kind, L):
    Q, K, V, la, kg, dO = inputs(900 + L % 7, 2, 3, 3, L, dqk, dv, kind)
    scale = 1.0 / math.sqrt(dqk)
    print(f"case {kind} {dqk}/{dv} L {L}", flush=True)
    got = run(A, Q, K, V, la, kg, dO, scale)
    ref, dots = oracle_all(Q, K, V, la, kg, dO, scale)
    compare(got, ref, f"{kind} {dqk}/{dv} L={L}", kg is not None, dots)


@pytest.mark.parametrize("dqk,dv", [(128, 64), (64, 64)])
def test_grouped_query_key_heads(A, dqk, dv):
    # Mamba2's structure at a reduced head count: B and C shared by the value heads of a group; dQ and dK are sums
    # over the group
    Q, K, V, la, kg, dO = inputs(910, 1, 8, 2, 300, dqk, dv, "mamba2")
    got = run(A, Q, K, V, la, kg, dO, 1.0)
    ref, dots = oracle_all(Q, K, V, la, kg, dO, 1.0)
    compare(got, ref, f"mamba2 groups {dqk}/{dv}", True, dots)


def test_strong_decay_and_no_decay(A):
    # per-token decays of e^-8, none at all (gradients are plain suffix sums), and a slow decay broken by single
    # tokens of e^-30
    w = Workload("dec", 913, 1, 3, 3, 260, 260, 64, 64)
    Q, K, V = make_inputs(w)
    dO = make_grad(w)
    la = torch.full((1, 3, 260), -8.0)
    la[:, 1] = 0.0
    la[:, 2] = -0.01
    la[:, 2, 5::37] = -30.0
    got = run(A, Q, K, V, la, None, dO, 0.125)
    ref, dots = oracle_all(Q, K, V, la, None, dO, 0.125)
    compare(got, ref, "decay e^-8 / none / resets", False, dots)


def test_sampled_heads_at_benchmark_size(A):
    # 8 x 32 heads x 8192 tokens, 128/128, gated retention: three heads against the oracle
    B, H, L = 8, 32, 8192
    Q, K, V, la, kg, dO = inputs(914, B, H, H, L, 128, 128, "gated_retention")
    scale = 1.0 / math.sqrt(128)
    dQ, dK, dV, dla, _ = run(A, Q, K, V, la, kg, dO, scale)
    for b, h in ((0, 0), (3, 17), (7, 31)):
        ref = gated_recurrent_backward_head(Q[b, h].float().numpy(), K[b, h].float().numpy(), V[b, h].float().numpy(), la[b, h].numpy(),
                                            None, dO[b, h].float().numpy(), scale=scale)
        check_rows(dQ[b, h], ref["dq"], f"benchmark size ({b},{h}) dQ")
        check_rows(dK[b, h], ref["dk"], f"benchmark size ({b},{h}) dK")
        check_rows(dV[b, h], ref["dv"], f"benchmark size ({b},{h}) dV")
        qn, kn = Q[b, h].float().numpy().astype(np.float64), K[b, h].float().numpy().astype(np.float64)
        b_dla, _ = token_bounds(np.sum(qn * ref["dq"], axis=-1), np.sum(kn * ref["dk"], axis=-1), ref["dkey_gate"])
        check_tokens(dla[b, h], b_dla, ref["dlog_decay"], f"benchmark size ({b},{h}) dlog_decay")

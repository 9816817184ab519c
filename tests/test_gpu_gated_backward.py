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
root of the sum of their squares.  The tests form G from the inputs (its entries are what the model needs, not an
expected value) and hold
    dkey_gate_j   to  3 x 2^-9 x sum_i |G_ij| / g_j                                         (+ 1e-4 absolute),
    dlog_decay_t  to  8 x 2^-9 x sqrt(sum_{i >= t} (sum_j G_ij^2 + sum_j G_ji^2))           (+ 1e-3 absolute).
The first is the worst case of the three roundings (a column of G has few terms of weight, and the rounded state and
the rounded weighted values are shared by many of them, so their errors add up coherently rather than at random).
The second is eight standard deviations of the model: a long sum over many tokens, near enough to Gaussian, with
the same shared roundings fattening its tails (measured: the mean error is 0.8 standard deviations, as the model
says; the worst of some 10^5 tokens 7.1).  At the benchmark size, where G does not fit, the root of a sum of squares is
replaced by max(|sum|, rms of such sums over the head): for terms of random sign the two are of one size.  The errors
of unrelated pairs (i, j >= t) do not cancel in the suffix sum as their exact values do, which is why the bar grows
with the root of the number of later tokens; an implementation that forms both sums from one set of rounded weights
would not need that.
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


def token_bounds_proxy(qdq, kdk):
    """The bar of dlog_decay where G is too large to form: qdq, kdk are the oracle's q_i . dq_i and k_i . dk_i [L]."""
    def floored(x):
        return np.maximum(np.abs(x), np.sqrt(np.mean(x ** 2, axis=-1, keepdims=True)))
    return 8 * U * np.sqrt(np.cumsum((floored(qdq) ** 2 + floored(kdk) ** 2)[..., ::-1], axis=-1)[..., ::-1]) + 1e-3


def head_bounds(q, k, v, la, g, dO, scale):
    """One value head: G_ij = P_ij dP_ij from the inputs, and from it the bars of dlog_decay and dkey_gate [L]."""
    L = q.shape[0]
    B = np.cumsum(la)
    expo = B[:, None] - B[None, :]
    A = np.where(np.tril(np.ones((L, L), dtype=bool)), np.exp(np.minimum(expo, 0.0)), 0.0)
    gg = np.ones(L) if g is None else g
    G = scale * A * (q @ k.T) * gg[None, :] * (dO @ v.T)
    row2, col2 = np.sum(G * G, axis=1), np.sum(G * G, axis=0)
    b_dla = 8 * U * np.sqrt(np.cumsum((row2 + col2)[::-1])[::-1]) + 1e-3
    b_dkg = 3 * U * np.sum(np.abs(G), axis=0) / np.abs(gg) + 1e-4
    return b_dla, b_dkg


def all_bounds(Q, K, V, la, kg, dO, scale):
    Bn, H, L = la.shape
    grp = H // Q.shape[1]
    b_dla, b_dkg = np.zeros((Bn, H, L)), np.zeros((Bn, H, L))
    for b in range(Bn):
        for h in range(H):
            b_dla[b, h], b_dkg[b, h] = head_bounds(Q[b, h // grp], K[b, h // grp], V[b, h], la[b, h], None if kg is None else kg[b, h],
                                                   dO[b, h], scale)
    return b_dla, b_dkg


def compare(got, ref, what, with_gate, dots):
    dQ, dK, dV, dla, dkg = got
    check_rows(dQ, ref["dQ"], what + " dQ")
    check_rows(dK, ref["dK"], what + " dK")
    check_rows(dV, ref["dV"], what + " dV")
    b_dla, b_dkg = dots
    check_tokens(dla, b_dla, ref["dlog_decay"], what + " dlog_decay")
    if with_gate:
        check_tokens(dkg, b_dkg, ref["dkey_gate"], what + " dkey_gate")
    else:
        assert dkg is None


def oracle_all(Q, K, V, la, kg, dO, scale):
    n = [Q.float().numpy().astype(np.float64), K.float().numpy().astype(np.float64), V.float().numpy().astype(np.float64),
         la.numpy().astype(np.float64), None if kg is None else kg.numpy().astype(np.float64), dO.float().numpy().astype(np.float64)]
    return oracle_backward(*n, scale=scale), all_bounds(*n, scale)


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


@pytest.mark.parametrize("dqk,dv,H,H_qk", [(128, 128, 2, 2), (64, 64, 3, 3), (128, 64, 4, 1)])
@pytest.mark.parametrize("kind", ["gated_retention", "mamba2"])
@pytest.mark.parametrize("L", [1061, 2560])
def test_few_heads_long_sequence(A, dqk, dv, H, H_qk, kind, L):
    # shapes whose walks the library cuts into segments (2 and 5 here, a ragged last one), forwards and backwards
    Q, K, V, la, kg, dO = inputs(920 + L % 5, 1, H, H_qk, L, dqk, dv, kind)
    scale = 1.0 / math.sqrt(dqk)
    got = run(A, Q, K, V, la, kg, dO, scale)
    ref, dots = oracle_all(Q, K, V, la, kg, dO, scale)
    compare(got, ref, f"segments {kind} {dqk}/{dv} L={L}", kg is not None, dots)


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
        b_dla = token_bounds_proxy(np.sum(qn * ref["dq"], axis=-1), np.sum(kn * ref["dk"], axis=-1))
        check_tokens(dla[b, h], b_dla, ref["dlog_decay"], f"benchmark size ({b},{h}) dlog_decay")

"""Pins for the CPU oracle: closed forms, invariants, a library special case,
a recurrent formulation and brute force.  None of these re-types the oracle's
own formula; each is chosen so a plausible slip in the oracle (dropped term,
wrong sign/index, transposed operand, wrong head mapping) fails at least one.
CPU only.
"""
import math

import numpy as np
import pytest
import torch

from oracle import attention, attention_head, brute, row_stats_head, weights_head

RNG = np.random.default_rng(20250215)


def rnd(*shape):
    return RNG.standard_normal(shape)


# ---------------------------------------------------------------- brute force
@pytest.mark.parametrize("norm,score_mod", [
    ("softmax", "none"), ("softmax", "bias"), ("sigmoid", "bias"),
    ("abssum", "head_decay"), ("abs_of_sum", "head_decay"),
    ("none", "relu"), ("abssum", "none"), ("softmax", "head_decay")])
@pytest.mark.parametrize("mask", ["none", "causal"])
@pytest.mark.parametrize("shape", [(1, 2, 1, 5, 7, 3, 4), (2, 4, 2, 6, 6, 4, 2), (1, 1, 1, 7, 4, 2, 3)])
def test_vectorised_equals_brute(norm, score_mod, mask, shape):
    B, Hq, Hkv, Lq, Lk, Dqk, Dv = shape
    Q, K, V = rnd(B, Hq, Lq, Dqk), rnd(B, Hkv, Lk, Dqk), rnd(B, Hkv, Lk, Dv)
    gamma = [0.9 - 0.1 * h for h in range(Hq)]
    kw = dict(scale=0.7, score_mod=score_mod, bias=-0.3, gamma=gamma, norm=norm, mask=mask)
    np.testing.assert_allclose(attention(Q, K, V, **kw), brute(Q, K, V, **kw), rtol=1e-12, atol=1e-13)


# ------------------------------------------------------------ softmax weights
@pytest.mark.parametrize("mask", ["none", "causal"])
def test_softmax_rows_sum_to_one_and_nonneg(mask):
    q, k = rnd(9, 5), rnd(13, 5)
    p = weights_head(q, k, scale=0.4, norm="softmax", mask=mask)
    assert (p >= 0).all()
    np.testing.assert_allclose(p.sum(axis=1), 1.0, atol=1e-12)
    if mask == "causal":
        off = 13 - 9
        for i in range(9):
            assert (p[i, i + off + 1:] == 0).all()
            assert (p[i, : i + off + 1] > 0).all()


def test_softmax_shift_invariance_via_bias():
    Q, K, V = rnd(1, 2, 6, 4), rnd(1, 2, 8, 4), rnd(1, 2, 8, 3)
    a = attention(Q, K, V, scale=0.5, norm="softmax")
    b = attention(Q, K, V, scale=0.5, score_mod="bias", bias=3.25, norm="softmax")
    np.testing.assert_allclose(a, b, atol=1e-13)


def test_softmax_two_keys_closed_form():
    # one query, two keys: weights are the logistic function of the score gap
    q = np.array([[1.0, 2.0]])
    k = np.array([[0.5, -1.0], [2.0, 0.25]])
    v = np.array([[1.0, 0.0], [0.0, 1.0]])
    scale = 0.3
    s0, s1 = scale * (0.5 - 2.0), scale * (2.0 + 0.5)
    w1 = 1.0 / (1.0 + math.exp(s0 - s1))
    o = attention_head(q, k, v, scale=scale, norm="softmax")
    np.testing.assert_allclose(o, [[1 - w1, w1]], atol=1e-15)


def test_transposed_operand_would_fail():
    # S must be Q K^T, not K Q^T: with L_q == L_k an accidental transpose keeps
    # shapes valid, so pin an asymmetric case against an explicit outer sum.
    q, k, v = rnd(3, 2), rnd(3, 2), rnd(3, 2)
    s = np.array([[sum(q[i, d] * k[j, d] for d in range(2)) for j in range(3)] for i in range(3)])
    e = np.exp(s - s.max(axis=1, keepdims=True))
    ref = (e / e.sum(axis=1, keepdims=True)) @ v
    np.testing.assert_allclose(attention_head(q, k, v, scale=1.0), ref, atol=1e-14)
    assert not np.allclose(s, s.T)


# ------------------------------------------------------------ softmax outputs
@pytest.mark.parametrize("mask", ["none", "causal"])
def test_constant_v_rows_reproduce_v(mask):
    vrow = rnd(5)
    Q, K = rnd(2, 3, 7, 4), rnd(2, 3, 7, 4)
    V = np.broadcast_to(vrow, (2, 3, 7, 5)).copy()
    O = attention(Q, K, V, scale=0.5, norm="softmax", mask=mask)
    np.testing.assert_allclose(O, np.broadcast_to(vrow, O.shape), atol=1e-13)


def test_single_key_returns_its_v_row():
    Q, K, V = rnd(1, 2, 5, 4), rnd(1, 2, 1, 4), rnd(1, 2, 1, 3)
    O = attention(Q, K, V, scale=0.5, norm="softmax")
    np.testing.assert_allclose(O, np.broadcast_to(V, O.shape), atol=1e-14)


def test_zero_q_gives_mean_and_causal_prefix_mean():
    K, V = rnd(1, 1, 6, 4), rnd(1, 1, 6, 3)
    Q = np.zeros((1, 1, 6, 4))
    O = attention(Q, K, V, scale=0.5, norm="softmax")
    np.testing.assert_allclose(O[0, 0], np.broadcast_to(V[0, 0].mean(axis=0), (6, 3)), atol=1e-14)
    Oc = attention(Q, K, V, scale=0.5, norm="softmax", mask="causal")
    pref = np.cumsum(V[0, 0], axis=0) / np.arange(1, 7)[:, None]
    np.testing.assert_allclose(Oc[0, 0], pref, atol=1e-14)


def test_kv_permutation_invariance_noncausal():
    Q, K, V = rnd(1, 1, 5, 4), rnd(1, 1, 9, 4), rnd(1, 1, 9, 3)
    perm = RNG.permutation(9)
    a = attention(Q, K, V, scale=0.5)
    b = attention(Q, K[:, :, perm], V[:, :, perm], scale=0.5)
    np.testing.assert_allclose(a, b, atol=1e-13)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("shape", [(1, 2, 16, 16, 8, 8), (2, 3, 33, 33, 16, 24), (1, 2, 64, 64, 64, 64)])
def test_softmax_equals_library_sdpa_fp64(causal, shape):
    # library special case: torch's CPU scaled_dot_product_attention in fp64
    B, H, Lq, Lk, Dqk, Dv = shape
    Q, K, V = rnd(B, H, Lq, Dqk), rnd(B, H, Lk, Dqk), rnd(B, H, Lk, Dv)
    scale = 1.0 / math.sqrt(Dqk)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(Q), torch.from_numpy(K), torch.from_numpy(V),
        is_causal=causal, scale=scale).numpy()
    got = attention(Q, K, V, scale=scale, norm="softmax", mask="causal" if causal else "none")
    np.testing.assert_allclose(got, ref, atol=1e-12)


def test_softmax_no_overflow_for_huge_scores():
    Q = np.full((1, 1, 2, 2), 100.0)
    K = np.array([[[[100.0, 0.0], [-100.0, 0.0], [100.0, 0.0]]]])
    V = np.array([[[[1.0], [5.0], [3.0]]]])
    O = attention(Q, K, V, scale=1.0)
    assert np.isfinite(O).all()
    np.testing.assert_allclose(O, 2.0, atol=1e-12)


# --------------------------------------------------------------------- causal
@pytest.mark.parametrize("norm,score_mod", [("softmax", "none"), ("sigmoid", "bias"), ("abssum", "none")])
@pytest.mark.parametrize("Lq,Lk", [(6, 6), (4, 9), (1, 5)])
def test_causal_row_equals_noncausal_on_prefix(norm, score_mod, Lq, Lk):
    q, k, v = rnd(Lq, 4), rnd(Lk, 4), rnd(Lk, 3)
    kw = dict(scale=0.6, score_mod=score_mod, bias=-0.2, norm=norm)
    full = attention_head(q, k, v, mask="causal", **kw)
    off = Lk - Lq
    for i in range(Lq):
        n = i + off + 1
        row = attention_head(q[i:i + 1], k[:n], v[:n], mask="none", **kw)
        np.testing.assert_allclose(full[i], row[0], atol=1e-13)


def test_causal_more_queries_than_keys_gives_zero_rows():
    # bottom-right alignment: the first L_q - L_k queries see no key at all
    q, k, v = rnd(5, 3), rnd(2, 3), rnd(2, 2)
    for norm in ("softmax", "sigmoid", "abssum"):
        o = attention_head(q, k, v, scale=1.0, norm=norm, mask="causal")
        assert (o[:3] == 0).all() and np.isfinite(o).all()
        assert (o[3:] != 0).any()


# ------------------------------------------------------------------------ GQA
def test_gqa_equals_mha_with_repeated_kv():
    Q, K, V = rnd(2, 6, 5, 4), rnd(2, 2, 7, 4), rnd(2, 2, 7, 3)
    a = attention(Q, K, V, scale=0.5, mask="causal")
    b = attention(Q, np.repeat(K, 3, axis=1), np.repeat(V, 3, axis=1), scale=0.5, mask="causal")
    np.testing.assert_allclose(a, b, atol=1e-14)
    # and the group is contiguous: q heads 0..2 read kv head 0
    c = attention(Q[:, :3], K[:, :1], V[:, :1], scale=0.5, mask="causal")
    np.testing.assert_allclose(a[:, :3], c, atol=1e-14)


# -------------------------------------------------- D_qk != D_v, zero padding
@pytest.mark.parametrize("norm,score_mod", [("softmax", "none"), ("abssum", "head_decay")])
def test_zero_padding_equivalence(norm, score_mod):
    # Section 5.2: unequal head dims are equivalent to padding, only cheaper
    Q, K, V = rnd(1, 2, 6, 3), rnd(1, 2, 6, 3), rnd(1, 2, 6, 5)
    kw = dict(scale=0.5, norm=norm, score_mod=score_mod, gamma=[0.9, 0.8], mask="causal")
    a = attention(Q, K, V, **kw)
    Qp = np.concatenate([Q, np.zeros((1, 2, 6, 2))], axis=3)
    Kp = np.concatenate([K, rnd(1, 2, 6, 2)], axis=3)  # padding of Q alone suffices
    Vp = np.concatenate([V, np.zeros((1, 2, 6, 1))], axis=3)
    b = attention(Qp, Kp, Vp, **kw)
    np.testing.assert_allclose(b[..., :5], a, atol=1e-14)
    assert (b[..., 5] == 0).all()


# -------------------------------------------------------------------- sigmoid
def test_sigmoid_zero_q_closed_form():
    L = 16
    K, V = rnd(1, 1, L, 4), rnd(1, 1, L, 3)
    Q = np.zeros((1, 1, L, 4))
    O = attention(Q, K, V, scale=0.5, score_mod="bias", bias=-math.log(L), norm="sigmoid", mask="causal")
    ref = np.cumsum(V[0, 0], axis=0) / (1.0 + L)   # sigmoid(-ln L) = 1/(1+L)
    np.testing.assert_allclose(O[0, 0], ref, atol=1e-14)


def test_sigmoid_single_key_and_symmetry():
    q, k, v = np.array([[2.0, -1.0]]), np.array([[0.5, 3.0]]), np.array([[4.0, -2.0]])
    s = 0.5 * (2.0 * 0.5 - 3.0) + 0.25
    o = attention_head(q, k, v, scale=0.5, score_mod="bias", bias=0.25, norm="sigmoid")
    np.testing.assert_allclose(o, [[4.0 / (1 + math.exp(-s)), -2.0 / (1 + math.exp(-s))]], atol=1e-15)
    qs, ks = rnd(4, 3), rnd(5, 3)
    p = weights_head(qs, ks, scale=1.0, norm="sigmoid")
    pn = weights_head(-qs, ks, scale=1.0, norm="sigmoid")
    assert ((p > 0) & (p < 1)).all()
    np.testing.assert_allclose(p + pn, 1.0, atol=1e-14)


def test_sigmoid_large_positive_score_saturates_to_v():
    q, k, v = np.array([[50.0]]), np.array([[1.0]]), np.array([[3.0]])
    np.testing.assert_allclose(attention_head(q, k, v, scale=1.0, norm="sigmoid"), [[3.0]], atol=1e-12)


# ------------------------------------------------------------------ retention
def _retention_recurrent(q, k, v, gamma, scale):
    """Recurrent pattern of the same function (Section 4.1, recurrent pattern):
    state S_n = gamma S_{n-1} + k_n^T v_n, numerator scale * q_n S_n; for the
    alternative normalizer, z_n = gamma z_{n-1} + k_n."""
    L, Dk = q.shape
    Dv = v.shape[1]
    S = np.zeros((Dk, Dv))
    z = np.zeros(Dk)
    num = np.zeros((L, Dv))
    ssum = np.zeros(L)
    for n in range(L):
        S = gamma * S + np.outer(k[n], v[n])
        z = gamma * z + k[n]
        num[n] = scale * (q[n] @ S)
        ssum[n] = scale * (q[n] @ z)
    return num, ssum


@pytest.mark.parametrize("gamma", [0.96875, 1.0 - 2.0 ** -12, 0.5])
def test_retention_matches_recurrent_form(gamma):
    L = 24
    q, k, v = rnd(L, 6), rnd(L, 6), rnd(L, 5)
    scale = 1.0 / math.sqrt(6)
    num, ssum = _retention_recurrent(q, k, v, gamma, scale)
    # numerator: un-normalised weights times V
    raw = weights_head(q, k, scale=scale, score_mod="head_decay", gamma_h=gamma, norm="none", mask="causal")
    np.testing.assert_allclose(raw @ v, num, atol=1e-12)
    # |sum| normaliser has a recurrent closed form
    o2 = attention_head(q, k, v, scale=scale, score_mod="head_decay", gamma_h=gamma, norm="abs_of_sum", mask="causal")
    np.testing.assert_allclose(o2, num / np.maximum(np.abs(ssum), 1.0)[:, None], atol=1e-12)
    # sum|.| normaliser: O * den == numerator with den recomputed by scalar loops
    o1 = attention_head(q, k, v, scale=scale, score_mod="head_decay", gamma_h=gamma, norm="abssum", mask="causal")
    den = np.array([max(sum(abs(scale * (q[n] @ k[j]) * gamma ** (n - j)) for j in range(n + 1)), 1.0) for n in range(L)])
    np.testing.assert_allclose(o1 * den[:, None], num, atol=1e-12)


def test_retention_nonnegative_scores_make_both_normalisers_agree():
    L = 12
    q, k, v = np.abs(rnd(L, 4)), np.abs(rnd(L, 4)), rnd(L, 3)
    kw = dict(scale=1.0, score_mod="head_decay", gamma_h=0.9, mask="causal")
    np.testing.assert_allclose(attention_head(q, k, v, norm="abssum", **kw),
                               attention_head(q, k, v, norm="abs_of_sum", **kw), atol=1e-14)


def test_retention_special_cases():
    # gamma = 1: plain causal linear attention with the abs-sum normaliser
    L = 10
    q, k, v = rnd(L, 4), rnd(L, 4), rnd(L, 3)
    a = attention_head(q, k, v, scale=0.5, score_mod="head_decay", gamma_h=1.0, norm="abssum", mask="causal")
    b = attention_head(q, k, v, scale=0.5, score_mod="none", norm="abssum", mask="causal")
    np.testing.assert_allclose(a, b, atol=1e-15)
    # single key: O = s / max(|s|, 1) * v, both below and above the clamp
    for qq in (0.25, 4.0):
        o = attention_head(np.array([[qq]]), np.array([[2.0]]), np.array([[3.0, -1.0]]), scale=1.0,
                           score_mod="head_decay", gamma_h=0.9, norm="abssum", mask="causal")
        s = qq * 2.0
        np.testing.assert_allclose(o, [[s / max(abs(s), 1.0) * 3.0, -s / max(abs(s), 1.0)]], atol=1e-15)
    # Q = 0 -> O = 0
    o = attention_head(np.zeros((L, 4)), k, v, scale=0.5, score_mod="head_decay", gamma_h=0.9, norm="abssum", mask="causal")
    assert (o == 0).all()
    # |O| <= max|v| under the sum|.| normaliser
    o = attention_head(q, k, v, scale=3.0, score_mod="head_decay", gamma_h=0.9, norm="abssum", mask="causal")
    assert np.abs(o).max() <= np.abs(v).max() + 1e-12


def test_retention_decay_uses_query_head_index_and_distance():
    # two heads with different gamma, identical q/k/v: head with gamma=0 keeps
    # only the diagonal key, so O_i = s_ii / max(|s_ii|,1) v_i
    L = 6
    q1, k1, v1 = rnd(L, 3), rnd(L, 3), rnd(L, 2)
    Q = np.stack([q1, q1])[None]
    K = np.stack([k1, k1])[None]
    V = np.stack([v1, v1])[None]
    O = attention(Q, K, V, scale=1.0, score_mod="head_decay", gamma=[0.0, 1.0], norm="abssum", mask="causal")
    sd = np.einsum("id,id->i", q1, k1)
    np.testing.assert_allclose(O[0, 0], (sd / np.maximum(np.abs(sd), 1.0))[:, None] * v1, atol=1e-14)
    lin = attention_head(q1, k1, v1, scale=1.0, norm="abssum", mask="causal")
    np.testing.assert_allclose(O[0, 1], lin, atol=1e-14)


# ----------------------------------------------------------------------- relu
def test_relu_attention_closed_form():
    q, k, v = rnd(5, 3), rnd(7, 3), rnd(7, 2)
    o = attention_head(q, k, v, scale=0.5, score_mod="relu", norm="none")
    ref = np.zeros((5, 2))
    for i in range(5):
        for j in range(7):
            ref[i] += max(0.5 * float(q[i] @ k[j]), 0.0) * v[j]
    np.testing.assert_allclose(o, ref, atol=1e-14)


# ------------------------------------------------------------ rows= sub-select
def test_row_subset_is_same_definition():
    q, k, v = rnd(20, 4), rnd(20, 4), rnd(20, 3)
    kw = dict(scale=0.5, score_mod="head_decay", gamma_h=0.9, norm="abssum", mask="causal")
    full = attention_head(q, k, v, **kw)
    rows = np.array([0, 3, 19, 7])
    np.testing.assert_allclose(attention_head(q, k, v, rows=rows, **kw), full[rows], atol=0)


# ------------------------------------------ planted mistakes are caught (CPU)
def test_pins_catch_planted_mistakes():
    """Variants of the definition with one slip each must violate a pin."""
    L = 8
    q, k, v = rnd(L, 4), rnd(L, 4), rnd(L, 3)
    good = attention_head(q, k, v, scale=0.5, mask="causal")
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q)[None], torch.from_numpy(k)[None], torch.from_numpy(v)[None],
        is_causal=True, scale=0.5)[0].numpy()
    np.testing.assert_allclose(good, ref, atol=1e-13)
    # (a) transposed score matrix, (b) strict instead of inclusive causal mask,
    # (c) missing scale: each differs from the library result
    for bad in (
        attention_head(k, q, v, scale=0.5, mask="causal"),
        np.vstack([np.zeros((1, 3)), attention_head(q[1:], k[:-1], v[:-1], scale=0.5, mask="causal")]),
        attention_head(q, k, v, scale=1.0, mask="causal"),
    ):
        assert np.abs(bad - ref).max() > 1e-3


# ---- the row statistic of the normalization (final row scales) -----------------------------------

def _scores_by_loops(q, k, scale, bias, gamma, off):
    """S' element by element (plain Python), None where the causal mask hides the pair."""
    L_q, L_k = q.shape[0], k.shape[0]
    out = [[None] * L_k for _ in range(L_q)]
    for i in range(L_q):
        for j in range(L_k):
            if off is not None and j > i + off:
                continue
            s = sum(float(q[i, d]) * float(k[j, d]) for d in range(q.shape[1])) * scale + bias
            if gamma is not None:
                s *= gamma ** (i + off - j)
            out[i][j] = s
    return out


def test_row_stats_softmax_closed_forms():
    k = rnd(9, 8)
    # Q = 0: every visible score is the bias, so lse = bias + ln(number of visible keys)
    q0 = np.zeros((5, 8))
    got = row_stats_head(q0, k, scale=0.3, score_mod="bias", bias=0.7, norm="softmax")
    assert np.allclose(got, 0.7 + math.log(9), rtol=0, atol=1e-13)
    got = row_stats_head(q0, k, scale=0.3, norm="softmax", mask="causal")       # off = 4: row i sees i + 5 keys
    assert np.allclose(got, [math.log(i + 5) for i in range(5)], rtol=0, atol=1e-13)
    # one key: lse is the modified score itself
    q = rnd(6, 8)
    k1 = rnd(1, 8)
    got = row_stats_head(q, k1, scale=0.25, score_mod="bias", bias=-1.5, norm="softmax")
    assert np.allclose(got, (q @ k1.T)[:, 0] * 0.25 - 1.5, rtol=0, atol=1e-13)
    # a constant added to every score moves lse by that constant
    a = row_stats_head(q, k, scale=0.25, norm="softmax", mask="causal")
    b = row_stats_head(q, k, scale=0.25, score_mod="bias", bias=3.25, norm="softmax", mask="causal")
    assert np.allclose(b - a, 3.25, rtol=0, atol=1e-12)
    # rows with no visible key (L_q > L_k, bottom-right alignment)
    got = row_stats_head(rnd(6, 8), rnd(2, 8), scale=1.0, norm="softmax", mask="causal")
    assert np.isneginf(got[:4]).all() and np.isfinite(got[4:]).all()


def test_row_stats_softmax_against_library_logsumexp_and_weights():
    q, k = rnd(7, 16), rnd(11, 16)
    for mask, off in (("none", None), ("causal", 4)):
        sc = _scores_by_loops(q, k, 0.2, 0.0, None, off)
        got = row_stats_head(q, k, scale=0.2, norm="softmax", mask=mask)
        # torch.logsumexp over the visible scores computed element by element above
        lib = [float(torch.logsumexp(torch.tensor([x for x in row if x is not None], dtype=torch.float64), 0))
               for row in sc]
        assert np.allclose(got, lib, rtol=0, atol=1e-12)
        # and it is the normaliser of the (separately pinned) weights: P_ij = exp(S'_ij - lse_i)
        P = weights_head(q, k, scale=0.2, norm="softmax", mask=mask)
        for i, row in enumerate(sc):
            for j, x in enumerate(row):
                assert abs(P[i, j] - (0.0 if x is None else math.exp(x - got[i]))) < 1e-13
    # huge scores do not overflow
    big = row_stats_head(q * 300, k * 300, scale=1.0, norm="softmax")
    assert np.isfinite(big).all()


def test_row_stats_abs_sums():
    q, k = rnd(6, 8), rnd(10, 8)
    gamma = 0.9
    sc = _scores_by_loops(q, k, 0.5, 0.0, gamma, 4)
    a = row_stats_head(q, k, scale=0.5, score_mod="head_decay", gamma_h=gamma, norm="abssum", mask="causal")
    s = row_stats_head(q, k, scale=0.5, score_mod="head_decay", gamma_h=gamma, norm="abs_of_sum", mask="causal")
    assert np.allclose(a, [sum(abs(x) for x in row if x is not None) for row in sc], rtol=1e-13, atol=0)
    assert np.allclose(s, [sum(x for x in row if x is not None) for row in sc], rtol=0, atol=1e-13)
    # the weights are the scores over max(statistic, 1): sum_j |P_ij| = a / max(a, 1)
    P = weights_head(q, k, scale=0.5, score_mod="head_decay", gamma_h=gamma, norm="abssum", mask="causal")
    assert np.allclose(np.abs(P).sum(axis=1), a / np.maximum(a, 1.0), rtol=1e-13, atol=0)
    # non-negative scores: the two statistics coincide
    qp, kp = np.abs(q), np.abs(k)
    a = row_stats_head(qp, kp, scale=0.5, norm="abssum")
    s = row_stats_head(qp, kp, scale=0.5, norm="abs_of_sum")
    assert np.allclose(a, s, rtol=1e-14, atol=0)
    # norms without a row reduction keep nothing
    for norm in ("sigmoid", "none"):
        with pytest.raises(ValueError):
            row_stats_head(q, k, scale=1.0, norm=norm)


# ---- sliding window mask -------------------------------------------------------------------------

def test_sliding_window_limits():
    q, k, v = rnd(9, 8), rnd(12, 8), rnd(12, 5)
    kw = dict(scale=0.4, norm="softmax")
    # a window that reaches past the first key is the causal mask
    a = attention_head(q, k, v, mask=("sliding_window", 12), **kw)
    b = attention_head(q, k, v, mask="causal", **kw)
    assert np.array_equal(a, b)
    # a window of one key: the output row is the value row on the diagonal (off = 3)
    a = attention_head(q, k, v, mask=("sliding_window", 1), **kw)
    assert np.allclose(a, v[3:12], rtol=0, atol=1e-15)
    # Q = 0: mean of the last W visible value rows
    W = 4
    a = attention_head(np.zeros((9, 8)), k, v, mask=("sliding_window", W), **kw)
    for i in range(9):
        lo = max(0, i + 3 - W + 1)
        assert np.allclose(a[i], v[lo:i + 4].mean(axis=0), rtol=0, atol=1e-14)
    # row i equals unmasked attention over exactly its window of keys
    for i in range(9):
        lo = max(0, i + 3 - W + 1)
        ref = attention_head(q[i:i + 1], k[lo:i + 4], v[lo:i + 4], mask="none", **kw)
        got = attention_head(q, k, v, mask=("sliding_window", W), rows=[i], **kw)
        assert np.allclose(got, ref, rtol=0, atol=1e-14)


@pytest.mark.parametrize("norm,score_mod", [("softmax", "none"), ("sigmoid", "bias"), ("abssum", "head_decay"), ("none", "relu")])
def test_sliding_window_equals_brute(norm, score_mod):
    Q, K, V = rnd(1, 2, 7, 3), rnd(1, 1, 10, 3), rnd(1, 1, 10, 4)
    kw = dict(scale=0.7, score_mod=score_mod, bias=-0.3, gamma=[0.9, 0.8], norm=norm, mask=("sliding_window", 3))
    np.testing.assert_allclose(attention(Q, K, V, **kw), brute(Q, K, V, **kw), rtol=1e-12, atol=1e-13)


# ---------------------------------------------------------------- additive bias tensor
def test_bias_tensor_reduces_to_known_cases():
    B, Hq, Hkv, Lq, Lk, D = 2, 4, 2, 6, 7, 3
    Q, K, V = rnd(B, Hq, Lq, D), rnd(B, Hkv, Lk, D), rnd(B, Hkv, Lk, 4)
    # a constant tensor is the constant bias, for every normalization that takes one
    for norm in ("softmax", "sigmoid", "abssum", "none"):
        a = attention(Q, K, V, scale=0.5, score_mod="bias", bias=0.7, norm=norm, mask="causal")
        b = attention(Q, K, V, scale=0.5, score_mod="bias_tensor", bias_tensor=np.full((1, 1, Lq, Lk), 0.7), norm=norm,
                      mask="causal")
        np.testing.assert_allclose(a, b, atol=1e-14)
    # softmax: a bias of -1e30 above the (bottom-right aligned) diagonal is the causal mask
    tri = np.where(np.arange(Lk)[None, :] <= np.arange(Lq)[:, None] + (Lk - Lq), 0.0, -1e30)[None, None]
    np.testing.assert_allclose(attention(Q, K, V, scale=0.5, score_mod="bias_tensor", bias_tensor=tri),
                               attention(Q, K, V, scale=0.5, mask="causal"), atol=1e-14)
    # softmax ignores a per-row shift of the bias; the log-sum-exp statistic moves by exactly that shift
    bt = rnd(B, Hq, Lq, Lk)
    shift = rnd(B, Hq, Lq, 1)
    np.testing.assert_allclose(attention(Q, K, V, scale=0.5, score_mod="bias_tensor", bias_tensor=bt),
                               attention(Q, K, V, scale=0.5, score_mod="bias_tensor", bias_tensor=bt + shift), atol=1e-13)
    s0 = row_stats_head(Q[1, 2], K[1, 1], scale=0.5, score_mod="bias_tensor", bias_t=bt[1, 2])
    s1 = row_stats_head(Q[1, 2], K[1, 1], scale=0.5, score_mod="bias_tensor", bias_t=(bt + shift)[1, 2])
    np.testing.assert_allclose(s1 - s0, shift[1, 2, :, 0], atol=1e-13)
    # Q = 0: the weights are softmax(bias row) whatever K is -- library softmax
    O = attention(np.zeros_like(Q), K, V, scale=0.5, score_mod="bias_tensor", bias_tensor=bt)
    P = torch.softmax(torch.from_numpy(bt), dim=-1).numpy()
    ref = np.einsum("bhij,bhjd->bhid", P, np.repeat(V, 2, axis=1))
    np.testing.assert_allclose(O, ref, atol=1e-13)


@pytest.mark.parametrize("norm", ["softmax", "sigmoid", "none", "abs_of_sum"])
@pytest.mark.parametrize("mask", ["none", "causal"])
def test_bias_tensor_equals_brute(norm, mask):
    B, Hq, Hkv, Lq, Lk, D = 2, 2, 1, 5, 6, 3
    Q, K, V = rnd(B, Hq, Lq, D), rnd(B, Hkv, Lk, D), rnd(B, Hkv, Lk, 2)
    for shape in ((B, Hq, Lq, Lk), (1, Hq, Lq, Lk), (1, 1, Lq, Lk)):   # per batch and head, shared over batch, over both
        bt = rnd(*shape)
        kw = dict(scale=0.6, score_mod="bias_tensor", bias_tensor=bt, norm=norm, mask=mask)
        np.testing.assert_allclose(attention(Q, K, V, **kw), brute(Q, K, V, **kw), atol=1e-13)

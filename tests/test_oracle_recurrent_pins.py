"""Pins of the recurrent retention oracle against what the mathematics fixes (CPU only)."""
import numpy as np
import pytest

from oracle.attention_oracle import attention_head
from oracle.retention_recurrent_oracle import retention_recurrent, retention_recurrent_head


def _rand(seed, L, dk, dv):
    g = np.random.default_rng(seed)
    return g.standard_normal((L, dk)), g.standard_normal((L, dk)), g.standard_normal((L, dv))


@pytest.mark.parametrize("L,dk,dv,gamma", [(1, 4, 3, 0.9), (7, 8, 5, 0.5), (33, 16, 24, 0.97), (64, 8, 8, 1.0)])
def test_equals_parallel_retention(L, dk, dv, gamma):
    # Recurrent and parallel pattern are two evaluation orders of the same sum (Section 4.1):
    # o_i = scale * sum_{j<=i} gamma^(i-j) (q_i . k_j) v_j; the parallel oracle has pins of its own.
    q, k, v = _rand(L, L, dk, dv)
    got = retention_recurrent_head(q, k, v, scale=0.3, gamma_h=gamma)
    ref = attention_head(q, k, v, scale=0.3, score_mod="head_decay", gamma_h=gamma, norm="none", mask="causal")
    np.testing.assert_allclose(got, ref, rtol=1e-11, atol=1e-11)


def test_gamma_one_is_a_prefix_sum():
    # gamma = 1: h_t = sum_{j<=t} k_j^T v_j, a cumulative sum of outer products
    q, k, v = _rand(5, 20, 6, 4)
    states = np.cumsum(np.einsum("ti,tj->tij", k, v), axis=0)
    ref = 2.0 * np.einsum("ti,tij->tj", q, states)
    np.testing.assert_allclose(retention_recurrent_head(q, k, v, scale=2.0, gamma_h=1.0), ref, rtol=1e-12, atol=1e-12)


def test_two_tokens_by_hand():
    # d_qk = d_v = 1: h_1 = k1 v1, h_2 = g k1 v1 + k2 v2
    q = np.array([[2.0], [3.0]]); k = np.array([[5.0], [7.0]]); v = np.array([[11.0], [13.0]])
    o, h = retention_recurrent_head(q, k, v, scale=0.5, gamma_h=0.25, return_state=True)
    assert o[0, 0] == 0.5 * 2.0 * 55.0
    assert o[1, 0] == 0.5 * 3.0 * (0.25 * 55.0 + 91.0)
    assert h[0, 0] == 0.25 * 55.0 + 91.0


def test_brute_force_triple_loop():
    q, k, v = _rand(9, 6, 3, 2)
    gamma, scale = 0.8, 0.7
    L = 6
    ref = np.zeros((L, 2))
    for i in range(L):
        for j in range(i + 1):
            s = sum(q[i, d] * k[j, d] for d in range(3))
            for e in range(2):
                ref[i, e] += scale * gamma ** (i - j) * s * v[j, e]
    np.testing.assert_allclose(retention_recurrent_head(q, k, v, scale=scale, gamma_h=gamma), ref, rtol=1e-12, atol=1e-12)


def test_planted_mistakes_are_caught():
    # a state that excludes the current token, or a decay applied after the update, must differ from the parallel form
    q, k, v = _rand(3, 12, 4, 4)
    ref = attention_head(q, k, v, scale=1.0, score_mod="head_decay", gamma_h=0.9, norm="none", mask="causal")
    h = np.zeros((4, 4)); wrong1 = np.zeros((12, 4)); wrong2 = np.zeros((12, 4)); h2 = np.zeros((4, 4))
    for t in range(12):
        wrong1[t] = q[t] @ h                      # reads before the update
        h = 0.9 * h + np.outer(k[t], v[t])
        h2 = 0.9 * (h2 + np.outer(k[t], v[t]))    # decays the new token too
        wrong2[t] = q[t] @ h2
    assert np.abs(wrong1 - ref).max() > 1e-3 and np.abs(wrong2 - ref).max() > 1e-3


def test_batched_and_per_head_gamma():
    g = np.random.default_rng(1)
    Q = g.standard_normal((2, 3, 10, 4)); K = g.standard_normal((2, 3, 10, 4)); V = g.standard_normal((2, 3, 10, 5))
    gam = [0.5, 0.9, 1.0]
    O = retention_recurrent(Q, K, V, scale=0.5, gamma=gam)
    for b in range(2):
        for h in range(3):
            np.testing.assert_array_equal(O[b, h], retention_recurrent_head(Q[b, h], K[b, h], V[b, h], scale=0.5, gamma_h=gam[h]))


def test_initial_state_continues_a_sequence():
    # a sequence walked in two pieces, the second starting from the first one's final state, is the sequence walked
    # in one go (which the pins above tie to the parallel form): fixes where h0 enters and what the final state is
    q, k, v = _rand(11, 30, 5, 4)
    full, h_full = retention_recurrent_head(q, k, v, scale=0.4, gamma_h=0.93, return_state=True)
    o1, h1 = retention_recurrent_head(q[:13], k[:13], v[:13], scale=0.4, gamma_h=0.93, return_state=True)
    o2, h2 = retention_recurrent_head(q[13:], k[13:], v[13:], scale=0.4, gamma_h=0.93, return_state=True, h0=h1)
    np.testing.assert_allclose(np.concatenate([o1, o2]), full, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(h2, h_full, rtol=1e-12, atol=1e-12)
    # the final state by its closed form: sum_j gamma^(L-1-j) k_j^T v_j
    w = 0.93 ** (29 - np.arange(30))
    np.testing.assert_allclose(h_full, np.einsum("t,ti,tj->ij", w, k, v), rtol=1e-12, atol=1e-12)

"""Pins of the gated recurrent oracle against what the mathematics fixes (CPU only)."""
import math

import numpy as np
import pytest

from oracle.gated_recurrent_oracle import gated_recurrent, gated_recurrent_head
from oracle.retention_recurrent_oracle import retention_recurrent_head


def _rand(seed, L, dk, dv):
    g = np.random.default_rng(seed)
    return (g.standard_normal((L, dk)), g.standard_normal((L, dk)), g.standard_normal((L, dv)),
            np.log(g.uniform(0.3, 1.0, L)), g.uniform(0.1, 2.0, L))


@pytest.mark.parametrize("gamma", [1.0, 0.96875, 0.5])
def test_constant_gate_is_the_retention_recurrence(gamma):
    # a_t = gamma, g_t = 1: the recurrent retention oracle, which has pins of its own
    q, k, v, _, _ = _rand(1, 40, 8, 6)
    got = gated_recurrent_head(q, k, v, np.full(40, math.log(gamma)), scale=0.7)
    np.testing.assert_allclose(got, retention_recurrent_head(q, k, v, scale=0.7, gamma_h=gamma), rtol=1e-12, atol=1e-12)


def test_no_decay_is_a_gated_prefix_sum():
    # a_t = 1: h_t = sum_{j<=t} g_j k_j^T v_j
    q, k, v, _, g = _rand(2, 25, 5, 4)
    states = np.cumsum(np.einsum("t,ti,tj->tij", g, k, v), axis=0)
    ref = 1.5 * np.einsum("ti,tij->tj", q, states)
    np.testing.assert_allclose(gated_recurrent_head(q, k, v, np.zeros(25), g, scale=1.5), ref, rtol=1e-12, atol=1e-12)


def test_two_tokens_by_hand():
    # d_qk = d_v = 1: h_1 = g1 k1 v1 (the zero state decays to zero), h_2 = a2 h_1 + g2 k2 v2
    q = np.array([[2.0], [3.0]]); k = np.array([[5.0], [7.0]]); v = np.array([[11.0], [13.0]])
    la = np.log(np.array([0.5, 0.25])); g = np.array([2.0, 4.0])
    o, h = gated_recurrent_head(q, k, v, la, g, scale=0.5, return_state=True)
    h1 = 2.0 * 5.0 * 11.0
    h2 = 0.25 * h1 + 4.0 * 7.0 * 13.0
    assert o[0, 0] == pytest.approx(0.5 * 2.0 * h1, rel=1e-15)
    assert o[1, 0] == pytest.approx(0.5 * 3.0 * h2, rel=1e-15)
    assert h[0, 0] == pytest.approx(h2, rel=1e-15)


@pytest.mark.parametrize("L,dk,dv", [(1, 3, 2), (9, 4, 5), (30, 6, 3)])
def test_equals_the_parallel_form_by_loops(L, dk, dv):
    # the same sum in the parallel pattern's order: o_i = scale sum_{j<=i} (prod_{r=j+1..i} a_r) g_j (q_i . k_j) v_j
    q, k, v, la, g = _rand(3 + L, L, dk, dv)
    ref = np.zeros((L, dv))
    for i in range(L):
        for j in range(i + 1):
            w = 1.0
            for r in range(j + 1, i + 1):
                w *= math.exp(la[r])
            s = sum(q[i, d] * k[j, d] for d in range(dk))
            for c in range(dv):
                ref[i, c] += 0.3 * w * g[j] * s * v[j, c]
    np.testing.assert_allclose(gated_recurrent_head(q, k, v, la, g, scale=0.3), ref, rtol=1e-11, atol=1e-12)


def test_scalar_state_space_closed_form():
    # Mamba2's recurrence with constant inputs in one dimension: h_t = a h_{t-1} + dt * B * x is a geometric series,
    # y_t = C h_t = C dt B x (1 - a^(t+1)) / (1 - a)
    L, a, dt, Bc, Cc, x = 50, 0.9, 0.05, 1.3, -0.7, 2.0
    o = gated_recurrent_head(np.full((L, 1), Cc), np.full((L, 1), Bc), np.full((L, 1), x), np.full(L, math.log(a)),
                             np.full(L, dt), scale=1.0)
    t = np.arange(L)
    np.testing.assert_allclose(o[:, 0], Cc * dt * Bc * x * (1 - a ** (t + 1)) / (1 - a), rtol=1e-12)


def test_state_carried_over_pieces_and_final_state():
    q, k, v, la, g = _rand(7, 37, 6, 5)
    o, h = gated_recurrent_head(q, k, v, la, g, scale=0.4, return_state=True)
    o1, h1 = gated_recurrent_head(q[:13], k[:13], v[:13], la[:13], g[:13], scale=0.4, return_state=True)
    o2, h2 = gated_recurrent_head(q[13:], k[13:], v[13:], la[13:], g[13:], scale=0.4, h0=h1, return_state=True)
    np.testing.assert_allclose(np.concatenate([o1, o2]), o, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(h2, h, rtol=1e-12, atol=1e-12)
    # closed form of the final state: sum_j exp(sum_{r>j} ln a_r) g_j k_j^T v_j
    tail = np.concatenate([np.cumsum(la[::-1])[::-1][1:], [0.0]])
    ref = np.einsum("t,ti,tj->ij", np.exp(tail) * g, k, v)
    np.testing.assert_allclose(h, ref, rtol=1e-11, atol=1e-12)


def test_grouped_query_key_heads():
    # Mamba2: B and C (k and q) are shared by the value heads of a group
    g = np.random.default_rng(11)
    B, H, Hqk, L, dk, dv = 2, 6, 2, 12, 4, 3
    Q, K = g.standard_normal((B, Hqk, L, dk)), g.standard_normal((B, Hqk, L, dk))
    V, la, kg = g.standard_normal((B, H, L, dv)), np.log(g.uniform(0.5, 1, (B, H, L))), g.uniform(0.1, 1, (B, H, L))
    got = gated_recurrent(Q, K, V, la, kg, scale=0.2)
    ref = gated_recurrent(np.repeat(Q, 3, axis=1), np.repeat(K, 3, axis=1), V, la, kg, scale=0.2)
    np.testing.assert_array_equal(got, ref)
    np.testing.assert_allclose(got[1, 4], gated_recurrent_head(Q[1, 1], K[1, 1], V[1, 4], la[1, 4], kg[1, 4], scale=0.2), rtol=1e-14)


def test_planted_mistakes_are_caught():
    # (a) decay applied after the update instead of before; (b) the gate of the wrong token; (c) decay of token t
    # applied to the read-out as well -- each must disagree with the loop form above
    q, k, v, la, g = _rand(21, 16, 4, 4)
    good = gated_recurrent_head(q, k, v, la, g, scale=1.0)

    def variant(kind):
        h = np.zeros((4, 4)); o = np.zeros((16, 4))
        for t in range(16):
            a = math.exp(la[t])
            if kind == "after":
                h = a * (h + np.outer(g[t] * k[t], v[t]))
            elif kind == "gate_prev":
                h = a * h + np.outer(g[t - 1] * k[t], v[t])
            else:
                h = a * h + np.outer(g[t] * k[t], v[t])
            o[t] = q[t] @ h * (a if kind == "readout" else 1.0)
        return o
    for kind in ("after", "gate_prev", "readout"):
        assert np.abs(variant(kind) - good).max() > 1e-3, kind
    np.testing.assert_allclose(variant("none"), good, rtol=1e-13, atol=1e-13)

"""Pins of the backward oracle of the gated recurrent pattern against what the mathematics fixes (CPU only): finite
differences of the pinned forward oracle, a library's automatic differentiation of an independently written loop,
closed forms, identities that follow from the form of the recurrence, the attention backward oracle on the
constant-decay case, and planted mistakes that these pins must catch."""
import math

import numpy as np
import pytest
import torch

from oracle import attention_backward_head
from oracle.gated_recurrent_backward_oracle import gated_recurrent_backward, gated_recurrent_backward_head
from oracle.gated_recurrent_oracle import gated_recurrent, gated_recurrent_head


def _rand(seed, L, dk, dv):
    g = np.random.default_rng(seed)
    return dict(q=g.standard_normal((L, dk)), k=g.standard_normal((L, dk)), v=g.standard_normal((L, dv)),
                la=np.log(g.uniform(0.3, 1.0, L)), g=g.uniform(0.1, 2.0, L), dO=g.standard_normal((L, dv)),
                h0=g.standard_normal((dk, dv)), dh=g.standard_normal((dk, dv)))


def _loss(x, scale, with_state):
    """The scalar whose gradient the backward oracle returns: sum(O * dO) + sum(h_final * dh)."""
    o, h = gated_recurrent_head(x["q"], x["k"], x["v"], x["la"], x["g"], scale=scale,
                                h0=x["h0"] if with_state else None, return_state=True)
    return float(np.sum(o * x["dO"]) + (np.sum(h * x["dh"]) if with_state else 0.0))


@pytest.mark.parametrize("L,dk,dv,with_state", [(1, 3, 2, False), (7, 4, 3, False), (7, 4, 3, True), (70, 3, 5, True)])
def test_central_finite_differences_of_the_forward_oracle(L, dk, dv, with_state):
    # every input, element by element (70 tokens cross a checkpoint of the backward walk)
    x = _rand(10 + L, L, dk, dv)
    scale = 0.6
    r = gated_recurrent_backward_head(x["q"], x["k"], x["v"], x["la"], x["g"], x["dO"], scale=scale,
                                      h0=x["h0"] if with_state else None, dh_out=x["dh"] if with_state else None)
    eps = 1e-6
    names = [("q", "dq"), ("k", "dk"), ("v", "dv"), ("la", "dlog_decay"), ("g", "dkey_gate")] + ([("h0", "dh0")] if with_state else [])
    rng = np.random.default_rng(0)
    for name, gname in names:
        flat = x[name].reshape(-1)
        idx = range(flat.size) if flat.size <= 60 else rng.choice(flat.size, 60, replace=False)
        for e in idx:
            old = flat[e]
            flat[e] = old + eps
            up = _loss(x, scale, with_state)
            flat[e] = old - eps
            dn = _loss(x, scale, with_state)
            flat[e] = old
            fd = (up - dn) / (2 * eps)
            got = r[gname].reshape(-1)[e]
            assert got == pytest.approx(fd, rel=2e-6, abs=2e-6), (name, e, got, fd)


@pytest.mark.parametrize("with_gate", [False, True])
def test_library_autodiff_of_an_independent_loop(with_gate):
    # the recurrence written once more with torch fp64 tensors; torch.autograd differentiates it
    x = _rand(31, 23, 5, 4)
    t = {n: torch.tensor(x[n], dtype=torch.float64, requires_grad=True) for n in ("q", "k", "v", "la", "g", "h0")}
    h = t["h0"]
    loss = torch.zeros((), dtype=torch.float64)
    for i in range(23):
        kk = t["k"][i] * t["g"][i] if with_gate else t["k"][i]
        h = torch.exp(t["la"][i]) * h + kk[:, None] * t["v"][i][None, :]
        loss = loss + torch.sum(0.4 * (t["q"][i] @ h) * torch.tensor(x["dO"][i]))
    loss = loss + torch.sum(h * torch.tensor(x["dh"]))
    loss.backward()
    r = gated_recurrent_backward_head(x["q"], x["k"], x["v"], x["la"], x["g"] if with_gate else None, x["dO"], scale=0.4,
                                      h0=x["h0"], dh_out=x["dh"])
    for name, gname in (("q", "dq"), ("k", "dk"), ("v", "dv"), ("la", "dlog_decay"), ("h0", "dh0")):
        np.testing.assert_allclose(r[gname], t[name].grad.numpy(), rtol=1e-11, atol=1e-11, err_msg=name)
    if with_gate:
        np.testing.assert_allclose(r["dkey_gate"], t["g"].grad.numpy(), rtol=1e-11, atol=1e-11)


def test_two_tokens_by_hand():
    # d_qk = d_v = 1, h_0 = 0, scale c: o_1 = c q1 g1 k1 v1, o_2 = c q2 (a2 g1 k1 v1 + g2 k2 v2); loss = o_1 d1 + o_2 d2
    q1, q2, k1, k2, v1, v2 = 2.0, 3.0, 5.0, 7.0, 11.0, 13.0
    a1, a2, g1, g2, d1, d2, c = 0.5, 0.25, 2.0, 4.0, 1.5, -0.5, 0.5
    r = gated_recurrent_backward_head([[q1], [q2]], [[k1], [k2]], [[v1], [v2]], np.log([a1, a2]), [g1, g2], [[d1], [d2]], scale=c)
    assert r["dq"][0, 0] == pytest.approx(c * g1 * k1 * v1 * d1, rel=1e-14)
    assert r["dq"][1, 0] == pytest.approx(c * (a2 * g1 * k1 * v1 + g2 * k2 * v2) * d2, rel=1e-14)
    assert r["dk"][0, 0] == pytest.approx(c * g1 * v1 * (q1 * d1 + q2 * a2 * d2), rel=1e-14)
    assert r["dk"][1, 0] == pytest.approx(c * q2 * g2 * v2 * d2, rel=1e-14)
    assert r["dv"][0, 0] == pytest.approx(c * g1 * k1 * (q1 * d1 + q2 * a2 * d2), rel=1e-14)
    assert r["dkey_gate"][0] == pytest.approx(c * k1 * v1 * (q1 * d1 + q2 * a2 * d2), rel=1e-14)
    assert r["dlog_decay"][1] == pytest.approx(c * q2 * a2 * g1 * k1 * v1 * d2, rel=1e-14)   # d/d ln a2 = a2 d/d a2
    assert r["dlog_decay"][0] == 0.0                                                            # a1 multiplies the zero state


def test_identities_of_the_bilinear_form():
    # o_t is linear in q_t; token j enters every later state through g_j k_j^T v_j, linear in each factor.  Hence
    # q_t . dq_t = o_t . dO_t, and k_j . dk_j = v_j . dv_j = g_j dg_j; and with B_i the cumulative log-decay, which
    # enters weight (i, j) as exp(B_i - B_j): dlog_decay_t = sum_{i >= t} (q_i . dq_i - k_i . dk_i)  (no state handed in)
    x = _rand(41, 50, 6, 4)
    r = gated_recurrent_backward_head(x["q"], x["k"], x["v"], x["la"], x["g"], x["dO"], scale=0.3)
    o = gated_recurrent_head(x["q"], x["k"], x["v"], x["la"], x["g"], scale=0.3)
    qdq, kdk = np.sum(x["q"] * r["dq"], axis=1), np.sum(x["k"] * r["dk"], axis=1)
    np.testing.assert_allclose(qdq, np.sum(o * x["dO"], axis=1), rtol=1e-10, atol=1e-11)
    np.testing.assert_allclose(kdk, np.sum(x["v"] * r["dv"], axis=1), rtol=1e-10, atol=1e-11)
    np.testing.assert_allclose(kdk, x["g"] * r["dkey_gate"], rtol=1e-10, atol=1e-11)
    np.testing.assert_allclose(r["dlog_decay"], np.cumsum((qdq - kdk)[::-1])[::-1], rtol=1e-9, atol=1e-10)


def test_linear_in_the_upstream_gradient():
    x = _rand(42, 20, 4, 4)
    r1 = gated_recurrent_backward_head(x["q"], x["k"], x["v"], x["la"], x["g"], x["dO"], scale=0.5)
    r2 = gated_recurrent_backward_head(x["q"], x["k"], x["v"], x["la"], x["g"], -2.0 * x["dO"], scale=0.5)
    for n in ("dq", "dk", "dv", "dlog_decay", "dkey_gate"):
        np.testing.assert_allclose(r2[n], -2.0 * r1[n], rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("gamma", [1.0, 0.9])
def test_constant_decay_is_the_parallel_retention_backward(gamma):
    # a_t = gamma, g_t = 1: causal retention without a normalizer, whose backward oracle is pinned on its own
    x = _rand(43, 33, 8, 6)
    r = gated_recurrent_backward_head(x["q"], x["k"], x["v"], np.full(33, math.log(gamma)), None, x["dO"], scale=0.7)
    ref = attention_backward_head(x["q"], x["k"], x["v"], x["dO"], scale=0.7, score_mod="head_decay", gamma_h=gamma,
                                  norm="none", mask="causal")
    for n, m in (("dq", 0), ("dk", 1), ("dv", 2)):
        np.testing.assert_allclose(r[n], ref[m], rtol=1e-10, atol=1e-11, err_msg=n)


def test_grouped_heads_sum_over_the_group():
    rng = np.random.default_rng(44)
    B, H, Hqk, L, dk, dv = 1, 4, 2, 12, 3, 2
    Q, K = rng.standard_normal((B, Hqk, L, dk)), rng.standard_normal((B, Hqk, L, dk))
    V, dO = rng.standard_normal((B, H, L, dv)), rng.standard_normal((B, H, L, dv))
    la, g = np.log(rng.uniform(0.5, 1.0, (B, H, L))), rng.uniform(0.5, 1.5, (B, H, L))
    r = gated_recurrent_backward(Q, K, V, la, g, dO, scale=0.8)
    # the same with q/k heads repeated per value head, then summed over each group
    rr = gated_recurrent_backward(np.repeat(Q, 2, axis=1), np.repeat(K, 2, axis=1), V, la, g, dO, scale=0.8)
    np.testing.assert_allclose(r["dQ"], rr["dQ"].reshape(B, Hqk, 2, L, dk).sum(axis=2), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(r["dK"], rr["dK"].reshape(B, Hqk, 2, L, dk).sum(axis=2), rtol=1e-12, atol=1e-12)
    for n in ("dV", "dlog_decay", "dkey_gate"):
        np.testing.assert_allclose(r[n], rr[n], rtol=1e-12, atol=1e-12)
    # and against finite differences of the pinned grouped forward oracle, on a few elements of Q
    eps = 1e-6
    for (h, t, d) in ((0, 0, 0), (1, 5, 2), (1, 11, 1)):
        Qp, Qm = Q.copy(), Q.copy()
        Qp[0, h, t, d] += eps
        Qm[0, h, t, d] -= eps
        fd = (np.sum(gated_recurrent(Qp, K, V, la, g, scale=0.8) * dO) - np.sum(gated_recurrent(Qm, K, V, la, g, scale=0.8) * dO)) / (2 * eps)
        assert r["dQ"][0, h, t, d] == pytest.approx(fd, rel=1e-6, abs=1e-6)


def test_planted_mistakes_are_caught():
    # each variant of the backward walk below carries one mistake; finite differences of the forward oracle (the
    # first pin above) must tell it from the right walk
    x = _rand(45, 9, 3, 3)
    scale = 0.9
    L = 9
    a, g = np.exp(x["la"]), x["g"]

    def walk(kind):
        hs = [np.zeros((3, 3))]
        for t in range(L):
            hs.append(a[t] * hs[-1] + np.outer(g[t] * x["k"][t], x["v"][t]))
        D = np.zeros((3, 3))
        out = dict(dq=np.zeros((L, 3)), dk=np.zeros((L, 3)), dlog_decay=np.zeros(L))
        for t in range(L - 1, -1, -1):
            if kind == "decay_before_readout":      # the factor a_t applied before token t's own read-out is added
                D = a[t] * D
            D = D + scale * np.outer(x["q"][t], x["dO"][t])
            out["dq"][t] = scale * ((hs[t] if kind == "stale_state" else hs[t + 1]) @ x["dO"][t])   # h_{t-1} instead of h_t
            out["dk"][t] = g[t] * (D @ x["v"][t])
            out["dlog_decay"][t] = (1.0 if kind == "no_chain_through_exp" else a[t]) * np.sum(D * hs[t])
            if kind != "decay_before_readout":
                D = a[t] * D
        return out

    good = gated_recurrent_backward_head(x["q"], x["k"], x["v"], x["la"], x["g"], x["dO"], scale=scale)
    right = walk("none")
    for n in right:
        np.testing.assert_allclose(right[n], good[n], rtol=1e-12, atol=1e-12)
    assert np.abs(walk("decay_before_readout")["dk"] - good["dk"]).max() > 1e-3
    assert np.abs(walk("stale_state")["dq"] - good["dq"]).max() > 1e-3
    assert np.abs(walk("no_chain_through_exp")["dlog_decay"] - good["dlog_decay"]).max() > 1e-3

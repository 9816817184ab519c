"""Pins for the backward oracle: finite differences of the forward oracle (pinned on its own in
test_oracle_pins.py), a library autograd for the softmax special case, closed forms, invariants, and planted
mistakes that these pins must catch.  CPU only."""
import math

import numpy as np
import pytest
import torch

from oracle import attention, attention_backward, attention_backward_head

RNG = np.random.default_rng(20250301)


def rnd(*shape):
    return RNG.standard_normal(shape)


def finite_difference(fn, x, dO, eps=1e-6):
    """d sum(fn(x) * dO) / dx by central differences, element by element."""
    g = np.zeros_like(x)
    it = np.nditer(x, flags=["multi_index"])
    for _ in it:
        idx = it.multi_index
        old = x[idx]
        x[idx] = old + eps
        up = (fn() * dO).sum()
        x[idx] = old - eps
        dn = (fn() * dO).sum()
        x[idx] = old
        g[idx] = (up - dn) / (2 * eps)
    return g


CASES = [("softmax", "none"), ("softmax", "bias"), ("sigmoid", "bias"), ("softmax", "head_decay"),
         ("none", "relu"), ("none", "none"), ("none", "head_decay"), ("sigmoid", "none"),
         ("abssum", "head_decay"), ("abs_of_sum", "head_decay"), ("abssum", "none"), ("abs_of_sum", "bias")]


@pytest.mark.parametrize("norm,score_mod", CASES)
@pytest.mark.parametrize("mask", ["none", "causal", ("sliding_window", 3)])
@pytest.mark.parametrize("shape", [(1, 2, 1, 5, 7, 3, 4), (2, 4, 2, 6, 4, 4, 2)])
def test_gradients_equal_finite_differences_of_the_forward_oracle(norm, score_mod, mask, shape):
    B, Hq, Hkv, Lq, Lk, Dqk, Dv = shape
    Q, K, V, dO = rnd(B, Hq, Lq, Dqk), rnd(B, Hkv, Lk, Dqk), rnd(B, Hkv, Lk, Dv), rnd(B, Hq, Lq, Dv)
    kw = dict(scale=0.7, score_mod=score_mod, bias=-0.3, gamma=np.linspace(0.8, 0.95, Hq), norm=norm, mask=mask)
    dQ, dK, dV = attention_backward(Q, K, V, dO, **kw)
    fwd = lambda: attention(Q, K, V, **kw)  # noqa: E731
    np.testing.assert_allclose(dQ, finite_difference(fwd, Q, dO), atol=2e-7)
    np.testing.assert_allclose(dK, finite_difference(fwd, K, dO), atol=2e-7)
    np.testing.assert_allclose(dV, finite_difference(fwd, V, dO), atol=2e-7)


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("shape", [(1, 2, 2, 16, 16, 8, 8), (2, 4, 2, 33, 33, 16, 24), (1, 6, 2, 20, 20, 64, 32)])
def test_softmax_equals_library_autograd_fp64(causal, shape):
    # library special case: autograd through torch's CPU scaled_dot_product_attention in fp64,
    # grouped heads written out as repeated k/v heads
    B, Hq, Hkv, Lq, Lk, Dqk, Dv = shape
    g = Hq // Hkv
    Q, K, V, dO = rnd(B, Hq, Lq, Dqk), rnd(B, Hkv, Lk, Dqk), rnd(B, Hkv, Lk, Dv), rnd(B, Hq, Lq, Dv)
    scale = 1.0 / math.sqrt(Dqk)
    tq, tk, tv = (torch.from_numpy(x).requires_grad_(True) for x in (Q, K, V))
    out = torch.nn.functional.scaled_dot_product_attention(
        tq, tk.repeat_interleave(g, dim=1), tv.repeat_interleave(g, dim=1), is_causal=causal, scale=scale)
    out.backward(torch.from_numpy(dO))
    dQ, dK, dV = attention_backward(Q, K, V, dO, scale=scale, norm="softmax", mask="causal" if causal else "none")
    np.testing.assert_allclose(dQ, tq.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(dK, tk.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(dV, tv.grad.numpy(), atol=1e-12)


def test_softmax_two_keys_closed_form():
    # one query, two keys, scalar values: O = v1 + p (v0 - v1) with p = 1 / (1 + exp(-(s0 - s1))),
    # so dO/ds0 = p (1 - p) (v0 - v1) and dq = scale * that * (k0 - k1)
    q, k, v = np.array([[0.5, -1.0]]), np.array([[1.0, 2.0], [-0.5, 0.25]]), np.array([[3.0], [-1.0]])
    scale, do = 0.8, np.array([[1.7]])
    s = scale * (q @ k.T)[0]
    p = 1.0 / (1.0 + math.exp(-(s[0] - s[1])))
    slope = p * (1 - p) * (v[0, 0] - v[1, 0]) * do[0, 0]
    dq, dk, dv = attention_backward_head(q, k, v, do, scale=scale)
    np.testing.assert_allclose(dq, scale * slope * (k[0] - k[1])[None, :], atol=1e-14)
    np.testing.assert_allclose(dk, scale * slope * np.stack([q[0], -q[0]]), atol=1e-14)
    np.testing.assert_allclose(dv, np.array([[p], [1 - p]]) * do[0, 0], atol=1e-14)


def test_softmax_score_gradients_sum_to_zero_per_row():
    # softmax is invariant to a per-row shift of the scores: with all keys equal to one vector u, every row's
    # score gradients sum to zero, hence dQ = scale * sum_j dS_ij u = 0; and a bias leaves every gradient unchanged
    Lq, Lk, D = 5, 6, 4
    q, v, do = rnd(Lq, D), rnd(Lk, 3), rnd(Lq, 3)
    k = np.tile(rnd(1, D), (Lk, 1))
    dq, _, _ = attention_backward_head(q, k, v, do, scale=0.5, mask="causal")
    np.testing.assert_allclose(dq, 0.0, atol=1e-14)
    k = rnd(Lk, D)
    a = attention_backward_head(q, k, v, do, scale=0.5, mask="causal")
    b = attention_backward_head(q, k, v, do, scale=0.5, mask="causal", score_mod="bias", bias=3.25)
    for x, y in zip(a, b):
        np.testing.assert_allclose(x, y, atol=1e-13)


def test_single_visible_key_passes_do_to_that_value_row_only():
    # causal, L_q = L_k: query 0 sees key 0 alone, its weight is the constant 1: dq_0 = 0 and the first row's
    # upstream gradient goes to v_0 undiminished
    L, D = 4, 3
    q, k, v = rnd(L, D), rnd(L, D), rnd(L, 2)
    do = np.zeros((L, 2))
    do[0] = [1.5, -2.0]
    dq, dk, dv = attention_backward_head(q, k, v, do, scale=1.0, mask="causal")
    np.testing.assert_allclose(dq, 0.0, atol=1e-15)
    np.testing.assert_allclose(dk, 0.0, atol=1e-15)
    np.testing.assert_allclose(dv[0], do[0], atol=1e-15)
    np.testing.assert_allclose(dv[1:], 0.0, atol=1e-15)


def test_rows_without_keys_have_zero_gradient():
    # more queries than keys, causal (bottom-right aligned): the first L_q - L_k queries see nothing
    Lq, Lk = 6, 2
    q, k, v, do = rnd(Lq, 3), rnd(Lk, 3), rnd(Lk, 2), rnd(Lq, 2)
    for norm in ("softmax", "sigmoid", "none"):
        dq, dk, dv = attention_backward_head(q, k, v, do, scale=1.0, norm=norm, mask="causal")
        np.testing.assert_allclose(dq[:Lq - Lk], 0.0, atol=0)
        do2 = do.copy()
        do2[:Lq - Lk] += 5.0   # their upstream gradient reaches nothing
        dq2, dk2, dv2 = attention_backward_head(q, k, v, do2, scale=1.0, norm=norm, mask="causal")
        np.testing.assert_allclose(dk, dk2, atol=0)
        np.testing.assert_allclose(dv, dv2, atol=0)


def test_sigmoid_and_relu_closed_forms():
    # one query, one key, scalar value: O = f(scale q.k + b) v
    q, k, v, do = np.array([[0.3, -0.2]]), np.array([[1.5, 0.5]]), np.array([[2.0]]), np.array([[0.7]])
    scale, b = 1.3, -0.4
    s = scale * (q @ k.T).item() + b
    sg = 1.0 / (1.0 + math.exp(-s))
    dq, dk, dv = attention_backward_head(q, k, v, do, scale=scale, score_mod="bias", bias=b, norm="sigmoid")
    np.testing.assert_allclose(dq, 0.7 * 2.0 * sg * (1 - sg) * scale * k, atol=1e-15)
    np.testing.assert_allclose(dk, 0.7 * 2.0 * sg * (1 - sg) * scale * q, atol=1e-15)
    np.testing.assert_allclose(dv, [[0.7 * sg]], atol=1e-15)
    for sign in (1.0, -1.0):   # ReLU: identity slope on a positive score, none on a negative one
        dq, dk, dv = attention_backward_head(sign * q, k, v, do, scale=scale, score_mod="relu", norm="none")
        live = 1.0 if sign * (q @ k.T).item() > 0 else 0.0
        np.testing.assert_allclose(dq, live * 0.7 * 2.0 * scale * k, atol=1e-15)
        np.testing.assert_allclose(dv, [[live * 0.7 * scale * sign * (q @ k.T).item()]], atol=1e-15)


@pytest.mark.parametrize("norm", ["abssum", "abs_of_sum"])
def test_abs_sum_normalizers_on_both_sides_of_the_clamp(norm):
    # rows below the clamp (r < 1) behave as no normalization; rows above it follow the quotient rule -- checked
    # against finite differences with scores scaled to land on either side, and in closed form for one key:
    # P = s / max(|s|, 1), so above the clamp O = sign(s) v is flat in s (zero gradient to q and k)
    L, D = 6, 3
    q, k, v, do = rnd(L, D), rnd(L, D), rnd(L, 2), rnd(L, 2)
    Q, K, V, dO = q[None, None], k[None, None], v[None, None], do[None, None]
    for scale in (0.02, 0.5, 3.0):
        kw = dict(scale=scale, norm=norm, mask="causal", score_mod="head_decay", gamma=[0.9])
        from oracle import row_stats_head
        r = np.abs(row_stats_head(q, k, scale=scale, norm=norm, mask="causal", score_mod="head_decay", gamma_h=0.9))
        assert np.abs(r - 1.0).min() > 1e-3          # no row sits on the kink
        dQ, dK, dV = attention_backward(Q, K, V, dO, **kw)
        fwd = lambda: attention(Q, K, V, **kw)  # noqa: E731
        np.testing.assert_allclose(dQ, finite_difference(fwd, Q, dO), atol=5e-7)
        np.testing.assert_allclose(dK, finite_difference(fwd, K, dO), atol=5e-7)
        np.testing.assert_allclose(dV, finite_difference(fwd, V, dO), atol=5e-7)
    assert (r > 1).any()                             # the largest scale is above the clamp somewhere
    q1, k1, v1, d1 = np.array([[2.0, 0.0]]), np.array([[1.5, 0.0]]), np.array([[3.0]]), np.array([[1.0]])
    dq, dk, dv = attention_backward_head(q1, k1, v1, d1, scale=1.0, norm=norm)   # s = 3 > 1: P = 1
    np.testing.assert_allclose(dq, 0.0, atol=1e-15)
    np.testing.assert_allclose(dk, 0.0, atol=1e-15)
    np.testing.assert_allclose(dv, [[1.0]], atol=1e-15)
    dq, dk, dv = attention_backward_head(q1, k1, v1, d1, scale=0.1, norm=norm)   # s = 0.3 < 1: P = s
    np.testing.assert_allclose(dq, 0.1 * 3.0 * k1, atol=1e-15)
    np.testing.assert_allclose(dv, [[0.3]], atol=1e-15)


@pytest.mark.parametrize("norm", ["softmax", "sigmoid", "none"])
@pytest.mark.parametrize("mask", ["none", "causal"])
def test_bias_tensor_gradients(norm, mask):
    # finite differences of the forward oracle with the same bias tensor (per batch and head, shared over batch,
    # shared over both), and: a constant tensor gives the gradients of the constant bias
    B, Hq, Hkv, Lq, Lk, D = 2, 2, 1, 5, 6, 3
    Q, K, V, dO = rnd(B, Hq, Lq, D), rnd(B, Hkv, Lk, D), rnd(B, Hkv, Lk, 2), rnd(B, Hq, Lq, 2)
    for shape in ((B, Hq, Lq, Lk), (1, Hq, Lq, Lk), (1, 1, Lq, Lk)):
        kw = dict(scale=0.6, score_mod="bias_tensor", bias_tensor=rnd(*shape), norm=norm, mask=mask)
        dQ, dK, dV = attention_backward(Q, K, V, dO, **kw)
        fwd = lambda: attention(Q, K, V, **kw)  # noqa: E731
        np.testing.assert_allclose(dQ, finite_difference(fwd, Q, dO), atol=2e-7)
        np.testing.assert_allclose(dK, finite_difference(fwd, K, dO), atol=2e-7)
        np.testing.assert_allclose(dV, finite_difference(fwd, V, dO), atol=2e-7)
    # the gradient with respect to the bias tensor itself, per batch and head: finite differences in the tensor;
    # for a tensor shared over the batch (or heads) the finite difference is the sum over the sharers
    for shape in ((B, Hq, Lq, Lk), (1, Hq, Lq, Lk), (1, 1, Lq, Lk)):
        bt = rnd(*shape)
        kw = dict(scale=0.6, score_mod="bias_tensor", norm=norm, mask=mask)
        dB = attention_backward(Q, K, V, dO, bias_tensor=bt, with_dbias=True, **kw)[3]
        fd = finite_difference(lambda: attention(Q, K, V, bias_tensor=bt, **kw), bt, dO)
        want = dB.sum(axis=0, keepdims=True) if shape[0] == 1 else dB
        want = want.sum(axis=1, keepdims=True) if shape[1] == 1 else want
        np.testing.assert_allclose(want, fd, atol=3e-7)
    a = attention_backward(Q, K, V, dO, scale=0.6, score_mod="bias", bias=0.4, norm=norm, mask=mask)
    b = attention_backward(Q, K, V, dO, scale=0.6, score_mod="bias_tensor", bias_tensor=np.full((1, 1, Lq, Lk), 0.4), norm=norm,
                           mask=mask)
    for x, y in zip(a, b):
        np.testing.assert_allclose(x, y, atol=1e-14)


def test_gqa_sums_over_the_query_heads_of_a_group():
    B, Hq, Hkv, L, D = 1, 4, 2, 7, 4
    Q, K, V, dO = rnd(B, Hq, L, D), rnd(B, Hkv, L, D), rnd(B, Hkv, L, D), rnd(B, Hq, L, D)
    dQ, dK, dV = attention_backward(Q, K, V, dO, scale=0.5, mask="causal")
    Kr, Vr = np.repeat(K, 2, axis=1), np.repeat(V, 2, axis=1)
    dQr, dKr, dVr = attention_backward(Q, Kr, Vr, dO, scale=0.5, mask="causal")
    np.testing.assert_allclose(dQ, dQr, atol=1e-14)
    np.testing.assert_allclose(dK, dKr.reshape(B, Hkv, 2, L, D).sum(axis=2), atol=1e-14)
    np.testing.assert_allclose(dV, dVr.reshape(B, Hkv, 2, L, D).sum(axis=2), atol=1e-14)


def test_linear_in_the_upstream_gradient():
    q, k, v = rnd(5, 3), rnd(6, 3), rnd(6, 2)
    d1, d2 = rnd(5, 2), rnd(5, 2)
    a = attention_backward_head(q, k, v, d1, scale=0.9, mask="causal")
    b = attention_backward_head(q, k, v, d2, scale=0.9, mask="causal")
    c = attention_backward_head(q, k, v, 2.0 * d1 - 3.0 * d2, scale=0.9, mask="causal")
    for x, y, z in zip(a, b, c):
        np.testing.assert_allclose(z, 2.0 * x - 3.0 * y, atol=1e-13)


def test_pins_catch_planted_mistakes():
    """Plausible slips (a dropped row-sum term, a missing scale, transposed operands, a gradient flowing through
    masked entries) must fail the finite-difference pin."""
    Lq, Lk, D, Dv = 5, 6, 3, 2
    q, k, v, do = rnd(Lq, D), rnd(Lk, D), rnd(Lk, Dv), rnd(Lq, Dv)
    scale = 0.7
    Q, K, V, dO = q[None, None], k[None, None], v[None, None], do[None, None]
    kw = dict(scale=scale, norm="softmax", mask="causal")
    fwd = lambda: attention(Q, K, V, **kw)  # noqa: E731
    fdq, fdk = finite_difference(fwd, Q, dO)[0, 0], finite_difference(fwd, K, dO)[0, 0]
    off = Lk - Lq
    vis = np.arange(Lk)[None, :] <= np.arange(Lq)[:, None] + off
    s = np.where(vis, scale * q @ k.T, -np.inf)
    p = np.exp(s - s.max(axis=1, keepdims=True))
    p /= p.sum(axis=1, keepdims=True)
    dp = do @ v.T
    good = p * (dp - (p * dp).sum(axis=1, keepdims=True))
    assert np.abs(scale * good @ k - fdq).max() < 2e-7          # the right formula passes
    planted = {
        "no row-sum term": p * dp,
        "row sum over unweighted dP": p * (dp - dp.sum(axis=1, keepdims=True)),
        "scale dropped": good / scale,
        "gradient through masked entries": good + np.where(vis, 0.0, 0.01 * dp),
    }
    for name, ds in planted.items():
        assert np.abs(scale * ds @ k - fdq).max() > 1e-4, name
    assert np.abs(scale * good.T @ q - fdk).max() < 2e-7
    assert np.abs(scale * (p * dp).T @ q - fdk).max() > 1e-4     # dK from the unnormalised product

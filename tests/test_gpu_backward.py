"""GPU parity of the backward pass: ae_attn_backward (through the C ABI, fed by the HIP forward pass's output and
row statistic) against the fp64 backward oracle on the same seeded bf16 inputs.  Bar as for the forward pass
(bf16 operands, bf16 weights and score gradients into the second MFMAs, fp32 accumulation): max-abs <= 1e-2 and
mean-abs <= 1e-3, relative to max(1, the largest |reference| of the row)."""
import math

import numpy as np
import pytest
import torch

from oracle import attention_backward
from paper_2502_15349_amd.workloads import C2, Workload, make_grad, make_inputs

pytestmark = pytest.mark.gpu

MAX_ABS, MEAN_ABS = 1e-2, 1e-3
DIMS = [(64, 64), (128, 128), (128, 256), (192, 128)]


@pytest.fixture(scope="module")
def A():
    from paper_2502_15349_amd import ae_attn
    return ae_attn


def hip_backward(A, w, Q, K, V, dO, out_dtype=None):
    dev = torch.device("cuda:0")
    Qd, Kd, Vd, dOd = Q.to(dev), K.to(dev), V.to(dev), dO.to(dev)
    stats = torch.empty((w.B, w.H_q, w.L_q), dtype=torch.float32, device=dev) if w.norm in ("softmax", "abssum", "abs_of_sum") else None
    O = A.run_workload(w, Qd, Kd, Vd, stats=stats, out_dtype=out_dtype)
    dQ, dK, dV = A.attention_backward(Qd, Kd, Vd, O, dOd, stats, scale=w.scale_value, score_mod=w.score_mod, bias=w.bias,
                                      gamma=w.gamma(), norm=w.norm, mask=w.mask, window=w.window)
    torch.cuda.synchronize()
    return [x.cpu().double().numpy() for x in (dQ, dK, dV)]


def oracle_backward(w, Q, K, V, dO):
    return attention_backward(Q, K, V, dO, scale=w.scale_value, score_mod=w.score_mod, bias=w.bias, gamma=w.gamma(),
                              norm=w.norm, mask=w.oracle_mask())


def check(got, ref, what):
    assert np.isfinite(got).all(), f"{what}: non-finite gradient"
    rs = np.maximum(np.abs(ref).max(axis=-1, keepdims=True), 1.0)
    err = np.abs(got - ref) / rs
    print(f"{what}: max_abs {err.max():.3e} mean_abs {err.mean():.3e} |ref|max {np.abs(ref).max():.3e}", flush=True)
    assert err.max() <= MAX_ABS, f"{what}: max-abs {err.max():.3e}"
    assert err.mean() <= MEAN_ABS, f"{what}: mean-abs {err.mean():.3e}"


def run_case(A, w, out_dtype=None, positive_scores=False):
    print(f"case {w}", flush=True)
    Q, K, V = make_inputs(w)
    if positive_scores:   # |q|, |k|: every score positive, so that a signed row sum does not cancel
        Q, K = Q.abs(), K.abs()
    dO = make_grad(w)
    got, ref = hip_backward(A, w, Q, K, V, dO, out_dtype), oracle_backward(w, Q, K, V, dO)
    for name, g, r in zip(("dQ", "dK", "dV"), got, ref):
        check(g, r, f"{w.name} {name}")


VARIANTS = {
    "softmax": dict(),
    "softmax_causal": dict(mask="causal"),
    "softmax_bias_causal": dict(score_mod="bias", bias=0.75, mask="causal"),
    "softmax_negative_scale": dict(scale=-0.11, mask="causal"),
    "sigmoid_causal": dict(score_mod="bias", norm="sigmoid", mask="causal", bias=-math.log(300.0)),
    "sigmoid": dict(norm="sigmoid", score_mod="bias", bias=-3.0),
    # no normalization: ReLU attention, and the bare (biased) scores as weights
    "relu": dict(score_mod="relu", norm="none", scale=0.01),
    "relu_causal": dict(score_mod="relu", norm="none", mask="causal", scale=0.01),
    "none_bias_causal": dict(score_mod="bias", bias=0.02, norm="none", mask="causal", scale=0.005),
    # retention (per-head decay, abs-sum normalizers): rows above the clamp, and (tiny scale) below it
    "retnet_abssum": dict(score_mod="head_decay", norm="abssum", mask="causal", decay=True),
    "retnet_abs_of_sum": dict(score_mod="head_decay", norm="abs_of_sum", mask="causal", decay=True),
    "retnet_abssum_below_clamp": dict(score_mod="head_decay", norm="abssum", mask="causal", decay=True, scale=0.0005),
    "decay_nonorm": dict(score_mod="head_decay", norm="none", mask="causal", decay=True, scale=0.01),
    "abssum_plain": dict(norm="abssum"),
    # (|sum| as normalizer: a bias that keeps the row sums away from cancellation, where the statistic itself --
    # and with it every gradient of the row -- is ill-conditioned)
    "abs_of_sum_bias_causal": dict(norm="abs_of_sum", score_mod="bias", bias=3.0, mask="causal"),
}


@pytest.mark.parametrize("dims", DIMS, ids=lambda d: f"d{d[0]}_{d[1]}")
@pytest.mark.parametrize("variant", sorted(VARIANTS))
def test_backward_small_ragged(A, dims, variant):
    # 3 own tiles with a ragged tail on either side, 5-6 LDS tiles with a ragged tail, grouped heads 2:1
    # The |sum| normalizer with zero-mean scores divides by a row sum that cancels (sum |s'| can be 50 x |sum s'|):
    # the operator itself is ill-conditioned there, gradients reach hundreds and no bf16 path meets an absolute bar.
    # With decay (no bias to shift the scores) it is therefore run on |q|, |k|.
    run_case(A, Workload(variant, 40, 2, 4, 2, 300, 333, dims[0], dims[1], **VARIANTS[variant]),
             positive_scores=variant == "retnet_abs_of_sum")


@pytest.mark.parametrize("dims", DIMS, ids=lambda d: f"d{d[0]}_{d[1]}")
def test_backward_abs_of_sum_decay_unnarrowed(A, dims):
    """The |sum| normalizer with decay on the plain N(0, 1) inputs (no |q|, |k|): the row sums cancel (sum |s'| is
    some 50 x |sum s'|), so the operator amplifies every rounding of its inputs by that factor and gradients reach
    hundreds; an absolute bar means nothing here.  Relative bar instead, per tensor: the largest error at most 2 % of
    the largest |reference|, the mean error at most 2 % of the mean |reference| (bf16 weights carry 2^-9 relative
    rounding each; amplified by the cancellation of the row sum, percent-level agreement is what the arithmetic
    supports)."""
    w = Workload("retnet_abs_of_sum_raw", 40, 2, 4, 2, 300, 333, dims[0], dims[1], score_mod="head_decay", norm="abs_of_sum",
                 mask="causal", decay=True)
    print(f"case {w}", flush=True)
    Q, K, V = make_inputs(w)
    dO = make_grad(w)
    got, ref = hip_backward(A, w, Q, K, V, dO), oracle_backward(w, Q, K, V, dO)
    for name, g, r in zip(("dQ", "dK", "dV"), got, ref):
        assert np.isfinite(g).all()
        err = np.abs(g - r)
        print(f"{w.name} {name}: max err {err.max():.3e} of max |ref| {np.abs(r).max():.3e}; mean err {err.mean():.3e} of mean |ref| "
              f"{np.abs(r).mean():.3e}", flush=True)
        assert err.max() <= 2e-2 * np.abs(r).max() and err.mean() <= 2e-2 * np.abs(r).mean(), name


@pytest.mark.parametrize("Lq,Lk", [(1, 1), (1, 200), (200, 1), (31, 33), (64, 64), (128, 128), (129, 257), (500, 130),
                                    (130, 500), (257, 129)])
@pytest.mark.parametrize("mask", ["none", "causal"])
def test_backward_lengths(A, Lq, Lk, mask):
    # L_q != L_k in both directions (causal: bottom-right aligned; with L_q > L_k the first rows see no key and
    # must get zero gradient), single rows, exact tile multiples
    run_case(A, Workload(f"len{Lq}x{Lk}{mask}", 41, 1, 3, 1, Lq, Lk, 64, 64, mask=mask))
    run_case(A, Workload(f"len{Lq}x{Lk}{mask}sig", 42, 1, 2, 2, Lq, Lk, 128, 128, mask=mask, norm="sigmoid", score_mod="bias", bias=-2.0))
    run_case(A, Workload(f"len{Lq}x{Lk}{mask}relu", 45, 1, 2, 1, Lq, Lk, 64, 64, mask=mask, norm="none", score_mod="relu", scale=0.02))


@pytest.mark.parametrize("window", [1, 7, 64, 100, 333, 5000])
@pytest.mark.parametrize("Lq,Lk", [(300, 333), (333, 300), (700, 700)])
def test_backward_sliding_window(A, window, Lq, Lk):
    # windows shorter than a sub-tile, spanning a few tiles, and wider than the keys (= the causal mask); the walk
    # of either kernel starts and ends at the tiles the window allows
    run_case(A, Workload(f"win{window}_{Lq}x{Lk}", 47, 1, 4, 2, Lq, Lk, 128, 128, mask="sliding_window", window=window))
    run_case(A, Workload(f"win{window}_{Lq}x{Lk}sig", 48, 2, 2, 2, Lq, Lk, 64, 64, mask="sliding_window", window=window,
                         norm="sigmoid", score_mod="bias", bias=-1.0))


def test_backward_more_heads_than_the_decay_table(A):
    # handles without a per-head decay may have more query heads than the decay table holds (256): the kernels of
    # the linear normalizations must not read the table then
    run_case(A, Workload("heads260_none", 49, 1, 260, 130, 70, 90, 64, 64, norm="none", scale=0.01, mask="causal"))
    run_case(A, Workload("heads260_abssum", 50, 1, 260, 260, 40, 40, 64, 64, norm="abssum"))


def test_backward_bf16_forward_output(A):
    # delta is formed from the forward output as stored: also when that is bf16
    run_case(A, Workload("bf16_O", 43, 1, 4, 2, 260, 260, 128, 128, mask="causal"), out_dtype=torch.bfloat16)


def test_backward_strided_inputs(A):
    # Q, K, V as [B, L, H, D] memory viewed as [B, H, L, D]
    w = Workload("strided", 44, 2, 4, 2, 200, 230, 128, 128, mask="causal")
    Q, K, V = make_inputs(w)
    dO = make_grad(w)
    dev = torch.device("cuda:0")
    Qd, Kd, Vd = (x.to(dev).permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for x in (Q, K, V))
    stats = torch.empty((w.B, w.H_q, w.L_q), dtype=torch.float32, device=dev)
    O = A.run_workload(w, Qd, Kd, Vd, stats=stats)
    got = A.attention_backward(Qd, Kd, Vd, O, dO.to(dev), stats, scale=w.scale_value, mask=w.mask)
    torch.cuda.synchronize()
    ref = oracle_backward(w, Q, K, V, dO)
    for name, g, r in zip(("dQ", "dK", "dV"), got, ref):
        check(g.cpu().double().numpy(), r, f"strided {name}")


def test_backward_full_size_c2_one_group(A):
    """The benchmark shape (4 x 32/8 heads x 2048 x 128, causal softmax) at full size; the oracle checks one
    (batch, k/v head) group: its four query heads' dQ and the group's dK, dV."""
    w = C2
    Q, K, V = make_inputs(w)
    dO = make_grad(w)
    got = hip_backward(A, w, Q, K, V, dO)
    b, hk, g = 2, 5, w.H_q // w.H_kv
    hs = slice(hk * g, hk * g + g)
    ref = attention_backward(Q[b:b + 1, hs], K[b:b + 1, hk:hk + 1], V[b:b + 1, hk:hk + 1], dO[b:b + 1, hs],
                             scale=w.scale_value, norm="softmax", mask="causal")
    check(got[0][b:b + 1, hs], ref[0], "C2 dQ")
    check(got[1][b:b + 1, hk:hk + 1], ref[1], "C2 dK")
    check(got[2][b:b + 1, hk:hk + 1], ref[2], "C2 dV")


def test_backward_seeded_random_shapes(A):
    """40 seeded draws over shapes (ragged, L_q != L_k in both directions), head grouping, head dims,
    normalization / modification / mask, each against the backward oracle."""
    rng = np.random.default_rng(20250305)
    combos = [("softmax", "none"), ("softmax", "bias"), ("sigmoid", "bias"), ("none", "relu"), ("none", "none"),
              ("abssum", "none"), ("abssum", "head_decay"), ("none", "head_decay")]
    for case in range(40):
        dims = DIMS[int(rng.integers(len(DIMS)))]
        norm, mod = combos[int(rng.integers(len(combos)))]
        g = int(rng.choice([1, 2, 4]))
        H_kv = int(rng.integers(1, 3))
        Lq, Lk = int(rng.integers(1, 500)), int(rng.integers(1, 600))
        mask = "causal" if mod == "head_decay" else str(rng.choice(["none", "causal", "sliding_window"]))
        if mask == "sliding_window" and (mod == "relu" or norm == "abssum"):
            mask = "causal"
        w = Workload(f"rand{case}", 500 + case, int(rng.integers(1, 3)), g * H_kv, H_kv, Lq, Lk, dims[0], dims[1],
                     score_mod=mod, norm=norm, mask=mask, window=int(rng.integers(1, 400)) if mask == "sliding_window" else 0,
                     decay=(mod == "head_decay"), bias=float(rng.uniform(-2, 1)) if norm != "none" else 0.01,
                     scale=(0.01 if norm == "none" else None))
        run_case(A, w)


def test_backward_hip_graph_replays(A):
    """ae_attn_backward allocates nothing: its three launches are captured into a HIP graph and replayed four
    times with new dO values and eager work in between; every replay must equal the eager call bit for bit."""
    dev = torch.device("cuda:0")
    w = Workload("graph_bwd", 46, 1, 4, 2, 300, 420, 128, 128, mask="causal")
    Q, K, V = (x.to(dev) for x in make_inputs(w))
    dO0 = make_grad(w).to(dev)
    stats = torch.empty((w.B, w.H_q, w.L_q), dtype=torch.float32, device=dev)
    O = A.run_workload(w, Q, K, V, stats=stats)
    h = A.ae_attn_create(B=w.B, H_q=w.H_q, H_kv=w.H_kv, L_q=w.L_q, L_k=w.L_k, D_qk=w.D_qk, D_v=w.D_v,
                         scale=w.scale_value, mask=w.mask)
    ws = torch.empty(A.ae_attn_backward_workspace_bytes(h), dtype=torch.uint8, device=dev)
    ws_e = torch.empty_like(ws)
    dO = dO0.clone()
    outs_g = [torch.zeros(x.shape, dtype=torch.float32, device=dev) for x in (Q, K, V)]
    outs_e = [torch.zeros(x.shape, dtype=torch.float32, device=dev) for x in (Q, K, V)]

    def launch(outs, wsp, stream):
        A.ae_attn_backward(h, Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), dO.data_ptr(), stats.data_ptr(),
                           outs[0].data_ptr(), outs[1].data_ptr(), outs[2].data_ptr(), wsp.data_ptr(), wsp.numel(),
                           stream.cuda_stream)

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.graph(graph, stream=side):
        launch(outs_g, ws, side)
    torch.cuda.synchronize()
    for replay in range(4):
        if replay:
            dO.copy_((dO0.float() * (1.0 + 0.3 * replay)).to(torch.bfloat16).roll(replay, dims=2))
        for x in outs_g:
            x.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        launch(outs_e, ws_e, torch.cuda.current_stream())
        torch.cuda.synchronize()
        for name, a, b in zip(("dQ", "dK", "dV"), outs_g, outs_e):
            assert torch.equal(a, b), f"replay {replay}: {name} differs from the eager call"
    del graph
    A.ae_attn_destroy(h)


@pytest.mark.parametrize("dims", [(64, 64), (128, 128), (192, 128)], ids=lambda d: f"d{d[0]}_{d[1]}")
@pytest.mark.parametrize("norm", ["softmax", "sigmoid", "none"])
@pytest.mark.parametrize("mask", ["none", "causal"])
def test_backward_bias_tensor(A, dims, norm, mask):
    """dQ, dK, dV with an additive bias tensor (per batch and head / shared over the batch / over both) on a ragged,
    grouped shape; the bias rows are padded to a multiple of 8 on the device."""
    from paper_2502_15349_amd.workloads import make_bias_tensor
    dev = torch.device("cuda:0")
    w = Workload(f"bwd_bias_{norm}_{mask}", 63, 2, 4, 2, 300, 333, dims[0], dims[1], score_mod="bias_tensor", norm=norm,
                 mask=mask, scale=(0.01 if norm == "none" else None))
    Q, K, V = make_inputs(w)
    dO = make_grad(w)
    Qd, Kd, Vd, dOd = Q.to(dev), K.to(dev), V.to(dev), dO.to(dev)
    for per_batch, per_head in ((True, True), (False, True), (False, False)):
        bt = make_bias_tensor(w, per_batch, per_head)
        if norm == "none":
            bt = (bt.float() * 0.01).to(torch.bfloat16)
        print(f"case {w.name} dims {dims} bias shape {tuple(bt.shape)}", flush=True)
        btd = torch.zeros(bt.shape[:3] + (336,), dtype=torch.bfloat16, device=dev)
        btd[..., :w.L_k] = bt.to(dev)
        btv = btd[..., :w.L_k]
        stats = torch.empty((w.B, w.H_q, w.L_q), dtype=torch.float32, device=dev) if norm == "softmax" else None
        O = A.run_workload(w, Qd, Kd, Vd, stats=stats, bias_tensor=btv)
        got = A.attention_backward(Qd, Kd, Vd, O, dOd, stats, scale=w.scale_value, score_mod="bias_tensor", norm=norm,
                                   mask=mask, bias_tensor=btv, want_dbias=True)
        torch.cuda.synchronize()
        ref = attention_backward(Q, K, V, dO, scale=w.scale_value, score_mod="bias_tensor", norm=norm, mask=mask, bias_tensor=bt,
                                 with_dbias=True)
        for name, g, r in zip(("dQ", "dK", "dV"), got, ref):
            check(g.cpu().double().numpy(), r, f"{w.name} {tuple(bt.shape)} {name}")
        # The bias gradient is dS' itself, element by element, stored as bf16.  Where one weight dominates a row,
        # dS' = P (dP - delta) is a difference of nearly equal numbers of size |dO| |V| (~ 8 here), and delta comes
        # from the forward output as stored (bf16 weights in its sum): single elements are off by a few 1e-2 where
        # the sums that form dQ, dK, dV average such errors out.  Bar: max-abs 3e-2, mean-abs 1e-3, relative to
        # max(1, largest |reference| of the row).
        gB, rB = got[3].float().cpu().double().numpy(), ref[3]
        errB = np.abs(gB - rB) / np.maximum(np.abs(rB).max(axis=-1, keepdims=True), 1.0)
        print(f"{w.name} {tuple(bt.shape)} dBias: max_abs {errB.max():.3e} mean_abs {errB.mean():.3e}", flush=True)
        assert np.isfinite(gB).all() and errB.max() <= 3e-2 and errB.mean() <= MEAN_ABS

"""GPU parity: the HIP path (through the C ABI) against the fp64 CPU oracle on
the same seeded bf16 inputs.  Bar (bf16 inputs, fp32 accumulation): max-abs
<= 1e-2 and mean-abs <= 1e-3 over every compared element.
"""
import math

import numpy as np
import pytest
import torch

from oracle import attention, attention_head
from paper_2502_15349_amd.workloads import BY_ID, C1, C2, C3, C4, C5, Workload, make_inputs

pytestmark = pytest.mark.gpu

MAX_ABS, MEAN_ABS = 1e-2, 1e-3
# Bar of the softmax row statistic ln sum_j exp(x_ij).  The kernels take the scale on q, rounded to bf16 again (the
# paper's own form of the modification, Section 4.1: q_mod = q / sqrt(d_k)), so every exponent carries that
# rounding: relative 2^-9 uniform per element of q, i.e. a standard deviation of |scale| 2^-9 / sqrt(3) sqrt(sum_d
# q_d^2 k_d^2) = about 1.1e-3 per score for unit-variance inputs at scale 1/sqrt(D); the statistic is a weighted mean
# of such errors, held to 3.5 standard deviations.  (With the scale kept in fp32 on the scores -- the kernels used for
# |scale| sqrt(D) > 2 -- the error is that of fp32 sums of fp32 exponentials, below 1e-3.)
LSE_ABS = 4e-3
DIMS = [(64, 64), (128, 128), (128, 256), (192, 128)]


@pytest.fixture(scope="module")
def A():
    from paper_2502_15349_amd import ae_attn
    return ae_attn


def gpu_run(A, w, Q, K, V):
    dev = torch.device("cuda:0")
    O = A.run_workload(w, Q.to(dev), K.to(dev), V.to(dev))
    torch.cuda.synchronize()
    return O.cpu().double().numpy()


def oracle_run(w, Q, K, V):
    return attention(Q, K, V, scale=w.scale_value, score_mod=w.score_mod, bias=w.bias,
                     gamma=w.gamma(), norm=w.norm, mask=w.oracle_mask())


def check(got, ref, what=""):
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    err = np.abs(got - ref)
    print(f"{what}: max_abs {err.max():.3e} mean_abs {err.mean():.3e} |ref|max {np.abs(ref).max():.3e}", flush=True)
    assert err.max() <= MAX_ABS, f"{what}: max-abs {err.max():.3e}"
    assert err.mean() <= MEAN_ABS, f"{what}: mean-abs {err.mean():.3e}"


VARIANTS = {
    "softmax": dict(),
    "softmax_causal": dict(mask="causal"),
    "softmax_bias_causal": dict(score_mod="bias", bias=0.75, mask="causal"),
    "sigmoid_causal": dict(score_mod="bias", norm="sigmoid", mask="causal", bias=-math.log(300.0)),
    "sigmoid": dict(norm="sigmoid"),
    # |bias| * log2(e) > 64: the kernel keeps scale and bias in the exponent FMA
    # instead of folding the scale into Q
    "sigmoid_big_bias_causal": dict(score_mod="bias", norm="sigmoid", mask="causal", bias=-48.0, scale=6.0),
    "retnet_abssum": dict(score_mod="head_decay", norm="abssum", mask="causal", decay=True),
    "retnet_abs_of_sum": dict(score_mod="head_decay", norm="abs_of_sum", mask="causal", decay=True),
    "decay_nonorm": dict(score_mod="head_decay", norm="none", mask="causal", decay=True, scale=0.01),
    "abssum_plain": dict(norm="abssum"),
    "abs_of_sum_plain_causal": dict(norm="abs_of_sum", mask="causal"),
    "relu": dict(score_mod="relu", norm="none", scale=0.01),
    "relu_causal": dict(score_mod="relu", norm="none", mask="causal", scale=0.01),
    "none_plain": dict(norm="none", scale=0.005),
}


# Variants whose outputs are not O(1) by construction: no normalisation, the |sum| normaliser (its
# denominators cancel), sigmoid without the -ln L bias.  Only these are judged relative to the row
# scale max(1, max |oracle row|); every other variant is held to the absolute bar as it stands.
ROW_SCALED = {"sigmoid", "sigmoid_big_bias_causal", "retnet_abs_of_sum", "decay_nonorm", "abs_of_sum_plain_causal",
              "relu", "relu_causal", "none_plain"}


@pytest.mark.parametrize("dims", DIMS, ids=lambda d: f"d{d[0]}_{d[1]}")
@pytest.mark.parametrize("variant", sorted(VARIANTS))
def test_small_ragged_all_variants(A, dims, variant):
    # 2 query tiles with a ragged tail, 6 key tiles with a ragged tail, GQA 2:1
    kw = dict(VARIANTS[variant])
    w = Workload(f"{variant}", 11, 2, 4, 2, 300, 333, dims[0], dims[1], **kw)
    Q, K, V = make_inputs(w)
    print(f"case {variant} dims {dims}", flush=True)
    got, ref = gpu_run(A, w, Q, K, V), oracle_run(w, Q, K, V)
    if variant in ROW_SCALED:
        rs = np.maximum(np.abs(ref).max(axis=-1, keepdims=True), 1.0)
        got, ref = got / rs, ref / rs
    check(got, ref, f"{variant} {dims}")


@pytest.mark.parametrize("dv", [128, 512])
@pytest.mark.parametrize("variant", ["retnet_abssum", "retnet_abs_of_sum", "decay_nonorm"])
@pytest.mark.parametrize("Lq,Lk", [(300, 333), (1, 1), (513, 513), (700, 40)])
def test_retention_head_dims_256(A, dv, variant, Lq, Lk):
    """Table 2's "Retention Parallel" head dims, D_qk = 256 with D_v = 512 (four launches over 128 value columns
    each) and D_v = 128 (one): ragged shapes, more queries than keys, grouped heads."""
    kw = dict(VARIANTS[variant])
    w = Workload(variant, 21, 2, 4, 2, Lq, Lk, 256, dv, **kw)
    Q, K, V = make_inputs(w)
    print(f"case {variant} 256/{dv} Lq {Lq} Lk {Lk}", flush=True)
    got, ref = gpu_run(A, w, Q, K, V), oracle_run(w, Q, K, V)
    if variant in ROW_SCALED:
        rs = np.maximum(np.abs(ref).max(axis=-1, keepdims=True), 1.0)
        got, ref = got / rs, ref / rs
    check(got, ref, f"{variant} 256/{dv}")


@pytest.mark.parametrize("Lq,Lk", [(1, 1), (1, 77), (77, 1), (64, 64), (257, 255), (40, 700), (700, 40), (513, 513)])
@pytest.mark.parametrize("mask", ["none", "causal"])
def test_shapes_softmax(A, Lq, Lk, mask):
    w = Workload("shape", 12, 1, 2, 1, Lq, Lk, 128, 128, mask=mask)
    Q, K, V = make_inputs(w)
    print(f"case Lq {Lq} Lk {Lk} mask {mask}", flush=True)
    got, ref = gpu_run(A, w, Q, K, V), oracle_run(w, Q, K, V)
    check(got, ref, f"softmax Lq={Lq} Lk={Lk} {mask}")
    if mask == "causal" and Lq > Lk:
        assert (got[:, :, : Lq - Lk] == 0).all()   # rows with no visible key


@pytest.mark.parametrize("Lq,Lk", [(777, 1111), (1111, 777), (1024, 1024)])
@pytest.mark.parametrize("mask", ["none", "causal"])
def test_shapes_many_tiles_mla_dims(A, Lq, Lk, mask):
    # several query tiles and a long key loop with ragged ends, D_qk != D_v
    w = Workload("shape192", 16, 1, 2, 2, Lq, Lk, 192, 128, mask=mask)
    Q, K, V = make_inputs(w)
    print(f"case 192/128 Lq {Lq} Lk {Lk} mask {mask}", flush=True)
    check(gpu_run(A, w, Q, K, V), oracle_run(w, Q, K, V), f"192/128 Lq={Lq} Lk={Lk} {mask}")


@pytest.mark.parametrize("cid", [3, 4])
@pytest.mark.parametrize("Lq,Lk", [(1, 1), (130, 130), (100, 400), (400, 100)])
def test_shapes_sigmoid_retnet(A, cid, Lq, Lk):
    w = BY_ID[cid].scaled(B=1, H_q=3, H_kv=3, L_q=Lq, L_k=Lk)
    Q, K, V = make_inputs(w)
    print(f"case config {cid} Lq {Lq} Lk {Lk}", flush=True)
    check(gpu_run(A, w, Q, K, V), oracle_run(w, Q, K, V), f"c{cid} Lq={Lq} Lk={Lk}")


def test_c1_full_elementwise(A):
    Q, K, V = make_inputs(C1)
    check(gpu_run(A, C1, Q, K, V), oracle_run(C1, Q, K, V), f"C1")


def _full_config(A, w, every_row, n_rows=40, seed=0):
    """Full-size launch (the configuration the benchmark times) against the oracle on EVERY (batch, head):
    every query row where the oracle finishes in seconds (every_row), otherwise tile edges plus random rows
    of every head, recomputed over the whole key range."""
    Q, K, V = make_inputs(w)
    dev = torch.device("cuda:0")
    print(f"case full {w.name}", flush=True)
    O = A.run_workload(w, Q.to(dev), K.to(dev), V.to(dev))
    torch.cuda.synchronize()
    assert torch.isfinite(O).all()
    O = O.cpu()
    rng = np.random.default_rng(seed)
    g = w.H_q // w.H_kv
    gam = w.gamma()
    worst, total, count = 0.0, 0.0, 0
    for b in range(w.B):
        for h in range(w.H_q):
            rows = None
            if not every_row:
                # first/last rows, edges of the 32-row wave blocks and the 256-row tiles, random rows
                rows = np.unique(np.concatenate([
                    [0, 1, 31, 32, 63, 64, 255, 256, 257, w.L_q - 257, w.L_q - 256, w.L_q - 2, w.L_q - 1],
                    rng.integers(0, w.L_q, n_rows)])).astype(np.int64)
                rows = rows[(rows >= 0) & (rows < w.L_q)]
            ref = attention_head(Q[b, h], K[b, h // g], V[b, h // g], scale=w.scale_value, score_mod=w.score_mod,
                                 bias=w.bias, gamma_h=None if gam is None else gam[h], norm=w.norm, mask=w.oracle_mask(),
                                 rows=rows)
            got = O[b, h].double().numpy()
            err = np.abs((got if rows is None else got[rows]) - ref)
            assert err.max() <= MAX_ABS, (w.name, b, h, err.max())
            worst, total, count = max(worst, float(err.max())), total + float(err.sum()), count + err.size
        print(f"  batch {b}: {w.H_q} heads, max_abs so far {worst:.3e} mean_abs so far {total / count:.3e}", flush=True)
    assert total / count <= MEAN_ABS, (w.name, total / count)


@pytest.mark.parametrize("w", [C2, C4], ids=lambda w: w.name)
def test_full_config_every_head_every_row(A, w):
    _full_config(A, w, every_row=True)


@pytest.mark.parametrize("w", [C3, C5], ids=lambda w: w.name)
def test_full_config_every_head_sampled_rows(A, w):
    _full_config(A, w, every_row=False)


def test_table2_shapes_sampled(A):
    """The paper's microbenchmark shapes (Table 2) at batch 1, sequence 2k: one sampled head each,
    rows compared after scaling by max(1, max |oracle row|) (ReLU attention is not normalised)."""
    from paper_2502_15349_amd.workloads import table2_workloads
    dev = torch.device("cuda:0")
    for w in table2_workloads():
        if w.B != 1 or w.L_q != 2048:
            continue
        Q, K, V = make_inputs(w)
        print(f"case {w.name}", flush=True)
        O = A.run_workload(w, Q.to(dev), K.to(dev), V.to(dev))
        torch.cuda.synchronize()
        rng = np.random.default_rng(w.config_id)
        h = int(rng.integers(w.H_q))
        rows = np.unique(np.concatenate([[0, 255, 256, w.L_q - 1], rng.integers(0, w.L_q, 40)])).astype(np.int64)
        ref = attention_head(Q[0, h], K[0, h], V[0, h], scale=w.scale_value, score_mod=w.score_mod, bias=w.bias,
                             gamma_h=None if w.gamma() is None else w.gamma()[h], norm=w.norm, mask=w.oracle_mask(), rows=rows)
        got = O[0, h].cpu().double().numpy()[rows]
        e = np.abs(got - ref) / np.maximum(1.0, np.abs(ref).max(axis=1, keepdims=True))
        assert e.max() <= MAX_ABS and e.mean() <= MEAN_ABS, (w.name, e.max(), e.mean())


def test_full_size_properties_c2(A):
    """Properties that hold at any size, at C2's full shape and launch geometry."""
    w = C2
    dev = torch.device("cuda:0")
    Q, K, V = (t.to(dev) for t in make_inputs(w))
    # constant V rows reproduce V (weights sum to 1); bf16 P rounding is unbiased
    vrow = torch.linspace(-2, 2, w.D_v, device=dev).to(torch.bfloat16)
    Vc = vrow.expand(w.B, w.H_kv, w.L_k, w.D_v).contiguous()
    O = A.run_workload(w, Q, K, Vc)
    assert (O - vrow.float()).abs().max().item() <= 1e-2
    # Q = 0: causal prefix mean of V
    O0 = A.run_workload(w, torch.zeros_like(Q), K, V)
    g = w.H_q // w.H_kv
    pref = torch.cumsum(V.double(), dim=2) / torch.arange(1, w.L_k + 1, device=dev, dtype=torch.float64)[:, None]
    pref = pref.repeat_interleave(g, dim=1)
    err = (O0.double() - pref).abs()
    assert err.max().item() <= MAX_ABS and err.mean().item() <= MEAN_ABS


def test_determinism_bit_exact(A):
    w = C2.scaled(B=1, H_q=8, H_kv=2, L_q=1024, L_k=1024)
    dev = torch.device("cuda:0")
    Q, K, V = (t.to(dev) for t in make_inputs(w))
    a = A.run_workload(w, Q, K, V)
    b = A.run_workload(w, Q, K, V)
    assert torch.equal(a, b)


@pytest.mark.parametrize("dims", DIMS, ids=lambda d: f"d{d[0]}_{d[1]}")
def test_strided_inputs_and_output(A, dims):
    # rows padded to a wider pitch, heads interleaved: [B, L, H, D] storage viewed as [B, H, L, D];
    # 300 rows: a full 256-row query tile plus a ragged one, five key tiles
    w = Workload("strided", 13, 2, 4, 2, 300, 300, dims[0], dims[1], mask="causal")
    Q, K, V = make_inputs(w)
    dev = torch.device("cuda:0")

    def blhd(t):
        return t.to(dev).permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)

    out = torch.full((w.B, w.L_q, w.H_q, w.D_v + 4), 7.0, dtype=torch.float32, device=dev)
    ov = out[..., : w.D_v].permute(0, 2, 1, 3)
    A.run_workload(w, blhd(Q), blhd(K), blhd(V), out=ov)
    torch.cuda.synchronize()
    check(ov.cpu().double().numpy(), oracle_run(w, Q, K, V), "strided")
    assert (out[..., w.D_v:] == 7.0).all()   # padding untouched


@pytest.mark.parametrize("dims", DIMS, ids=lambda d: f"d{d[0]}_{d[1]}")
@pytest.mark.parametrize("norm,mod", [("softmax", "none"), ("abssum", "head_decay")])
def test_bf16_output(A, dims, norm, mod):
    """AE_OUT_BF16: the fp32 rows rounded to bf16 when stored.  Bound: the fp32 path's bound plus
    one bf16 rounding of the result (half an ulp = 2^-9 relative; 2^-8 allowed)."""
    w = Workload("bf16out", 15, 2, 4, 2, 300, 333, dims[0], dims[1], mask="causal", norm=norm, score_mod=mod,
                 decay=(mod == "head_decay"))
    Q, K, V = make_inputs(w)
    dev = torch.device("cuda:0")
    O = A.run_workload(w, Q.to(dev), K.to(dev), V.to(dev), out_dtype=torch.bfloat16)
    torch.cuda.synchronize()
    assert O.dtype == torch.bfloat16
    got = O.float().cpu().double().numpy()
    ref = oracle_run(w, Q, K, V)
    err = np.abs(got - ref)
    assert (err <= MAX_ABS + np.abs(ref) * 2.0 ** -8).all(), err.max()
    assert err.mean() <= MEAN_ABS + np.abs(ref).mean() * 2.0 ** -8
    # and it is exactly the fp32 result rounded to nearest even
    O32 = A.run_workload(w, Q.to(dev), K.to(dev), V.to(dev))
    assert torch.equal(O32.to(torch.bfloat16), O)


@pytest.mark.parametrize("dims", DIMS, ids=lambda d: f"d{d[0]}_{d[1]}")
@pytest.mark.parametrize("norm,mod,mask", [("softmax", "none", "causal"), ("softmax", "bias", "none"),
                                           ("abssum", "head_decay", "causal"), ("abs_of_sum", "none", "causal")])
def test_row_statistics(A, dims, norm, mod, mask):
    """ae_attn_forward_stats: the row statistic against the oracle's (LSE_ABS absolute on ln-sum-exp, see above;
    1e-4 relative on the abs sums: fp32 sums of fp32 terms), and O unchanged by asking for it."""
    from oracle import row_stats_head
    w = Workload("stats", 16, 2, 4, 2, 300, 333 if mask == "causal" else 280, dims[0], dims[1], mask=mask, norm=norm,
                 score_mod=mod, bias=0.75, decay=(mod == "head_decay"))
    Q, K, V = make_inputs(w)
    dev = torch.device("cuda:0")
    st = torch.full((w.B, w.H_q, w.L_q), 123.0, dtype=torch.float32, device=dev)
    O = A.run_workload(w, Q.to(dev), K.to(dev), V.to(dev), stats=st)
    O0 = A.run_workload(w, Q.to(dev), K.to(dev), V.to(dev))
    torch.cuda.synchronize()
    assert torch.equal(O, O0)
    got = st.cpu().double().numpy()
    g = w.H_q // w.H_kv
    gam = w.gamma()
    for b in range(w.B):
        for h in range(w.H_q):
            ref = row_stats_head(Q[b, h], K[b, h // g], scale=w.scale_value, score_mod=w.score_mod, bias=w.bias,
                                 gamma_h=None if gam is None else gam[h], norm=w.norm, mask=w.oracle_mask())
            if norm == "softmax":
                assert np.abs(got[b, h] - ref).max() <= LSE_ABS, (b, h, np.abs(got[b, h] - ref).max())
            else:
                assert np.allclose(got[b, h], ref, rtol=1e-4, atol=1e-4), (b, h)


def test_row_statistics_rows_without_keys(A):
    from oracle import row_stats_head
    w = Workload("stats0", 17, 1, 2, 2, 100, 37, 64, 64, mask="causal")   # rows 0..62 see no key
    Q, K, V = make_inputs(w)
    dev = torch.device("cuda:0")
    st = torch.zeros((w.B, w.H_q, w.L_q), dtype=torch.float32, device=dev)
    O = A.run_workload(w, Q.to(dev), K.to(dev), V.to(dev), stats=st)
    torch.cuda.synchronize()
    got = st.cpu().double().numpy()
    for h in range(w.H_q):
        ref = row_stats_head(Q[0, h], K[0, h], scale=w.scale_value, norm="softmax", mask="causal")
        assert (np.isneginf(got[0, h]) == np.isneginf(ref)).all()
        fin = np.isfinite(ref)
        assert np.abs(got[0, h][fin] - ref[fin]).max() <= LSE_ABS
    assert (O[:, :, :63] == 0).all()


@pytest.mark.parametrize("dims", DIMS, ids=lambda d: f"d{d[0]}_{d[1]}")
@pytest.mark.parametrize("norm,mod", [("softmax", "none"), ("sigmoid", "bias"), ("none", "none")])
@pytest.mark.parametrize("Lq,Lk,W", [(300, 333, 100), (700, 700, 64), (513, 600, 1), (40, 300, 129), (300, 300, 5000),
                                     (200, 90, 33)])
def test_sliding_window(A, dims, norm, mod, Lq, Lk, W):
    """AE_MASK_SLIDING_WINDOW: the W keys nearest the causal diagonal; windows shorter than a
    sub-tile, longer than the sequence, ragged sizes, L_q != L_k (rows without keys included)."""
    w = Workload("window", 18, 1, 4, 2, Lq, Lk, dims[0], dims[1], mask="sliding_window", window=W, norm=norm,
                 score_mod=mod, bias=-1.0, scale=0.005 if norm == "none" else None)
    Q, K, V = make_inputs(w)
    got, ref = gpu_run(A, w, Q, K, V), oracle_run(w, Q, K, V)
    if norm != "softmax":   # no normalisation, sigmoid with a bias of -1: not O(1) by construction, judged relative to the row scale
        rs = np.maximum(np.abs(ref).max(axis=-1, keepdims=True), 1.0)
        got, ref = got / rs, ref / rs
    check(got, ref, f"window {W}")


def test_sliding_window_full_size_sampled(A):
    w = C2.scaled(name="c2_window_512", mask="sliding_window", window=512)
    _full_config(A, w, every_row=False)


def test_sliding_window_wider_than_everything(A):
    """A window of 2^31 - 1 keys with more queries than keys is the causal mask (rows without keys stay zero)."""
    w = Workload("window_max", 18, 1, 4, 2, 700, 300, 128, 128, mask="sliding_window", window=2**31 - 1)
    Q, K, V = make_inputs(w)
    got = gpu_run(A, w, Q, K, V)
    check(got, oracle_run(w.scaled(mask="causal"), Q, K, V), "window 2^31-1")
    assert (got[:, :, :400] == 0).all()


@pytest.mark.parametrize("dims", DIMS, ids=lambda d: f"d{d[0]}_{d[1]}")
@pytest.mark.parametrize("Lq,Lk,mask,splits", [(1, 2048, "none", 8), (1, 4000, "causal", 32), (5, 1000, "causal", 3),
                                               (1, 100, "none", 4), (300, 700, "causal", 5), (7, 64, "none", 2)])
def test_split_keys(A, dims, Lq, Lk, mask, splits):
    """kv_splits > 1 (decoding shapes and a few others): partial results per key range plus the
    merge kernel against the oracle; the row statistic too; GQA 4:1."""
    from oracle import row_stats_head
    w = Workload("split", 19, 2, 8, 2, Lq, Lk, dims[0], dims[1], mask=mask)
    Q, K, V = make_inputs(w)
    dev = torch.device("cuda:0")
    st = torch.zeros((w.B, w.H_q, w.L_q), dtype=torch.float32, device=dev)
    O = A.run_workload(w, Q.to(dev), K.to(dev), V.to(dev), stats=st, kv_splits=splits)
    torch.cuda.synchronize()
    check(O.cpu().double().numpy(), oracle_run(w, Q, K, V), f"split {splits}")
    got = st.cpu().double().numpy()
    for b in range(w.B):
        for h in range(w.H_q):
            ref = row_stats_head(Q[b, h], K[b, h // 4], scale=w.scale_value, norm="softmax", mask=w.oracle_mask())
            assert np.abs(got[b, h] - ref).max() <= LSE_ABS
    # bf16 output through the merge kernel: the fp32 merge result rounded
    Ob = A.run_workload(w, Q.to(dev), K.to(dev), V.to(dev), kv_splits=splits, out_dtype=torch.bfloat16)
    assert torch.equal(Ob, O.to(torch.bfloat16))


@pytest.mark.parametrize("dims", [(64, 64), (128, 128), (192, 128)], ids=lambda d: f"d{d[0]}_{d[1]}")
@pytest.mark.parametrize("Lk,splits", [(65, 2), (130, 3), (131, 2), (1000, 7), (1027, 16), (4099, 5)])
def test_decoding_rows(A, dims, Lk, splits):
    """One query row per head with split keys (the streaming kernel): key counts that leave the last range, the last
    wavefront and the last group of four keys ragged (a range of 2 or 3 keys among them); 8 q heads per k/v head; a
    constant bias; a negative scale; the row statistic; bf16 output."""
    from oracle import row_stats_head
    dev = torch.device("cuda:0")
    for kw in (dict(), dict(score_mod="bias", bias=-3.0), dict(scale=-0.05)):
        w = Workload("decode_rows", 21, 2, 8, 1, 1, Lk, dims[0], dims[1], mask="causal", **kw)
        Q, K, V = make_inputs(w)
        st = torch.zeros((w.B, w.H_q, 1), dtype=torch.float32, device=dev)
        O = A.run_workload(w, Q.to(dev), K.to(dev), V.to(dev), stats=st, kv_splits=splits)
        torch.cuda.synchronize()
        check(O.cpu().double().numpy(), oracle_run(w, Q, K, V), f"decoding rows {dims} L_k {Lk} {kw}")
        got = st.cpu().double().numpy()
        for b in range(w.B):
            for h in range(w.H_q):
                ref = row_stats_head(Q[b, h], K[b, 0], scale=w.scale_value, score_mod=w.score_mod, bias=w.bias, norm="softmax",
                                     mask=w.oracle_mask())
                assert np.abs(got[b, h] - ref).max() <= 1e-3, (b, h)      # (the scale stays in fp32 on this path)
        Ob = A.run_workload(w, Q.to(dev), K.to(dev), V.to(dev), kv_splits=splits, out_dtype=torch.bfloat16)
        assert torch.equal(Ob, O.to(torch.bfloat16))


def test_split_keys_decode_full_size(A):
    """The paper's decoding row (Table 2: one query row, 16 heads, 192/128) at 8k keys, batch 8."""
    w = Workload("decode", 20, 8, 16, 16, 1, 8192, 192, 128, mask="causal")
    Q, K, V = make_inputs(w)
    dev = torch.device("cuda:0")
    ref = oracle_run(w, Q, K, V)
    for splits in (16, -1):   # -1: the library picks the number of key ranges
        O = A.run_workload(w, Q.to(dev), K.to(dev), V.to(dev), kv_splits=splits)
        torch.cuda.synchronize()
        check(O.cpu().double().numpy(), ref, f"decode, kv_splits {splits}")


def test_hip_graph_replays(A):
    """The entry points allocate nothing and clear nothing, so their launches can be captured into a HIP
    graph.  Each graph (plain, with row statistics, split keys) is replayed four times with new Q values
    and eager work between the replays; every replay must equal the eager launch on the same inputs bit
    for bit, and the first one is also held against the oracle."""
    dev = torch.device("cuda:0")
    w = Workload("graph", 31, 2, 4, 2, 300, 1333, 128, 128, mask="causal")
    Qc, Kc, Vc = make_inputs(w)
    Q, K, V = Qc.to(dev), Kc.to(dev), Vc.to(dev)
    ref = oracle_run(w, Qc, Kc, Vc)
    side = torch.cuda.Stream()
    for name, splits, with_stats in (("plain", 0, False), ("stats", 0, True), ("split", 4, True)):
        print(f"graph case {name}", flush=True)
        h = A.ae_attn_create(B=w.B, H_q=w.H_q, H_kv=w.H_kv, L_q=w.L_q, L_k=w.L_k, D_qk=w.D_qk, D_v=w.D_v,
                             scale=w.scale_value, mask=w.mask, kv_splits=splits)
        ws = torch.empty(max(A.ae_attn_workspace_bytes(h), 16), dtype=torch.uint8, device=dev)
        Qg = Q.clone()
        Og, Oe = (torch.zeros((w.B, w.H_q, w.L_q, w.D_v), dtype=torch.float32, device=dev) for _ in range(2))
        Sg, Se = (torch.zeros((w.B, w.H_q, w.L_q), dtype=torch.float32, device=dev) for _ in range(2))

        def launch(O, S, stream):
            sp = S.data_ptr() if with_stats else 0
            if splits:
                A.ae_attn_forward_split(h, Qg.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), sp,
                                        ws.data_ptr(), ws.numel(), stream.cuda_stream)
            elif with_stats:
                A.ae_attn_forward_stats(h, Qg.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), sp, stream.cuda_stream)
            else:
                A.ae_attn_forward(h, Qg.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(), stream.cuda_stream)

        graph = torch.cuda.CUDAGraph()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.graph(graph, stream=side):
            launch(Og, Sg, side)
        torch.cuda.synchronize()
        for replay in range(4):
            if replay:
                Qg.copy_((Q.float() * (1.0 - 0.2 * replay)).to(torch.bfloat16).roll(replay, dims=2))
            Og.zero_()
            Sg.zero_()
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            launch(Oe, Se, torch.cuda.current_stream())
            torch.cuda.synchronize()
            assert torch.equal(Og, Oe), f"{name}: replay {replay} differs from the eager launch"
            if with_stats:
                assert torch.equal(Sg, Se), f"{name}: replay {replay} statistics differ from the eager launch"
            if replay == 0:
                check(Og.cpu().double().numpy(), ref, f"graph {name}")
        del graph
        A.ae_attn_destroy(h)


def test_seeded_random_shapes(A):
    """48 seeded draws over shapes (ragged, L_q != L_k in both directions), head grouping, head dims,
    (norm, mod, mask) combinations, window sizes and split counts, each against the oracle."""
    rng = np.random.default_rng(20250222)
    combos = [("softmax", "none"), ("softmax", "bias"), ("sigmoid", "bias"), ("abssum", "none"), ("abssum", "head_decay"),
              ("abs_of_sum", "head_decay"), ("none", "relu"), ("none", "none")]
    dev = torch.device("cuda:0")
    for case in range(48):
        dims = DIMS[int(rng.integers(len(DIMS)))]
        norm, mod = combos[int(rng.integers(len(combos)))]
        g = int(rng.choice([1, 2, 4]))
        H_kv = int(rng.integers(1, 3))
        Lq, Lk = int(rng.integers(1, 600)), int(rng.integers(1, 700))
        mask = "causal" if mod == "head_decay" else str(rng.choice(["none", "causal", "sliding_window"]))
        if mask == "sliding_window" and norm not in ("softmax", "sigmoid", "none"):
            mask = "causal"
        if mask == "sliding_window" and mod == "relu":
            mask = "none"
        window = int(rng.integers(1, 400)) if mask == "sliding_window" else 0
        splits = int(rng.integers(2, 9)) if (norm == "softmax" and mask != "sliding_window" and rng.random() < 0.5) else 0
        w = Workload(f"rand{case}", 300 + case, int(rng.integers(1, 3)), g * H_kv, H_kv, Lq, Lk, dims[0], dims[1],
                     score_mod=mod, norm=norm, mask=mask, window=window, bias=float(rng.uniform(-2, 1)),
                     decay=(mod == "head_decay"), scale=(0.01 if norm == "none" else None))
        print(f"case {case}: {w} splits {splits}", flush=True)
        Q, K, V = make_inputs(w)
        O = A.run_workload(w, Q.to(dev), K.to(dev), V.to(dev), kv_splits=splits)
        torch.cuda.synchronize()
        got, ref = O.cpu().double().numpy(), oracle_run(w, Q, K, V)
        if norm in ("none", "abs_of_sum", "sigmoid"):   # not O(1) by construction (the sigmoid bias here is not -ln L)
            rs = np.maximum(np.abs(ref).max(axis=-1, keepdims=True), 1.0)
            got, ref = got / rs, ref / rs
        check(got, ref, f"random case {case}")


def test_negative_scale_and_large_scores(A):
    w = Workload("neg", 14, 1, 2, 2, 150, 150, 64, 64, mask="causal", scale=-0.125)
    Q, K, V = make_inputs(w)
    check(gpu_run(A, w, Q, K, V), oracle_run(w, Q, K, V), "negative scale")
    w2 = Workload("big", 15, 1, 2, 2, 150, 150, 64, 64, scale=40.0)   # scores ~ +-1e3: no overflow
    Q, K, V = make_inputs(w2)
    check(gpu_run(A, w2, Q, K, V), oracle_run(w2, Q, K, V), "large scores")


def test_online_equals_two_pass_across_key_tilings(A):
    # the same keys presented with different tile phase (prefix padding via L_k) must agree
    w = Workload("phase", 16, 1, 1, 1, 96, 1000, 128, 128)
    Q, K, V = make_inputs(w)
    full = gpu_run(A, w, Q, K, V)
    perm = torch.randperm(1000, generator=torch.Generator().manual_seed(5))
    shuf = gpu_run(A, w, Q, K[:, :, perm].contiguous(), V[:, :, perm].contiguous())
    assert np.abs(full - shuf).max() <= 2e-3   # same math, different blocking of the online update


def test_calibration_kernel_runs(A):
    # measurement aid: launches, reports its flop count, writes its sink
    dev = torch.device("cuda:0")
    sink = torch.full((4 * 512,), float("nan"), dtype=torch.float32, device=dev)
    flop = A.ae_calib_mfma_bf16(sink.data_ptr(), sink.numel() * 4, 4, 10, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert flop == 4 * 8 * 10 * 16 * 32768.0
    assert torch.isfinite(sink).all()


def test_decay_rates_outside_the_factorised_range(A):
    # gamma < 1/16 and gamma > 1 take the per-score exponential, the others the
    # per-sub-tile factorisation; both against the oracle
    from oracle.attention_oracle import attention as oracle_attention
    B, H, L, D = 1, 4, 90, 128
    gam = [0.01, 0.5, 1.25, 1.0]
    g = torch.Generator("cpu").manual_seed(4242)
    Q, K, V = (torch.randn(B, H, L, d, generator=g).to(torch.bfloat16) for d in (D, D, 256))
    dev = torch.device("cuda:0")
    for norm in ("abssum", "none"):
        scale = 0.09 if norm == "abssum" else 1e-4
        O = A.attention_forward(Q.to(dev), K.to(dev), V.to(dev), scale=scale, score_mod="head_decay", gamma=gam,
                                norm=norm, mask="causal")
        torch.cuda.synchronize()
        ref = oracle_attention(Q, K, V, scale=scale, score_mod="head_decay", gamma=gam, norm=norm, mask="causal")
        # Judged relative to the row scale for both norms: with gamma = 0.01 a row's weight sits on one key, so O_i is
        # v_i itself (|v| up to 4.1 here) and the half-ulp of that one bf16 weight, 2^-9 |v_i| = 8e-3, is most of the
        # absolute bar on its own -- the row is not a mean over many keys as in the benchmark configurations.
        rs = np.maximum(np.abs(ref).max(axis=-1, keepdims=True), 1.0)
        check(O.cpu().double().numpy() / rs, ref / rs, f"decay gammas {gam} norm {norm}")


@pytest.mark.parametrize("dims", [(64, 64), (128, 128), (192, 128)], ids=lambda d: f"d{d[0]}_{d[1]}")
@pytest.mark.parametrize("norm", ["softmax", "sigmoid", "none"])
@pytest.mark.parametrize("mask", ["none", "causal"])
def test_bias_tensor(A, dims, norm, mask):
    """score_mod "bias_tensor": an additive bf16 bias per (query, key) pair, per batch and head, shared over the
    batch, or over batch and heads; ragged sizes (L_k = 333 is no multiple of 4: the row ends are read element by
    element), grouped heads; softmax also returns the row statistic."""
    from oracle import row_stats_head
    from paper_2502_15349_amd.workloads import make_bias_tensor
    dev = torch.device("cuda:0")
    w = Workload(f"bias_t_{norm}_{mask}", 60, 2, 4, 2, 300, 333, dims[0], dims[1], score_mod="bias_tensor", norm=norm, mask=mask,
                 scale=(0.01 if norm == "none" else None))
    Q, K, V = make_inputs(w)
    for per_batch, per_head in ((True, True), (False, True), (False, False)):
        bt = make_bias_tensor(w, per_batch, per_head)
        if norm == "none":
            bt = (bt.float() * 0.01).to(torch.bfloat16)
        print(f"case {w.name} dims {dims} bias shape {tuple(bt.shape)}", flush=True)
        stats = torch.empty((w.B, w.H_q, w.L_q), dtype=torch.float32, device=dev) if norm == "softmax" else None
        # rows of the device copy start at multiples of 8 elements (the row stride the library asks for)
        btd = torch.zeros(bt.shape[:3] + (336,), dtype=torch.bfloat16, device=dev)
        btd[..., :w.L_k] = bt.to(dev)
        O = A.run_workload(w, Q.to(dev), K.to(dev), V.to(dev), stats=stats, bias_tensor=btd[..., :w.L_k])
        torch.cuda.synchronize()
        ref = attention(Q, K, V, scale=w.scale_value, score_mod="bias_tensor", norm=norm, mask=mask, bias_tensor=bt)
        # (sigmoid and no normalization: outputs are not O(1); judged relative to the row scale as elsewhere)
        rs = np.maximum(np.abs(ref).max(axis=-1, keepdims=True), 1.0) if norm != "softmax" else 1.0
        check(O.cpu().double().numpy() / rs, ref / rs, f"bias tensor {norm} {mask} {tuple(bt.shape)}")
        if stats is not None:
            b, h = 1, 3
            want = row_stats_head(Q[b, h], K[b, h // 2], scale=w.scale_value, score_mod="bias_tensor", mask=mask,
                                  bias_t=bt[b if per_batch else 0, h if per_head else 0])
            np.testing.assert_allclose(stats[b, h].cpu().double().numpy(), want, atol=2e-3)


def test_bias_tensor_alibi_and_padded_rows(A):
    """A structured bias (ALiBi: -slope_h * distance) on a longer causal problem, stored with padded rows."""
    dev = torch.device("cuda:0")
    w = Workload("alibi", 61, 1, 4, 4, 1000, 1000, 128, 128, score_mod="bias_tensor", mask="causal")
    Q, K, V = make_inputs(w)
    dist = (torch.arange(w.L_q)[:, None] - torch.arange(w.L_k)[None, :]).clamp(min=0).float()
    slopes = torch.tensor([2.0 ** (-2 * (h + 1)) for h in range(w.H_q)])
    bt = (-slopes[None, :, None, None] * dist[None, None]).to(torch.bfloat16)
    padded = torch.zeros((1, w.H_q, w.L_q, 1024), dtype=torch.bfloat16, device=dev)
    padded[..., :w.L_k] = bt.to(dev)
    O = A.run_workload(w, Q.to(dev), K.to(dev), V.to(dev), bias_tensor=padded[..., :w.L_k])
    torch.cuda.synchronize()
    ref = attention(Q, K, V, scale=w.scale_value, score_mod="bias_tensor", mask="causal", bias_tensor=bt)
    check(O.cpu().double().numpy(), ref, "alibi")


@pytest.mark.parametrize("Lq,Lk", [(1, 8), (5, 16), (40, 24), (64, 64), (100, 72), (257, 136), (33, 520)])
@pytest.mark.parametrize("mask", ["none", "causal"])
def test_bias_tensor_small_and_uneven_lengths(A, Lq, Lk, mask):
    """Bias tensor on problems of one sub-tile, one tile, a few tiles; L_q != L_k in both directions."""
    from paper_2502_15349_amd.workloads import make_bias_tensor
    dev = torch.device("cuda:0")
    w = Workload(f"bias_small_{Lq}x{Lk}_{mask}", 62, 2, 2, 1, Lq, Lk, 128, 128, score_mod="bias_tensor", mask=mask)
    Q, K, V = make_inputs(w)
    bt = make_bias_tensor(w)
    O = A.run_workload(w, Q.to(dev), K.to(dev), V.to(dev), bias_tensor=bt.to(dev))
    torch.cuda.synchronize()
    ref = attention(Q, K, V, scale=w.scale_value, score_mod="bias_tensor", mask=mask, bias_tensor=bt)
    check(O.cpu().double().numpy(), ref, f"bias tensor {Lq}x{Lk} {mask}")

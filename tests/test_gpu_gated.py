"""GPU parity of the recurrent pattern with per-token gates (ae_gated_forward, through the C ABI) against the fp64
token-by-token oracle on the same seeded inputs.  Bar as for the parallel pattern (bf16 operands, bf16 weights and
state into the MFMAs, fp32 accumulation): max-abs <= 1e-2 and mean-abs <= 1e-3 relative to max(1, the largest
|reference| of the row) -- the outputs are sums that grow with the number of tokens the decay lets through, they are
not normalised."""
import math

import numpy as np
import pytest
import torch

from oracle.gated_recurrent_oracle import gated_recurrent as oracle_gated
from paper_2502_15349_amd.workloads import Workload, make_gates, make_inputs

pytestmark = pytest.mark.gpu
MAX_ABS, MEAN_ABS = 1e-2, 1e-3


@pytest.fixture(scope="module")
def A():
    from paper_2502_15349_amd import ae_attn
    return ae_attn


def check(got, ref, what):
    assert np.isfinite(got).all(), what
    rs = np.maximum(np.abs(ref).max(axis=-1, keepdims=True), 1.0)
    err = np.abs(got - ref) / rs
    print(f"{what}: max_abs {err.max():.3e} mean_abs {err.mean():.3e} |ref|max {np.abs(ref).max():.3e}", flush=True)
    assert err.max() <= MAX_ABS and err.mean() <= MEAN_ABS, (what, err.max(), err.mean())


def inputs(cid, B, H, H_qk, L, dqk, dv, kind):
    wq = Workload("gq", cid, B, H_qk, H_qk, L, L, dqk, dqk)
    wv = Workload("gv", cid, B, H, H, L, L, dv, dv)
    Q, K, _ = make_inputs(wq)
    _, _, V = make_inputs(wv)
    la, kg = make_gates(B, H, L, 1000 * cid + 5, kind)
    return Q, K, V, la, kg


def run(A, Q, K, V, la, kg, scale, h_in=None, want_state=False, segmented=False):
    dev = torch.device("cuda:0")
    r = A.gated_recurrent(Q.to(dev), K.to(dev), V.to(dev), la.to(dev), None if kg is None else kg.to(dev), scale=scale,
                          h_in=None if h_in is None else h_in.to(dev), want_state=want_state, segmented=segmented)
    torch.cuda.synchronize()
    return r


@pytest.mark.parametrize("dqk,dv", [(64, 64), (128, 64), (64, 128), (128, 128)])
@pytest.mark.parametrize("kind", ["gated_retention", "mamba2"])
@pytest.mark.parametrize("L", [1, 63, 64, 65, 200, 513])
def test_matches_oracle(A, dqk, dv, kind, L):
    # one token, a ragged single chunk, exact chunk, several chunks with a short last one
    Q, K, V, la, kg = inputs(800 + L % 7, 2, 3, 3, L, dqk, dv, kind)
    scale = 1.0 / math.sqrt(dqk)
    print(f"case {kind} {dqk}/{dv} L {L}", flush=True)
    got = run(A, Q, K, V, la, kg, scale)
    ref = oracle_gated(Q.float().numpy(), K.float().numpy(), V.float().numpy(), la.numpy(), None if kg is None else kg.numpy(), scale=scale)
    check(got.cpu().double().numpy(), ref, f"{kind} {dqk}/{dv} L={L}")


def test_grouped_query_key_heads_mamba2_shape(A):
    # Mamba2's structure at a reduced head count: B and C shared by the value heads of a group, D_qk 128, D_v 64
    Q, K, V, la, kg = inputs(810, 1, 8, 2, 300, 128, 64, "mamba2")
    got = run(A, Q, K, V, la, kg, 1.0)
    ref = oracle_gated(Q.float().numpy(), K.float().numpy(), V.float().numpy(), la.numpy(), kg.numpy(), scale=1.0)
    check(got.cpu().double().numpy(), ref, "mamba2 groups")


def test_constant_decay_is_retention(A):
    # log_decay = ln gamma per head: the retention recurrence of the constant-decay path (same oracle family)
    from oracle.retention_recurrent_oracle import retention_recurrent
    w = Workload("ret", 811, 1, 4, 4, 400, 400, 128, 128)
    Q, K, V = make_inputs(w)
    gam = [1.0, 0.96875, 0.5, 0.984375]
    la = torch.log(torch.tensor(gam, dtype=torch.float32)).view(1, 4, 1).expand(1, 4, 400).contiguous()
    got = run(A, Q, K, V, la, None, w.scale_value)
    ref = retention_recurrent(Q.float().numpy(), K.float().numpy(), V.float().numpy(), scale=w.scale_value, gamma=gam)
    check(got.cpu().double().numpy(), ref, "constant decay")


def test_sequence_in_pieces_with_carried_state(A):
    Q, K, V, la, kg = inputs(812, 1, 2, 2, 330, 128, 128, "mamba2")
    scale = 0.1
    ref, ref_h = oracle_gated(Q.float().numpy(), K.float().numpy(), V.float().numpy(), la.numpy(), kg.numpy(), scale=scale, return_state=True)
    outs, h = [], None
    for a, b in ((0, 100), (100, 101), (101, 330)):
        o, h = run(A, Q[:, :, a:b].contiguous(), K[:, :, a:b].contiguous(), V[:, :, a:b].contiguous(), la[:, :, a:b].contiguous(),
                   kg[:, :, a:b].contiguous(), scale, h_in=h, want_state=True)
        outs.append(o.cpu())
    check(torch.cat(outs, dim=2).double().numpy(), ref, "pieces: outputs")
    hs = np.maximum(np.abs(ref_h).max(axis=-1, keepdims=True), 1.0)
    assert (np.abs(h.cpu().double().numpy() - ref_h) / hs).max() <= MAX_ABS


def test_strong_decay_and_no_decay(A):
    # a_t down to e^-8 per token (the chunk's cumulative exponents reach -500: weights underflow to zero, nothing
    # overflows), a_t = 1 throughout (a plain prefix sum: outputs grow with the position), and a slow decay broken by
    # single tokens of e^-30 (beyond the -20 at which the kernel clamps a token's log-decay inside a chunk: what came
    # before such a token is gone to fp32 resolution either way)
    w = Workload("dec", 813, 1, 3, 3, 260, 260, 64, 64)
    Q, K, V = make_inputs(w)
    la = torch.full((1, 3, 260), -8.0)
    la[:, 1] = 0.0
    la[:, 2] = -0.01
    la[:, 2, 5::37] = -30.0
    got = run(A, Q, K, V, la, None, 0.125)
    ref = oracle_gated(Q.float().numpy(), K.float().numpy(), V.float().numpy(), la.numpy(), None, scale=0.125)
    check(got.cpu().double().numpy(), ref, "decay e^-8 / none / resets")


@pytest.mark.parametrize("dqk,dv,H,H_qk", [(128, 128, 2, 2), (64, 64, 3, 3), (128, 64, 4, 1), (64, 128, 2, 2)])
@pytest.mark.parametrize("kind", ["gated_retention", "mamba2"])
@pytest.mark.parametrize("L", [1061, 2560])
def test_segmented_walk(A, dqk, dv, H, H_qk, kind, L):
    # few heads, a long sequence: ae_gated_forward_segmented cuts the walks into segments (2 and 5 here; a ragged
    # last one), with a state handed in and the final state handed back; against the oracle's single walk
    Q, K, V, la, kg = inputs(820 + L % 5, 1, H, H_qk, L, dqk, dv, kind)
    g = torch.Generator().manual_seed(77)
    h0 = torch.randn((1, H, dqk, dv), generator=g, dtype=torch.float32)
    scale = 1.0 / math.sqrt(dqk)
    dev = torch.device("cuda:0")
    h = A.ae_gated_create(B=1, H=H, H_qk=H_qk, L=L, D_qk=dqk, D_v=dv, scale=scale)
    assert A.ae_gated_workspace_bytes(h) > 0          # this shape is cut
    A.ae_gated_destroy(h)
    o, hN = run(A, Q, K, V, la, kg, scale, h_in=h0, want_state=True, segmented=True)
    ref, ref_h = oracle_gated(Q.float().numpy(), K.float().numpy(), V.float().numpy(), la.numpy(), None if kg is None else kg.numpy(),
                              scale=scale, h0=h0.double().numpy(), return_state=True)
    check(o.cpu().double().numpy(), ref, f"segmented {kind} {dqk}/{dv} L={L}")
    hs = np.maximum(np.abs(ref_h).max(axis=-1, keepdims=True), 1.0)
    assert (np.abs(hN.cpu().double().numpy() - ref_h) / hs).max() <= MAX_ABS


def test_segmented_entry_point_on_a_shape_that_is_not_cut(A):
    # many heads or a short sequence: no workspace, and the bits of ae_gated_forward
    Q, K, V, la, kg = inputs(830, 2, 3, 3, 300, 64, 64, "mamba2")
    h = A.ae_gated_create(B=2, H=3, H_qk=3, L=300, D_qk=64, D_v=64, scale=0.125)
    assert A.ae_gated_workspace_bytes(h) == 0
    A.ae_gated_destroy(h)
    a = run(A, Q, K, V, la, kg, 0.125)
    b = run(A, Q, K, V, la, kg, 0.125, segmented=True)
    assert torch.equal(a, b)


def test_sampled_heads_at_benchmark_size(A):
    # 8 x 32 heads x 8192 tokens, 128/128, gated retention: three heads against the oracle
    B, H, L = 8, 32, 8192
    Q, K, V, la, kg = inputs(814, B, H, H, L, 128, 128, "gated_retention")
    scale = 1.0 / math.sqrt(128)
    got = run(A, Q, K, V, la, kg, scale).cpu()
    from oracle.gated_recurrent_oracle import gated_recurrent_head
    for b, h in ((0, 0), (3, 17), (7, 31)):
        ref = gated_recurrent_head(Q[b, h].float().numpy(), K[b, h].float().numpy(), V[b, h].float().numpy(), la[b, h].numpy(), scale=scale)
        check(got[b, h].double().numpy(), ref, f"benchmark size head ({b},{h})")

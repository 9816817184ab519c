"""GPU parity of the recurrent pattern: ae_recurrent_forward (chunk-parallel retention, through the C ABI) against
the token-by-token fp64 oracle on the same seeded bf16 inputs.  Bar as for the parallel pattern (bf16 operands,
bf16 chunk states into the read-out MFMAs, fp32 accumulation and fp32 running state): max-abs <= 1e-2 and
mean-abs <= 1e-3, relative to max(1, the largest |reference| of the row)."""
import math

import numpy as np
import pytest
import torch

from oracle.retention_recurrent_oracle import retention_recurrent as oracle_recurrent
from oracle.retention_recurrent_oracle import retention_recurrent_head
from paper_2502_15349_amd.workloads import Workload, make_inputs

pytestmark = pytest.mark.gpu

MAX_ABS, MEAN_ABS = 1e-2, 1e-3


@pytest.fixture(scope="module")
def A():
    from paper_2502_15349_amd import ae_attn
    return ae_attn


def _check(got, ref, what):
    rs = np.maximum(np.abs(ref).max(axis=-1, keepdims=True), 1.0)
    err = np.abs(got - ref) / rs
    print(f"{what}: max_abs {err.max():.3e} mean_abs {err.mean():.3e} |ref|max {np.abs(ref).max():.3e}", flush=True)
    assert np.isfinite(got).all()
    assert err.max() <= MAX_ABS and err.mean() <= MEAN_ABS, what


def _workload(name, cid, B, H, L, D):
    return Workload(name, cid, B, H, H, L, L, D, D, score_mod="head_decay", norm="none", mask="causal")


def _gammas(H):
    # RetNet's per-head rates 1 - 2^(-5-h), cycled, plus the undamped and a fast-forgetting head
    base = [1.0 - 2.0 ** (-5 - i) for i in range(6)] + [1.0, 0.5]
    return [base[i % len(base)] for i in range(H)]


# (L, chunk): several chunks with a short last one; exact multiples; a single chunk; shorter than a chunk; one row
CASES = [(300, 64), (700, 256), (512, 256), (384, 128), (64, 64), (50, 128), (1, 64), (257, 256), (129, 64)]


@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("L,chunk", CASES)
def test_recurrent_matches_oracle(A, D, L, chunk):
    w = _workload(f"rec_d{D}_L{L}_c{chunk}", 700 + D + L % 97, 2, 3, L, D)
    Q, K, V = make_inputs(w)
    gam = _gammas(w.H_q)
    scale = 1.0 / math.sqrt(D)
    print(f"case {w.name}", flush=True)
    dev = torch.device("cuda:0")
    O = A.retention_recurrent(Q.to(dev), K.to(dev), V.to(dev), scale=scale, gamma=gam, chunk=chunk)
    torch.cuda.synchronize()
    ref = oracle_recurrent(Q.float().numpy(), K.float().numpy(), V.float().numpy(), scale=scale, gamma=gam)
    _check(O.cpu().double().numpy(), ref, w.name)


def test_many_heads_take_one_launch_per_batch_entry(A):
    # B * H beyond the decay table of the intra-chunk kernel: the batch entries are launched one by one
    w = _workload("rec_many_heads", 791, 5, 64, 200, 64)
    Q, K, V = make_inputs(w)
    gam = _gammas(64)
    dev = torch.device("cuda:0")
    print(f"case {w.name}", flush=True)
    O = A.retention_recurrent(Q.to(dev), K.to(dev), V.to(dev), scale=0.125, gamma=gam, chunk=64).cpu().double().numpy()
    for b, h in ((0, 0), (2, 7), (4, 63), (3, 38)):
        ref = retention_recurrent_head(Q[b, h].float().numpy(), K[b, h].float().numpy(), V[b, h].float().numpy(), scale=0.125, gamma_h=gam[h])
        _check(O[b, h], ref, f"{w.name} b{b} h{h}")


def test_chunk_sizes_agree_and_workspace_is_reusable(A):
    # the same inputs through every chunk size (different cuts of the same sum), the workspace handed in and reused
    w = _workload("rec_chunks", 792, 1, 4, 1000, 128)
    Q, K, V = make_inputs(w)
    dev = torch.device("cuda:0")
    Qd, Kd, Vd = Q.to(dev), K.to(dev), V.to(dev)
    gam = _gammas(4)
    ref = oracle_recurrent(Q.float().numpy(), K.float().numpy(), V.float().numpy(), scale=0.09, gamma=gam)
    ws = torch.empty(1 << 24, dtype=torch.uint8, device=dev)
    for chunk in (64, 128, 256, 64):
        print(f"case {w.name} chunk {chunk}", flush=True)
        O = A.retention_recurrent(Qd, Kd, Vd, scale=0.09, gamma=gam, chunk=chunk, workspace=ws)
        torch.cuda.synchronize()
        _check(O.cpu().double().numpy(), ref, f"{w.name} chunk {chunk}")


def test_sampled_rows_at_benchmark_size(A):
    # the benchmark's launch configuration; the oracle walks three heads to the end
    B, H, L, D, chunk = 8, 32, 8192, 128, 256
    w = _workload("rec_b8_h32_s8192_d128", 793, B, H, L, D)
    Q, K, V = make_inputs(w)
    gam = [1.0 - 2.0 ** (-5 - (i % 8)) for i in range(H)]
    dev = torch.device("cuda:0")
    print(f"case {w.name}", flush=True)
    O = A.retention_recurrent(Q.to(dev), K.to(dev), V.to(dev), scale=1.0 / math.sqrt(D), gamma=gam, chunk=chunk)
    torch.cuda.synchronize()
    for b, h in ((0, 0), (5, 17), (7, 31)):
        ref = retention_recurrent_head(Q[b, h].float().numpy(), K[b, h].float().numpy(), V[b, h].float().numpy(),
                                       scale=1.0 / math.sqrt(D), gamma_h=gam[h])
        _check(O[b, h].cpu().double().numpy(), ref, f"{w.name} b{b} h{h}")


def test_hip_graph_replays(A):
    """ae_recurrent_forward allocates nothing and clears nothing (the states are overwritten whole), so its
    launches can be captured into a HIP graph: replayed four times with new K values and eager work between
    the replays, every replay must equal the eager call on the same inputs bit for bit; the first one is also
    held against the oracle."""
    dev = torch.device("cuda:0")
    w = _workload("rec_graph", 794, 2, 4, 600, 128)
    Qc, Kc, Vc = make_inputs(w)
    Q, K, V = Qc.to(dev), Kc.to(dev), Vc.to(dev)
    gam = _gammas(4)
    scale = 1.0 / math.sqrt(128)
    h = A.ae_recurrent_create(B=w.B, H=w.H_q, L=w.L_q, D_qk=128, D_v=128, chunk=256, scale=scale, gamma=gam)
    try:
        need = A.ae_recurrent_workspace_bytes(h)
        wsg, wse = (torch.zeros(need, dtype=torch.uint8, device=dev) for _ in range(2))
        Kg = K.clone()
        Og, Oe = (torch.zeros((w.B, w.H_q, w.L_q, 128), dtype=torch.float32, device=dev) for _ in range(2))

        def launch(O, ws, stream):
            A.ae_recurrent_forward(h, Q.data_ptr(), Kg.data_ptr(), V.data_ptr(), O.data_ptr(), ws.data_ptr(), need, stream.cuda_stream)

        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.graph(graph, stream=side):
            launch(Og, wsg, side)
        torch.cuda.synchronize()
        for replay in range(4):
            print(f"graph replay {replay}", flush=True)
            if replay:
                Kg.copy_((K.float() * (1.0 - 0.2 * replay)).to(torch.bfloat16).roll(replay, dims=2))
            Og.zero_()
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            launch(Oe, wse, torch.cuda.current_stream())
            torch.cuda.synchronize()
            assert torch.equal(Og, Oe), f"replay {replay} differs from the eager call"
            if replay == 0:
                ref = oracle_recurrent(Qc.float().numpy(), Kc.float().numpy(), Vc.float().numpy(), scale=scale, gamma=gam)
                _check(Og.cpu().double().numpy(), ref, "rec_graph replay 0")
    finally:
        A.ae_recurrent_destroy(h)


@pytest.mark.parametrize("D,chunk,cuts", [(128, 256, (0, 700, 1000)), (64, 64, (0, 50, 51, 300, 620)), (128, 128, (0, 128, 384, 385))])
def test_sequence_in_pieces_with_carried_state(A, D, chunk, cuts):
    """ae_recurrent_forward_state: a sequence processed in pieces, each starting from the state the piece before
    handed back, against the oracle's single walk; the last state against the oracle's final state."""
    L = cuts[-1]
    w = _workload(f"rec_pieces_d{D}_c{chunk}", 795 + D, 2, 3, L, D)
    Q, K, V = make_inputs(w)
    gam = [0.96875, 1.0, 0.9]
    scale = 1.0 / math.sqrt(D)
    dev = torch.device("cuda:0")
    Qd, Kd, Vd = Q.to(dev), K.to(dev), V.to(dev)
    state, outs = None, []
    for a, b in zip(cuts[:-1], cuts[1:]):
        print(f"case {w.name} tokens {a}..{b}", flush=True)
        O, state = A.retention_recurrent(Qd[:, :, a:b].contiguous(), Kd[:, :, a:b].contiguous(), Vd[:, :, a:b].contiguous(),
                                         scale=scale, gamma=gam, chunk=chunk, h_in=state, return_state=True)
        outs.append(O)
    torch.cuda.synchronize()
    got = torch.cat(outs, dim=2).cpu().double().numpy()
    ref = np.zeros_like(got)
    for b_ in range(w.B):
        for h_ in range(w.H_q):
            ref[b_, h_], hs = retention_recurrent_head(Q[b_, h_].float().numpy(), K[b_, h_].float().numpy(), V[b_, h_].float().numpy(),
                                                       scale=scale, gamma_h=gam[h_], return_state=True)
            _check(state[b_, h_].cpu().double().numpy(), hs, f"{w.name} final state b{b_} h{h_}")
    _check(got, ref, w.name)
    # the state alone (no piece before, none after) equals the one of a plain call
    O1, s1 = A.retention_recurrent(Qd, Kd, Vd, scale=scale, gamma=gam, chunk=chunk, return_state=True)
    torch.cuda.synchronize()
    _check(O1.cpu().double().numpy(), ref, w.name + " one call")
    for b_ in range(w.B):
        hs = retention_recurrent_head(Q[b_, 1].float().numpy(), K[b_, 1].float().numpy(), V[b_, 1].float().numpy(), scale=scale,
                                      gamma_h=gam[1], return_state=True)[1]
        _check(s1[b_, 1].cpu().double().numpy(), hs, f"{w.name} one call final state b{b_}")


@pytest.mark.parametrize("D", [64, 128])
def test_decoding_steps_after_a_prefill(A, D):
    """ae_recurrent_step: a prefill through ae_recurrent_forward_state, then six tokens one at a time on the
    carried fp32 state, against the oracle's single walk over all tokens (outputs of the steps and the last state)."""
    B, H, L0, T = 3, 5, 200, 6
    w = _workload(f"rec_step_d{D}", 797 + D, B, H, L0 + T, D)
    Q, K, V = make_inputs(w)
    gam = _gammas(H)
    scale = 1.0 / math.sqrt(D)
    dev = torch.device("cuda:0")
    Qd, Kd, Vd = Q.to(dev), K.to(dev), V.to(dev)
    print(f"case {w.name} prefill", flush=True)
    _, state = A.retention_recurrent(Qd[:, :, :L0].contiguous(), Kd[:, :, :L0].contiguous(), Vd[:, :, :L0].contiguous(),
                                     scale=scale, gamma=gam, chunk=64, return_state=True)
    h = A.ae_recurrent_create(B=B, H=H, L=1, D_qk=D, D_v=D, chunk=64, scale=scale, gamma=gam)
    outs = []
    try:
        st = torch.cuda.current_stream()
        for t in range(L0, L0 + T):
            print(f"case {w.name} step {t}", flush=True)
            q, k, v = (x[:, :, t].contiguous() for x in (Qd, Kd, Vd))
            o = torch.empty((B, H, D), dtype=torch.float32, device=dev)
            A.ae_recurrent_step(h, q.data_ptr(), k.data_ptr(), v.data_ptr(), state.data_ptr(), o.data_ptr(), st.cuda_stream)
            outs.append(o)
        torch.cuda.synchronize()
    finally:
        A.ae_recurrent_destroy(h)
    got = torch.stack(outs, dim=2).cpu().double().numpy()
    for b_ in range(B):
        for h_ in range(H):
            ref, hs = retention_recurrent_head(Q[b_, h_].float().numpy(), K[b_, h_].float().numpy(), V[b_, h_].float().numpy(),
                                               scale=scale, gamma_h=gam[h_], return_state=True)
            _check(got[b_, h_], ref[L0:], f"{w.name} steps b{b_} h{h_}")
            _check(state[b_, h_].cpu().double().numpy(), hs, f"{w.name} state b{b_} h{h_}")
    # from a zero state the steps alone are the recurrence in fp32: much tighter than the bf16 bar
    h = A.ae_recurrent_create(B=B, H=H, L=1, D_qk=D, D_v=D, chunk=64, scale=scale, gamma=gam)
    state0 = torch.zeros((B, H, D, D), dtype=torch.float32, device=dev)
    outs = []
    try:
        for t in range(T):
            q, k, v = (x[:, :, t].contiguous() for x in (Qd, Kd, Vd))
            o = torch.empty((B, H, D), dtype=torch.float32, device=dev)
            A.ae_recurrent_step(h, q.data_ptr(), k.data_ptr(), v.data_ptr(), state0.data_ptr(), o.data_ptr(), torch.cuda.current_stream().cuda_stream)
            outs.append(o)
        torch.cuda.synchronize()
    finally:
        A.ae_recurrent_destroy(h)
    got = torch.stack(outs, dim=2).cpu().double().numpy()
    ref = oracle_recurrent(Q[:, :, :T].float().numpy(), K[:, :, :T].float().numpy(), V[:, :, :T].float().numpy(), scale=scale, gamma=gam)
    err = np.abs(got - ref).max()
    print(f"{w.name} steps from zero: max abs {err:.3e}", flush=True)
    assert err <= 1e-4


def test_state_updated_in_place(A):
    """h_out may be the buffer h_in points to (every workgroup reads its slice of the state before it writes it):
    the in-place call must give the bits of the call with separate buffers."""
    dev = torch.device("cuda:0")
    w = _workload("rec_inplace", 799, 2, 4, 333, 128)
    Q, K, V = (x.to(dev) for x in make_inputs(w))
    gam = _gammas(4)
    g = torch.Generator(device="cpu")
    g.manual_seed(799)
    h0 = torch.randn((2, 4, 128, 128), generator=g, dtype=torch.float32).to(dev)
    O1, s1 = A.retention_recurrent(Q, K, V, scale=0.09, gamma=gam, chunk=128, h_in=h0, return_state=True)
    h = A.ae_recurrent_create(B=2, H=4, L=333, D_qk=128, D_v=128, chunk=128, scale=0.09, gamma=gam)
    try:
        ws = torch.empty(A.ae_recurrent_workspace_bytes(h), dtype=torch.uint8, device=dev)
        O2 = torch.empty_like(O1)
        buf = h0.clone()
        print("case rec_inplace", flush=True)
        A.ae_recurrent_forward_state(h, Q.data_ptr(), K.data_ptr(), V.data_ptr(), buf.data_ptr(), O2.data_ptr(), buf.data_ptr(),
                                     ws.data_ptr(), ws.numel(), torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
    finally:
        A.ae_recurrent_destroy(h)
    assert torch.equal(O1, O2) and torch.equal(s1, buf)
    # and against the oracle, which starts from the same state
    for b_, h_ in ((0, 0), (1, 3)):
        ref, hs = retention_recurrent_head(Q[b_, h_].float().cpu().numpy(), K[b_, h_].float().cpu().numpy(), V[b_, h_].float().cpu().numpy(),
                                           scale=0.09, gamma_h=gam[h_], return_state=True, h0=h0[b_, h_].cpu().double().numpy())
        _check(O2[b_, h_].cpu().double().numpy(), ref, f"rec_inplace b{b_} h{h_}")
        _check(buf[b_, h_].cpu().double().numpy(), hs, f"rec_inplace state b{b_} h{h_}")


def test_bf16_output(A):
    """desc.out_dtype = bf16: the same fp32 rows, rounded to nearest even when stored (bit-equal to rounding the
    fp32 output; the fp32 output itself is held against the oracle above)."""
    dev = torch.device("cuda:0")
    for D, L, chunk in ((128, 700, 256), (64, 300, 64)):
        w = _workload(f"rec_bf16_d{D}", 800 + D, 2, 4, L, D)
        Q, K, V = (x.to(dev) for x in make_inputs(w))
        gam = _gammas(4)
        print(f"case {w.name}", flush=True)
        O32 = A.retention_recurrent(Q, K, V, scale=0.1, gamma=gam, chunk=chunk)
        O16 = A.retention_recurrent(Q, K, V, scale=0.1, gamma=gam, chunk=chunk, out_dtype=torch.bfloat16)
        torch.cuda.synchronize()
        assert O16.dtype == torch.bfloat16 and torch.equal(O16, O32.to(torch.bfloat16))

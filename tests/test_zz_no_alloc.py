"""The entry point that allocates nothing (ae_attn_forward_split_static: partial results in the library's static
device scratch) against ae_attn_forward_split with a caller's workspace, through the C ABI: the same kernels in the
same order, so the outputs must be equal bit for bit -- on two calls in a row, the second with a smaller input (the
scratch keeps the first call's contents), and both against the fp64 oracle at the forward bar."""
import numpy as np
import pytest
import torch

from oracle import attention, row_stats_head
from paper_2502_15349_amd.workloads import Workload, make_inputs

pytestmark = pytest.mark.gpu

MAX_ABS, MEAN_ABS = 1e-2, 1e-3


@pytest.fixture(scope="module")
def A():
    from paper_2502_15349_amd import ae_attn
    return ae_attn


def _both(A, w, splits):
    dev = torch.device("cuda:0")
    Q, K, V = make_inputs(w)
    Qd, Kd, Vd = Q.to(dev), K.to(dev), V.to(dev)
    h = A.ae_attn_create(B=w.B, H_q=w.H_q, H_kv=w.H_kv, L_q=w.L_q, L_k=w.L_k, D_qk=w.D_qk, D_v=w.D_v, scale=w.scale_value,
                         mask=w.mask, kv_splits=splits)
    try:
        need = A.ae_attn_workspace_bytes(h)
        assert 0 < need <= A.AE_ATTN_STATIC_SCRATCH_BYTES
        ws = torch.empty(need, dtype=torch.uint8, device=dev)
        O1 = torch.full((w.B, w.H_q, w.L_q, w.D_v), float("nan"), dtype=torch.float32, device=dev)
        O2 = torch.full_like(O1, float("nan"))
        s1 = torch.full((w.B, w.H_q, w.L_q), float("nan"), dtype=torch.float32, device=dev)
        s2 = torch.full_like(s1, float("nan"))
        st = torch.cuda.current_stream().cuda_stream
        A.ae_attn_forward_split(h, Qd.data_ptr(), Kd.data_ptr(), Vd.data_ptr(), O1.data_ptr(), s1.data_ptr(), ws.data_ptr(), need, st)
        A.ae_attn_forward_split_static(h, Qd.data_ptr(), Kd.data_ptr(), Vd.data_ptr(), O2.data_ptr(), s2.data_ptr(), st)
        torch.cuda.synchronize()
    finally:
        A.ae_attn_destroy(h)
    assert torch.equal(O1, O2), "static scratch and workspace disagree"
    assert torch.equal(s1, s2)
    ref = attention(Q, K, V, scale=w.scale_value, mask=w.oracle_mask())
    err = np.abs(O2.cpu().double().numpy() - ref)
    print(f"{w.name}: max_abs {err.max():.3e} mean_abs {err.mean():.3e}", flush=True)
    assert err.max() <= MAX_ABS and err.mean() <= MEAN_ABS
    g = w.H_q // w.H_kv
    want = row_stats_head(Q[0, 1], K[0, 1 // g], scale=w.scale_value, mask=w.oracle_mask())
    got = s2[0, 1].cpu().double().numpy()
    fin = np.isfinite(want)
    assert (np.isneginf(got) == np.isneginf(want)).all() and np.abs(got[fin] - want[fin]).max() <= 4e-3   # (the bar of the row statistic, see test_gpu_parity.LSE_ABS)


def test_static_scratch_equals_workspace_two_calls_second_smaller(A):
    # a decoding shape (one query row, 8k keys, 12 ranges), then a smaller one with fewer rows, keys and ranges
    _both(A, Workload("static_big", 90, 2, 16, 4, 1, 8192, 192, 128, mask="causal"), 12)
    _both(A, Workload("static_small", 91, 1, 4, 2, 3, 700, 192, 128, mask="causal"), 3)


def test_static_scratch_refuses_what_does_not_fit(A):
    # 64 x 16 x 40 rows x 8 ranges x 129 floats = 21 MB of partial results: more than the static scratch holds
    h = A.ae_attn_create(B=64, H_q=16, H_kv=16, L_q=40, L_k=4096, D_qk=128, D_v=128, scale=0.1, kv_splits=8)
    try:
        assert A.ae_attn_workspace_bytes(h) > A.AE_ATTN_STATIC_SCRATCH_BYTES
        with pytest.raises(A.AeAttnError) as ei:
            A.ae_attn_forward_split_static(h, 256, 512, 768, 1024)
        assert ei.value.status == A.AE_ERR_UNSUPPORTED
    finally:
        A.ae_attn_destroy(h)

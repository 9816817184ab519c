"""CPU-only checks of the C ABI: the library loads, exports every symbol the
header declares, and rejects bad descriptors without touching a device."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2502_15349_amd", "libae_attn.so")

pytestmark = pytest.mark.skipif(not os.path.exists(LIB), reason="libae_attn.so not built (run __graft_entry__.build())")


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "ae_attn.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(ae_(?:attn|calib|recurrent|gated)_[a-z0-9_]+)\s*\(", hdr))
    assert {"ae_attn_create", "ae_attn_forward", "ae_attn_destroy", "ae_attn_query", "ae_calib_mfma_bf16"} <= names
    lib = ctypes.CDLL(LIB)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in the header but not exported"


def _ok_desc():
    return dict(B=1, H_q=4, H_kv=2, L_q=100, L_k=100, D_qk=128, D_v=128, scale=0.1)


def test_create_query_destroy_roundtrip():
    from paper_2502_15349_amd import ae_attn as A
    h = A.ae_attn_create(**_ok_desc(), mask="causal")
    q = A.ae_attn_query(h)
    assert q["block_n"] == 64 and q["block_m"] % 32 == 0 and q["block_threads"] % 64 == 0
    assert q["lds_bytes"] <= 160 * 1024
    # grid covers every (group, q head in group, q tile) at least once
    n_qt = -(-100 // q["block_m"])
    assert q["grid_size"] >= 1 * 2 * 2 * n_qt
    assert "attn_fwd" in q["kernel"]
    A.ae_attn_destroy(h)
    A.ae_attn_destroy(None)
    assert A.ae_attn_version() >= 1
    # Table 2's retention head dims: 256 / 512 and 256 / 128, for the retention variants only
    ret = dict(B=1, H_q=4, H_kv=4, L_q=100, L_k=100, D_qk=256, scale=0.1, score_mod="head_decay", gamma=[.9] * 4, mask="causal")
    for dv in (128, 512):
        h = A.ae_attn_create(**ret, D_v=dv, norm="abssum")
        assert "256,128" in A.ae_attn_query(h)["kernel"]
        A.ae_attn_destroy(h)
    for bad in (dict(D_v=512, norm="abssum", kv_splits=4), dict(D_v=256, norm="abssum")):
        with pytest.raises(A.AeAttnError) as ei:
            A.ae_attn_create(**ret, **bad)
        assert ei.value.status == A.AE_ERR_UNSUPPORTED
    with pytest.raises(A.AeAttnError) as ei:     # softmax is not built at these head dims
        A.ae_attn_create(B=1, H_q=4, H_kv=4, L_q=100, L_k=100, D_qk=256, D_v=512, scale=0.1)
    assert ei.value.status == A.AE_ERR_UNSUPPORTED


@pytest.mark.parametrize("patch,status", [
    (dict(B=0), 1), (dict(L_q=-3), 1), (dict(H_q=3), 1), (dict(scale=float("nan")), 1),
    (dict(scale=0.0), 1), (dict(scale=float("inf")), 1),
    (dict(D_qk=96), 2), (dict(D_qk=64), 2), (dict(D_v=64), 2),
    (dict(norm=9), 2), (dict(score_mod=7), 2), (dict(mask=5), 2),
    (dict(score_mod="head_decay", norm="abssum", mask="causal"), 1),            # gamma missing
    (dict(score_mod="head_decay", norm="abssum", mask="none", gamma=[.9] * 4), 2),
    (dict(score_mod="head_decay", norm="softmax", mask="causal", gamma=[.9] * 4), 2),
    (dict(score_mod="head_decay", norm="abssum", mask="causal", gamma=[.9, 0.0, .9, .9]), 1),
    (dict(score_mod="relu", norm="softmax"), 2),
    (dict(score_mod="bias", bias=float("inf")), 1),
    (dict(q_stride=(100 * 4 * 128, 100 * 128, 132)), 1),                          # not a multiple of 8
    (dict(k_stride=(100 * 2 * 128, 100 * 128, 64)), 1),                           # row stride < D
    (dict(o_stride=(100 * 4 * 130, 100 * 130, 130)), 1),                          # not a multiple of 4
])
def test_create_rejects_bad_descriptors(patch, status):
    from paper_2502_15349_amd import ae_attn as A
    d = _ok_desc()
    d.update(patch)
    with pytest.raises(A.AeAttnError) as ei:
        A.ae_attn_create(**d)
    assert ei.value.status == status
    assert A.ae_attn_last_error() != ""


def test_forward_rejects_bad_pointers_without_launching():
    from paper_2502_15349_amd import ae_attn as A
    h = A.ae_attn_create(**_ok_desc())
    try:
        for args in ((0, 256, 512, 768), (256, 512, 768, 0), (256 + 4, 512, 768, 1024), (256, 512, 768, 256)):
            with pytest.raises(A.AeAttnError) as ei:
                A.ae_attn_forward(h, *args)
            assert ei.value.status == A.AE_ERR_INVALID_ARG
        with pytest.raises(A.AeAttnError):
            A.ae_attn_forward(None, 256, 512, 768, 1024)
    finally:
        A.ae_attn_destroy(h)


def test_forward_stats_rejects_bad_arguments_without_launching():
    from paper_2502_15349_amd import ae_attn as A
    h = A.ae_attn_create(**_ok_desc())
    try:
        for args in ((256, 512, 768, 1024, 0), (256, 512, 768, 1024, 2048 + 2), (256, 512, 768, 1024, 1024),
                     (0, 512, 768, 1024, 2048)):
            with pytest.raises(A.AeAttnError) as ei:
                A.ae_attn_forward_stats(h, *args)
            assert ei.value.status == A.AE_ERR_INVALID_ARG
    finally:
        A.ae_attn_destroy(h)
    # a normalization without a row reduction keeps no statistic
    d = _ok_desc()
    d.update(norm="sigmoid")
    h = A.ae_attn_create(**d)
    try:
        with pytest.raises(A.AeAttnError) as ei:
            A.ae_attn_forward_stats(h, 256, 512, 768, 1024, 2048)
        assert ei.value.status == A.AE_ERR_UNSUPPORTED
    finally:
        A.ae_attn_destroy(h)


def test_bf16_output_accepted_and_unknown_dtype_rejected():
    from paper_2502_15349_amd import ae_attn as A
    A.ae_attn_destroy(A.ae_attn_create(**_ok_desc(), out_dtype="bf16"))
    with pytest.raises(A.AeAttnError) as ei:
        A.ae_attn_create(**_ok_desc(), out_dtype=7)
    assert ei.value.status == A.AE_ERR_UNSUPPORTED


def test_sliding_window_descriptor_checks():
    from paper_2502_15349_amd import ae_attn as A
    A.ae_attn_destroy(A.ae_attn_create(**_ok_desc(), mask="sliding_window", window=17))
    for window in (0, -3):
        with pytest.raises(A.AeAttnError) as ei:
            A.ae_attn_create(**_ok_desc(), mask="sliding_window", window=window)
        assert ei.value.status == A.AE_ERR_INVALID_ARG
    # a window far wider than the sequence is the causal mask (also with more queries than keys)
    A.ae_attn_destroy(A.ae_attn_create(**_ok_desc(), mask="sliding_window", window=2**31 - 1))
    d = _ok_desc()
    d.update(L_q=300, L_k=40)
    A.ae_attn_destroy(A.ae_attn_create(**d, mask="sliding_window", window=2**31 - 1))
    # the window comes with softmax, sigmoid and no normalization only
    d = _ok_desc()
    d.update(norm="abssum")
    with pytest.raises(A.AeAttnError) as ei:
        A.ae_attn_create(**d, mask="sliding_window", window=8)
    assert ei.value.status == A.AE_ERR_UNSUPPORTED


def test_split_keys_descriptor_and_workspace():
    from paper_2502_15349_amd import ae_attn as A
    d = dict(B=2, H_q=4, H_kv=2, L_q=3, L_k=1000, D_qk=128, D_v=128, scale=0.1)
    h = A.ae_attn_create(**d)
    assert A.ae_attn_workspace_bytes(h) == 0
    A.ae_attn_destroy(h)
    h = A.ae_attn_create(**d, kv_splits=4)          # 16 key tiles -> 4 ranges of 4
    try:
        assert A.ae_attn_workspace_bytes(h) == 4 * (2 * 4 * 3) * (128 + 1) * 4
        with pytest.raises(A.AeAttnError) as ei:     # the plain entry point has no workspace to give
            A.ae_attn_forward(h, 256, 512, 768, 1024)
        assert ei.value.status == A.AE_ERR_INVALID_ARG
        for ws, nbytes in ((0, 1 << 20), (4096 + 8, 1 << 20), (4096, 100), (1024, 1 << 20)):
            with pytest.raises(A.AeAttnError) as ei:
                A.ae_attn_forward_split(h, 256, 512, 768, 1024, 0, ws, nbytes)
            assert ei.value.status == A.AE_ERR_INVALID_ARG
    finally:
        A.ae_attn_destroy(h)
    h = A.ae_attn_create(**d, kv_splits=100)        # more ranges than tiles: one tile each
    assert A.ae_attn_workspace_bytes(h) == 16 * (2 * 4 * 3) * (128 + 1) * 4
    A.ae_attn_destroy(h)
    for bad in (dict(norm="sigmoid"), dict(mask="sliding_window", window=5)):
        with pytest.raises(A.AeAttnError) as ei:
            A.ae_attn_create(**d, kv_splits=4, **bad)
        assert ei.value.status == A.AE_ERR_UNSUPPORTED
    with pytest.raises(A.AeAttnError) as ei:
        A.ae_attn_create(**d, kv_splits=-2)
    assert ei.value.status == A.AE_ERR_INVALID_ARG
    # automatic choice: splits a decoding shape, leaves a prefill shape and a sigmoid alone
    h = A.ae_attn_create(B=1, H_q=16, H_kv=16, L_q=1, L_k=8192, D_qk=192, D_v=128, scale=0.1, kv_splits=-1)
    assert A.ae_attn_workspace_bytes(h) == 12 * 16 * (128 + 1) * 4      # 128 key tiles in 12 ranges of 11
    A.ae_attn_destroy(h)
    h = A.ae_attn_create(B=8, H_q=16, H_kv=4, L_q=1, L_k=8192, D_qk=128, D_v=128, scale=0.1, kv_splits=-1)
    assert A.ae_attn_workspace_bytes(h) == 2 * 128 * (128 + 1) * 4      # 128 rows: about 192 workgroups = 2 ranges
    A.ae_attn_destroy(h)
    for kw in (dict(B=4, H_q=32, H_kv=8, L_q=2048, L_k=2048), dict(B=1, H_q=16, H_kv=16, L_q=1, L_k=8192, norm="sigmoid"),
               dict(B=1, H_q=16, H_kv=16, L_q=1, L_k=200)):
        h = A.ae_attn_create(D_qk=128, D_v=128, scale=0.1, kv_splits=-1, **kw)
        assert A.ae_attn_workspace_bytes(h) == 0
        A.ae_attn_destroy(h)


def test_backward_rejects_bad_arguments_without_launching():
    from paper_2502_15349_amd import ae_attn as A
    d = _ok_desc()
    h = A.ae_attn_create(**d)
    try:
        rows = d["B"] * d["H_q"] * d["L_q"]
        assert A.ae_attn_backward_workspace_bytes(h) == 4 * rows
        ok = [256 * (i + 1) for i in range(10)]   # Q K V O dO stats dQ dK dV workspace
        bad = []
        for pos in (0, 4, 6, 9):                  # a null pointer
            a = list(ok)
            a[pos] = 0
            bad.append((a, 4 * rows))
        a = list(ok)
        a[7] = ok[7] + 8                          # misaligned output
        bad.append((a, 4 * rows))
        a = list(ok)
        a[6] = ok[0]                              # dQ aliases Q
        bad.append((a, 4 * rows))
        a = list(ok)
        a[8] = ok[7]                              # dV aliases dK
        bad.append((a, 4 * rows))
        bad.append((list(ok), 4 * rows - 4))      # workspace too small
        for args, ws_bytes in bad:
            with pytest.raises(A.AeAttnError) as ei:
                A.ae_attn_backward(h, *args, ws_bytes)
            assert ei.value.status == A.AE_ERR_INVALID_ARG, A.ae_attn_last_error()
    finally:
        A.ae_attn_destroy(h)
    # only softmax needs a workspace; normalizations and masks outside the built set are refused
    for patch, want in ((dict(norm="sigmoid"), None), (dict(norm="abssum"), "ws"),
                        (dict(norm="none", score_mod="relu"), None),
                        (dict(norm="abssum", score_mod="head_decay", mask="causal", gamma=[.9] * 4), "ws"),
                        (dict(norm="none", score_mod="head_decay", mask="causal", gamma=[.9] * 4), None),
                        # a bias-tensor handle runs through ae_attn_backward_bias
                        (dict(score_mod="bias_tensor", bias_stride=(0, 0, 104)), A.AE_ERR_INVALID_ARG),
                        (dict(mask="sliding_window", window=8), "ws")):
        dd = _ok_desc()
        dd.update(patch)
        h = A.ae_attn_create(**dd)
        try:
            if want == "ws":       # supported, softmax: the workspace holds delta
                assert A.ae_attn_backward_workspace_bytes(h) == 4 * dd["B"] * dd["H_q"] * dd["L_q"]
            elif want is None:
                assert A.ae_attn_backward_workspace_bytes(h) == 0
            else:
                with pytest.raises(A.AeAttnError) as ei:
                    A.ae_attn_backward(h, *[256 * (i + 1) for i in range(10)], 1 << 20)
                assert ei.value.status == want
        finally:
            A.ae_attn_destroy(h)


def test_bias_tensor_descriptor_and_entry_point_checks():
    from paper_2502_15349_amd import ae_attn as A
    d = _ok_desc()
    d.update(score_mod="bias_tensor", bias_stride=(0, 0, 104))    # L_k = 100: rows padded to a multiple of 8
    h = A.ae_attn_create(**d)
    try:
        with pytest.raises(A.AeAttnError) as ei:      # needs its own entry point
            A.ae_attn_forward(h, 256, 512, 768, 1024)
        assert ei.value.status == A.AE_ERR_INVALID_ARG
        for args in ((256, 512, 768, 0, 1024), (256, 512, 768, 2056, 1024), (256, 512, 768, 1024, 1024)):   # null, misaligned, aliasing O
            with pytest.raises(A.AeAttnError) as ei:
                A.ae_attn_forward_bias(h, *args)
            assert ei.value.status == A.AE_ERR_INVALID_ARG
        # backward with the bias gradient: Q K V bias O dO stats dQ dK dV | dBias, row stride | workspace, bytes
        ok = [256 * (i + 1) for i in range(10)]
        ws = A.ae_attn_backward_workspace_bytes(h)
        for db, ld in ((8192 + 4, 104),        # misaligned
                       (8192, 96),             # row stride < L_k
                       (8192, 102),            # row stride not a multiple of 4
                       (ok[3], 104),           # aliases the bias tensor
                       (ok[7], 104)):          # aliases dQ
            with pytest.raises(A.AeAttnError) as ei:
                A.ae_attn_backward_bias(h, *ok, db, ld, 1 << 16, ws)
            assert ei.value.status == A.AE_ERR_INVALID_ARG, (db, ld, A.ae_attn_last_error())
        with pytest.raises(A.AeAttnError) as ei:      # null bias tensor
            A.ae_attn_backward_bias(h, *ok[:3], 0, *ok[4:], 0, 0, 1 << 16, ws)
        assert ei.value.status == A.AE_ERR_INVALID_ARG
    finally:
        A.ae_attn_destroy(h)
    h = A.ae_attn_create(**_ok_desc())
    try:
        with pytest.raises(A.AeAttnError) as ei:      # a bias tensor for a handle that takes none
            A.ae_attn_forward_bias(h, 256, 512, 768, 2048, 1024)
        assert ei.value.status == A.AE_ERR_INVALID_ARG
    finally:
        A.ae_attn_destroy(h)
    for patch, status in ((dict(norm="abssum"), A.AE_ERR_UNSUPPORTED), (dict(mask="sliding_window", window=4), A.AE_ERR_UNSUPPORTED),
                          (dict(kv_splits=4), A.AE_ERR_UNSUPPORTED), (dict(D_v=256), A.AE_ERR_UNSUPPORTED),
                          (dict(bias_stride=(0, 0, 96)), A.AE_ERR_INVALID_ARG),      # row stride < L_k
                          (dict(bias_stride=(0, 0, 100)), A.AE_ERR_INVALID_ARG)):    # not a multiple of 8
        dd = _ok_desc()
        dd.update(score_mod="bias_tensor", bias_stride=(0, 0, 104))
        dd.update(patch)
        with pytest.raises(A.AeAttnError) as ei:
            A.ae_attn_create(**dd)
        assert ei.value.status == status, (patch, A.ae_attn_last_error())
    dd = _ok_desc()
    dd.update(score_mod="bias_tensor", bias_stride=(0, 0, 104))    # shared over batch and heads, padded rows
    A.ae_attn_destroy(A.ae_attn_create(**dd))
    # the automatic split choice leaves a handle with a bias tensor alone (its entry point takes no workspace):
    # a decoding shape that would be split without the bias tensor
    dec = dict(B=1, H_q=16, H_kv=16, L_q=1, L_k=8192, D_qk=128, D_v=128, scale=0.1, kv_splits=-1)
    h = A.ae_attn_create(**dec)
    assert A.ae_attn_workspace_bytes(h) > 0
    A.ae_attn_destroy(h)
    h = A.ae_attn_create(**dec, score_mod="bias_tensor")
    assert A.ae_attn_workspace_bytes(h) == 0
    A.ae_attn_destroy(h)


def test_slabs_beyond_32_bit_offsets_are_refused():
    from paper_2502_15349_amd import ae_attn as A
    d = _ok_desc()
    d.update(L_q=1 << 20, L_k=1 << 20, q_stride=(0, 0, 4096))      # 2^20 rows x 8 KB = 8 GiB per (batch, head)
    d["q_stride"] = ((1 << 20) * 4096 * 4, (1 << 20) * 4096, 4096)
    with pytest.raises(A.AeAttnError) as ei:
        A.ae_attn_create(**d)
    assert ei.value.status == A.AE_ERR_UNSUPPORTED
    d = _ok_desc()
    d.update(L_q=1 << 16, L_k=1 << 16, score_mod="bias_tensor")    # bias rows of 128 KB x 65536 rows = 8 GiB
    with pytest.raises(A.AeAttnError) as ei:
        A.ae_attn_create(**d)
    assert ei.value.status == A.AE_ERR_UNSUPPORTED


def test_padded_strides_accepted():
    from paper_2502_15349_amd import ae_attn as A
    h = A.ae_attn_create(**_ok_desc(), q_stride=(100 * 4 * 136, 100 * 136, 136))
    A.ae_attn_destroy(h)


def test_calibration_kernel_rejects_bad_arguments_without_launching():
    from paper_2502_15349_amd import ae_attn as A
    for args in [(0, 1 << 20, 4, 10), (4096, 100, 4, 10), (4096, 1 << 20, 0, 10), (4096, 1 << 20, 4, 0)]:
        with pytest.raises(A.AeAttnError) as ei:
            A.ae_calib_mfma_bf16(*args)
        assert ei.value.status == A.AE_ERR_INVALID_ARG


def test_recurrent_descriptor_and_entry_point_checks():
    from paper_2502_15349_amd import ae_attn as A
    ok = dict(B=2, H=4, L=300, D_qk=128, D_v=128, chunk=64, scale=0.1, gamma=[0.9, 0.95, 0.99, 1.0])
    h = A.ae_recurrent_create(**ok)
    try:
        need = A.ae_recurrent_workspace_bytes(h)
        assert need == 2 * 4 * 5 * 128 * 128 * 2          # 5 chunks: a bf16 state in front of each
        good = (1 << 20, 2 << 20, 3 << 20, 4 << 20, 5 << 20)
        for args, nbytes in (((0,) + good[1:], need), (good[:3] + (0,) + good[4:], need), ((good[0] + 8,) + good[1:], need),
                             (good[:3] + (good[0],) + good[4:], need),             # O aliases Q
                             (good[:4] + (0,), need), (good[:4] + (good[4] + 64,), need), (good, need - 1),
                             (good[:4] + (good[3],), need)):                       # workspace aliases O
            with pytest.raises(A.AeAttnError) as ei:
                A.ae_recurrent_forward(h, *args, nbytes)
            assert ei.value.status == A.AE_ERR_INVALID_ARG, (args, A.ae_attn_last_error())
        with pytest.raises(A.AeAttnError):
            A.ae_recurrent_forward(None, *good, need)
        # states: Q K V h_in O h_out workspace
        q, k, v, o, ws = good
        for args in ((q, k, v, (6 << 20) + 4, o, 0, ws),      # misaligned h_in
                     (q, k, v, 0, o, o, ws),                   # h_out aliases O
                     (q, k, v, o, o, 0, ws),                   # h_in aliases O
                     (q, k, v, 0, o, ws, ws)):                 # h_out aliases the workspace
            with pytest.raises(A.AeAttnError) as ei:
                A.ae_recurrent_forward_state(h, *args, need)
            assert ei.value.status == A.AE_ERR_INVALID_ARG, (args, A.ae_attn_last_error())
        # one-token step: q k v state o
        for args in ((0, k, v, ws, o), (q, k, v, ws + 4, o), (q, k, v, ws, ws), (q, k, v, q, o)):
            with pytest.raises(A.AeAttnError) as ei:
                A.ae_recurrent_step(h, *args)
            assert ei.value.status == A.AE_ERR_INVALID_ARG, (args, A.ae_attn_last_error())
    finally:
        A.ae_recurrent_destroy(h)
    A.ae_recurrent_destroy(None)
    one = dict(ok, L=64)                                   # a single chunk: one slot (used when a state is handed in)
    h = A.ae_recurrent_create(**one)
    assert A.ae_recurrent_workspace_bytes(h) == 2 * 4 * 128 * 128 * 2
    A.ae_recurrent_destroy(h)
    for patch, status in ((dict(chunk=100), A.AE_ERR_UNSUPPORTED), (dict(D_qk=192), A.AE_ERR_UNSUPPORTED),
                          (dict(D_qk=256, D_v=512), A.AE_ERR_UNSUPPORTED), (dict(H=300, gamma=[0.9] * 300), A.AE_ERR_UNSUPPORTED),
                          (dict(gamma=[0.9, 0.9, 0.9, 1.5]), A.AE_ERR_INVALID_ARG), (dict(gamma=[0.9, 0.0, 0.9, 0.9]), A.AE_ERR_INVALID_ARG),
                          (dict(gamma=None), A.AE_ERR_INVALID_ARG), (dict(L=0), A.AE_ERR_INVALID_ARG), (dict(out_dtype=7), A.AE_ERR_INVALID_ARG),
                          (dict(scale=float("nan")), A.AE_ERR_INVALID_ARG), (dict(B=0), A.AE_ERR_INVALID_ARG)):
        with pytest.raises(A.AeAttnError) as ei:
            A.ae_recurrent_create(**dict(ok, **patch))
        assert ei.value.status == status, (patch, A.ae_attn_last_error())


def test_gated_descriptor_and_entry_point_checks():
    """ae_gated_*: every descriptor and pointer check answers with a status before anything is launched."""
    from paper_2502_15349_amd import ae_attn as A
    ok = dict(B=2, H=8, H_qk=2, L=300, D_qk=128, D_v=64, scale=0.1)
    h = A.ae_gated_create(**ok)
    try:
        # Q K V log_decay key_gate h_in O h_out
        q, k, v, la, kg, hin, o, hout = (i << 20 for i in range(1, 9))
        for args in ((0, k, v, la, kg, hin, o, hout), (q, k, v, 0, kg, hin, o, hout), (q, k, v, la, kg, hin, 0, hout),
                     (q + 8, k, v, la, 0, 0, o, 0),            # misaligned Q
                     (q, k, v, la + 2, 0, 0, o, 0),            # misaligned gate
                     (q, k, v, la, 0, hin + 4, o, 0),          # misaligned state
                     (q, k, v, la, 0, 0, q, 0),                # O aliases Q
                     (q, k, v, la, kg, 0, o, kg),              # h_out aliases an input
                     (q, k, v, la, 0, 0, o, o)):               # h_out aliases O
            with pytest.raises(A.AeAttnError) as ei:
                A.ae_gated_forward(h, *args)
            assert ei.value.status == A.AE_ERR_INVALID_ARG, (args, A.ae_attn_last_error())
        with pytest.raises(A.AeAttnError):
            A.ae_gated_forward(None, q, k, v, la, 0, 0, o, 0)
    finally:
        A.ae_gated_destroy(h)
    A.ae_gated_destroy(None)
    for patch, status in ((dict(D_qk=192), A.AE_ERR_UNSUPPORTED), (dict(D_v=256), A.AE_ERR_UNSUPPORTED),
                          (dict(H_qk=3), A.AE_ERR_INVALID_ARG), (dict(H_qk=0), A.AE_ERR_INVALID_ARG), (dict(L=0), A.AE_ERR_INVALID_ARG),
                          (dict(B=0), A.AE_ERR_INVALID_ARG), (dict(scale=0.0), A.AE_ERR_INVALID_ARG),
                          (dict(scale=float("inf")), A.AE_ERR_INVALID_ARG), (dict(out_dtype=9), A.AE_ERR_INVALID_ARG),
                          (dict(L=1 << 30), A.AE_ERR_UNSUPPORTED)):
        with pytest.raises(A.AeAttnError) as ei:
            A.ae_gated_create(**dict(ok, **patch))
        assert ei.value.status == status, (patch, A.ae_attn_last_error())


def test_gated_backward_entry_point_checks():
    from paper_2502_15349_amd import ae_attn as A
    h = A.ae_gated_create(B=2, H=8, H_qk=2, L=300, D_qk=128, D_v=64, scale=0.1)
    hu = A.ae_gated_create(B=2, H=8, H_qk=8, L=300, D_qk=128, D_v=64, scale=0.1)
    try:
        rows = 2 * 8 * 300 * 4
        assert A.ae_gated_backward_workspace_bytes(hu) == (rows + 255) // 256 * 256            # per-token terms only
        need = A.ae_gated_backward_workspace_bytes(h)
        assert need == (rows + 255) // 256 * 256 + 2 * 2 * 8 * 300 * 128 * 4                    # + two per-head gradients
        # Q K V log_decay key_gate dO dQ dK dV dlog_decay dkey_gate workspace
        q, k, v, la, kg, do, dq, dk, dv, dla, dkg, ws = (i << 24 for i in range(1, 13))
        good = (q, k, v, la, kg, do, dq, dk, dv, dla, dkg, ws)
        for pos, val in ((0, 0), (5, 0), (6, 0), (9, 0),             # null Q, dO, dQ, dlog_decay
                         (10, 0),                                     # key gate without a buffer for its gradient
                         (2, v + 8), (8, dv + 4), (9, dla + 2),       # misaligned
                         (6, q), (7, dq), (10, la), (11, dv),         # aliases
                         (11, ws + 128), (11, 0)):                    # workspace misaligned / missing
            args = list(good)
            args[pos] = val
            with pytest.raises(A.AeAttnError) as ei:
                A.ae_gated_backward(h, *args, need)
            assert ei.value.status == A.AE_ERR_INVALID_ARG, (pos, val, A.ae_attn_last_error())
        with pytest.raises(A.AeAttnError) as ei:
            A.ae_gated_backward(h, *good, need - 1)
        assert ei.value.status == A.AE_ERR_INVALID_ARG
        with pytest.raises(A.AeAttnError) as ei:                     # dkey_gate without a key gate
            A.ae_gated_backward(h, q, k, v, la, 0, do, dq, dk, dv, dla, dkg, ws, need)
        assert ei.value.status == A.AE_ERR_INVALID_ARG
        with pytest.raises(A.AeAttnError):
            A.ae_gated_backward(None, *good, need)
    finally:
        A.ae_gated_destroy(h)
        A.ae_gated_destroy(hu)

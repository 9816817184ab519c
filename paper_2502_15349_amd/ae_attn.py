"""ctypes binding of libae_attn.so: argument marshalling only.

Names mirror the C ABI (include/ae_attn.h): ae_attn_create, ae_attn_forward,
ae_attn_destroy, ae_attn_query.  Every step of the attention path runs in the
HIP kernels; PyTorch supplies device memory and the stream, nothing else.
Importing this module fails if the library has not been built
(`python -m paper_2502_15349_amd.build`): there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libae_attn.so")
if not os.path.exists(_LIB_PATH):
    raise ImportError(
        f"{_LIB_PATH} is missing: build it with `python -m paper_2502_15349_amd.build` "
        "(the HIP library is the only implementation; there is no fallback)")
_lib = C.CDLL(_LIB_PATH)

AE_OK, AE_ERR_INVALID_ARG, AE_ERR_UNSUPPORTED, AE_ERR_HIP, AE_ERR_NOMEM = range(5)
SCORE_MODS = {"none": 0, "bias": 1, "head_decay": 2, "relu": 3, "bias_tensor": 4}
NORMS = {"softmax": 0, "sigmoid": 1, "abssum": 2, "abs_of_sum": 3, "none": 4}
MASKS = {"none": 0, "causal": 1, "sliding_window": 2}
OUT_DTYPES = {"f32": 0, "bf16": 1}


class ae_attn_desc_t(C.Structure):
    _fields_ = [
        ("B", C.c_int32), ("H_q", C.c_int32), ("H_kv", C.c_int32), ("L_q", C.c_int32),
        ("L_k", C.c_int32), ("D_qk", C.c_int32), ("D_v", C.c_int32),
        ("score_mod", C.c_int), ("bias", C.c_float), ("gamma", C.POINTER(C.c_float)),
        ("norm", C.c_int), ("mask", C.c_int), ("scale", C.c_float), ("out_dtype", C.c_int),
        ("window", C.c_int32), ("kv_splits", C.c_int32),
        ("q_stride", C.c_int64 * 3), ("k_stride", C.c_int64 * 3),
        ("v_stride", C.c_int64 * 3), ("o_stride", C.c_int64 * 3),
        ("bias_stride", C.c_int64 * 3),
    ]


_lib.ae_attn_create.argtypes = [C.POINTER(ae_attn_desc_t), C.POINTER(C.c_void_p)]
_lib.ae_attn_create.restype = C.c_int
_lib.ae_attn_forward.argtypes = [C.c_void_p] * 6
_lib.ae_attn_forward.restype = C.c_int
_lib.ae_attn_forward_stats.argtypes = [C.c_void_p] * 7
_lib.ae_attn_forward_stats.restype = C.c_int
_lib.ae_attn_forward_bias.argtypes = [C.c_void_p] * 8
_lib.ae_attn_forward_bias.restype = C.c_int
_lib.ae_attn_workspace_bytes.argtypes = [C.c_void_p, C.POINTER(C.c_size_t)]
_lib.ae_attn_workspace_bytes.restype = C.c_int
_lib.ae_attn_forward_split.argtypes = [C.c_void_p] * 7 + [C.c_size_t, C.c_void_p]
_lib.ae_attn_forward_split.restype = C.c_int
_lib.ae_attn_forward_split_static.argtypes = [C.c_void_p] * 7
_lib.ae_attn_forward_split_static.restype = C.c_int
_lib.ae_attn_backward_workspace_bytes.argtypes = [C.c_void_p, C.POINTER(C.c_size_t)]
_lib.ae_attn_backward_workspace_bytes.restype = C.c_int
_lib.ae_attn_backward.argtypes = [C.c_void_p] * 11 + [C.c_size_t, C.c_void_p]
_lib.ae_attn_backward.restype = C.c_int
_lib.ae_attn_backward_bias.argtypes = [C.c_void_p] * 12 + [C.c_int64, C.c_void_p, C.c_size_t, C.c_void_p]
_lib.ae_attn_backward_bias.restype = C.c_int


class ae_recurrent_desc_t(C.Structure):
    _fields_ = [("B", C.c_int32), ("H", C.c_int32), ("L", C.c_int32), ("D_qk", C.c_int32), ("D_v", C.c_int32),
                ("chunk", C.c_int32), ("scale", C.c_float), ("gamma", C.POINTER(C.c_float)), ("out_dtype", C.c_int)]


_lib.ae_recurrent_create.argtypes = [C.POINTER(ae_recurrent_desc_t), C.POINTER(C.c_void_p)]
_lib.ae_recurrent_create.restype = C.c_int
_lib.ae_recurrent_workspace_bytes.argtypes = [C.c_void_p, C.POINTER(C.c_size_t)]
_lib.ae_recurrent_workspace_bytes.restype = C.c_int
_lib.ae_recurrent_forward.argtypes = [C.c_void_p] * 6 + [C.c_size_t, C.c_void_p]
_lib.ae_recurrent_forward.restype = C.c_int
_lib.ae_recurrent_forward_state.argtypes = [C.c_void_p] * 8 + [C.c_size_t, C.c_void_p]
_lib.ae_recurrent_forward_state.restype = C.c_int
_lib.ae_recurrent_step.argtypes = [C.c_void_p] * 7
_lib.ae_recurrent_step.restype = C.c_int
_lib.ae_recurrent_destroy.argtypes = [C.c_void_p]
_lib.ae_recurrent_destroy.restype = C.c_int
_lib.ae_attn_destroy.argtypes = [C.c_void_p]
_lib.ae_attn_destroy.restype = C.c_int
_lib.ae_attn_query.argtypes = [C.c_void_p] + [C.POINTER(C.c_int32)] * 5
_lib.ae_attn_query.restype = C.c_int
_lib.ae_attn_kernel_name.argtypes = [C.c_void_p]
_lib.ae_attn_kernel_name.restype = C.c_char_p
_lib.ae_calib_mfma_bf16.argtypes = [C.c_void_p, C.c_size_t, C.c_int32, C.c_int32, C.POINTER(C.c_double), C.c_void_p]
_lib.ae_calib_mfma_bf16.restype = C.c_int
_lib.ae_attn_last_error.argtypes = []
_lib.ae_attn_last_error.restype = C.c_char_p
_lib.ae_attn_version.argtypes = []
_lib.ae_attn_version.restype = C.c_int32


class AeAttnError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"ae_attn status {status}: {message}")
        self.status = status


def ae_attn_last_error() -> str:
    return _lib.ae_attn_last_error().decode()


def ae_attn_version() -> int:
    return int(_lib.ae_attn_version())


def _check(status: int) -> None:
    if status != AE_OK:
        raise AeAttnError(status, ae_attn_last_error())


def ae_attn_create(*, B: int, H_q: int, H_kv: int, L_q: int, L_k: int, D_qk: int, D_v: int,
                   scale: float, score_mod="none", bias: float = 0.0,
                   gamma: Optional[Sequence[float]] = None, norm="softmax", mask="none",
                   q_stride=(0, 0, 0), k_stride=(0, 0, 0), v_stride=(0, 0, 0), o_stride=(0, 0, 0),
                   out_dtype="f32", window: int = 0, kv_splits: int = 0, bias_stride=(0, 0, 0)) -> int:
    """Returns an opaque handle (int).  Enum arguments accept names or raw ints."""
    d = ae_attn_desc_t()
    d.B, d.H_q, d.H_kv, d.L_q, d.L_k, d.D_qk, d.D_v = B, H_q, H_kv, L_q, L_k, D_qk, D_v
    d.score_mod = SCORE_MODS[score_mod] if isinstance(score_mod, str) else int(score_mod)
    d.norm = NORMS[norm] if isinstance(norm, str) else int(norm)
    d.mask = MASKS[mask] if isinstance(mask, str) else int(mask)
    d.bias, d.scale = float(bias), float(scale)
    d.out_dtype = OUT_DTYPES[out_dtype] if isinstance(out_dtype, str) else int(out_dtype)
    d.window = int(window)
    d.kv_splits = int(kv_splits)
    keep = None
    if gamma is not None:
        keep = (C.c_float * len(gamma))(*[float(x) for x in gamma])
        d.gamma = C.cast(keep, C.POINTER(C.c_float))
    for name, val in (("q_stride", q_stride), ("k_stride", k_stride), ("v_stride", v_stride), ("o_stride", o_stride),
                      ("bias_stride", bias_stride)):
        setattr(d, name, (C.c_int64 * 3)(*[int(x) for x in val]))
    h = C.c_void_p()
    _check(_lib.ae_attn_create(C.byref(d), C.byref(h)))
    return h.value


def ae_attn_workspace_bytes(handle: int) -> int:
    n = C.c_size_t(0)
    _check(_lib.ae_attn_workspace_bytes(handle, C.byref(n)))
    return int(n.value)


def ae_attn_forward_split(handle: int, Q: int, K: int, V: int, O: int, stats: int, workspace: int,
                          workspace_bytes: int, stream: int = 0) -> None:
    """Forward of a handle created with kv_splits > 1; stats may be 0 (not written)."""
    _check(_lib.ae_attn_forward_split(handle, Q, K, V, O, stats, workspace, workspace_bytes, stream))


def ae_attn_forward_split_static(handle: int, Q: int, K: int, V: int, O: int, stats: int = 0, stream: int = 0) -> None:
    """ae_attn_forward_split with the partial results in the library's static device scratch (no workspace, no allocation)."""
    _check(_lib.ae_attn_forward_split_static(handle, Q, K, V, O, stats, stream))


AE_ATTN_STATIC_SCRATCH_BYTES = 4 << 20


def ae_attn_backward_workspace_bytes(handle: int) -> int:
    """Bytes of device workspace ae_attn_backward needs for this handle."""
    n = C.c_size_t(0)
    _check(_lib.ae_attn_backward_workspace_bytes(handle, C.byref(n)))
    return int(n.value)


def ae_attn_backward(handle: int, Q: int, K: int, V: int, O: int, dO: int, stats: int, dQ: int, dK: int, dV: int,
                     workspace: int, workspace_bytes: int, stream: int = 0) -> None:
    """Device addresses throughout: dQ, dK, dV (fp32, contiguous) receive the gradients for the upstream
    gradient dO (bf16, contiguous); O and stats are what ae_attn_forward_stats wrote."""
    _check(_lib.ae_attn_backward(handle, Q, K, V, O, dO, stats, dQ, dK, dV, workspace, workspace_bytes, stream))


def ae_attn_backward_bias(handle: int, Q: int, K: int, V: int, bias: int, O: int, dO: int, stats: int, dQ: int, dK: int,
                          dV: int, dBias: int, dbias_row_stride: int, workspace: int, workspace_bytes: int,
                          stream: int = 0) -> None:
    """ae_attn_backward for a handle created with score_mod "bias_tensor" (bias: device address of the tensor; dBias:
    0, or the address of a zero-filled bf16 buffer [B, H_q, L_q, dbias_row_stride] for the bias gradient)."""
    _check(_lib.ae_attn_backward_bias(handle, Q, K, V, bias, O, dO, stats, dQ, dK, dV, dBias, dbias_row_stride, workspace,
                                      workspace_bytes, stream))


def ae_attn_forward_bias(handle: int, Q: int, K: int, V: int, bias: int, O: int, stats: int = 0, stream: int = 0) -> None:
    """Forward of a handle created with score_mod "bias_tensor"; bias is the device address of the bf16 bias tensor,
    stats may be 0 (not written)."""
    _check(_lib.ae_attn_forward_bias(handle, Q, K, V, bias, O, stats, stream))


def ae_attn_forward_stats(handle: int, Q: int, K: int, V: int, O: int, stats: int, stream: int = 0) -> None:
    """ae_attn_forward that also writes the row statistic (fp32 [B, H_q, L_q]) to `stats`."""
    _check(_lib.ae_attn_forward_stats(handle, Q, K, V, O, stats, stream))


def ae_attn_forward(handle: int, Q: int, K: int, V: int, O: int, stream: int = 0) -> None:
    """Q, K, V, O are device addresses (tensor.data_ptr()); stream is a raw hipStream_t."""
    _check(_lib.ae_attn_forward(handle, Q, K, V, O, stream))


def ae_calib_mfma_bf16(sink: int, sink_bytes: int, workgroups: int, iters: int, stream: int = 0) -> float:
    """Enqueues the pure-MFMA calibration kernel; returns the flop it performs."""
    flop = C.c_double(0.0)
    _check(_lib.ae_calib_mfma_bf16(sink, sink_bytes, workgroups, iters, C.byref(flop), stream))
    return float(flop.value)


def ae_attn_destroy(handle: Optional[int]) -> None:
    _check(_lib.ae_attn_destroy(handle))


def ae_attn_query(handle: int) -> dict:
    v = [C.c_int32() for _ in range(5)]
    _check(_lib.ae_attn_query(handle, *[C.byref(x) for x in v]))
    keys = ("block_m", "block_n", "lds_bytes", "grid_size", "block_threads")
    out = {k: int(x.value) for k, x in zip(keys, v)}
    out["kernel"] = _lib.ae_attn_kernel_name(handle).decode()
    return out


# ---- convenience for torch callers (still marshalling only) -------------------
def ae_recurrent_create(*, B: int, H: int, L: int, D_qk: int, D_v: int, chunk: int, scale: float,
                        gamma: Optional[Sequence[float]], out_dtype="f32") -> int:
    """Handle for chunk-parallel recurrent retention (h_t = gamma h_{t-1} + k_t^T v_t, o_t = scale q_t h_t)."""
    d = ae_recurrent_desc_t(B=B, H=H, L=L, D_qk=D_qk, D_v=D_v, chunk=chunk, scale=scale,
                            out_dtype=OUT_DTYPES[out_dtype] if isinstance(out_dtype, str) else int(out_dtype))
    keep = None
    if gamma is not None:
        keep = (C.c_float * len(gamma))(*[float(g) for g in gamma])
        d.gamma = C.cast(keep, C.POINTER(C.c_float))
    out = C.c_void_p()
    _check(_lib.ae_recurrent_create(C.byref(d), C.byref(out)))
    return out.value


def ae_recurrent_workspace_bytes(handle: int) -> int:
    n = C.c_size_t()
    _check(_lib.ae_recurrent_workspace_bytes(handle, C.byref(n)))
    return n.value


def ae_recurrent_forward(handle: int, Q: int, K: int, V: int, O: int, workspace: int, workspace_bytes: int,
                         stream: int = 0) -> None:
    _check(_lib.ae_recurrent_forward(handle, Q, K, V, O, workspace, workspace_bytes, stream))


def ae_recurrent_forward_state(handle: int, Q: int, K: int, V: int, h_in: int, O: int, h_out: int, workspace: int,
                               workspace_bytes: int, stream: int = 0) -> None:
    """ae_recurrent_forward with the state in front of the first token (h_in, 0: zero) and the state after the last
    one (h_out, 0: not computed), both fp32 [B, H, D_qk, D_v] device addresses."""
    _check(_lib.ae_recurrent_forward_state(handle, Q, K, V, h_in, O, h_out, workspace, workspace_bytes, stream))


def ae_recurrent_step(handle: int, q: int, k: int, v: int, state: int, o: int, stream: int = 0) -> None:
    """One token: state <- gamma state + k^T v (fp32 [B, H, D_qk, D_v], in place), o = scale q state (fp32 [B, H, D_v])."""
    _check(_lib.ae_recurrent_step(handle, q, k, v, state, o, stream))


def ae_recurrent_destroy(handle: Optional[int]) -> None:
    _check(_lib.ae_recurrent_destroy(handle))


def retention_recurrent(Q, K, V, *, scale, gamma, chunk=256, out=None, workspace=None, stream=None, h_in=None,
                        return_state=False, out_dtype=None):
    """Recurrent retention on contiguous bf16 device tensors Q, K [B, H, L, D_qk], V [B, H, L, D_v];
    returns O [B, H, L, D_v] fp32 (bf16 with out_dtype=torch.bfloat16 or a bf16 `out`).  workspace: device byte tensor of ae_recurrent_workspace_bytes() bytes
    (allocated here if not given).  h_in: optional contiguous fp32 device tensor [B, H, D_qk, D_v], the state in
    front of the first token; return_state: also return the state after the last token (same layout)."""
    import torch

    for t in (Q, K, V):
        if not t.is_cuda or t.dtype != torch.bfloat16 or t.dim() != 4 or not t.is_contiguous():
            raise ValueError("Q, K, V must be contiguous 4-D bf16 device tensors; there is no CPU path")
    B, H, L, D_qk = Q.shape
    D_v = V.shape[3]
    if K.shape != Q.shape or V.shape[:3] != Q.shape[:3]:
        raise ValueError("K / V shape does not match Q")
    if out is None:
        out = torch.empty((B, H, L, D_v), dtype=out_dtype or torch.float32, device=Q.device)
    if out.dtype not in (torch.float32, torch.bfloat16) or tuple(out.shape) != (B, H, L, D_v) or not out.is_contiguous():
        raise ValueError("O must be a contiguous fp32 or bf16 tensor [B, H, L, D_v]")
    h = ae_recurrent_create(B=B, H=H, L=L, D_qk=D_qk, D_v=D_v, chunk=chunk, scale=scale, gamma=gamma,
                            out_dtype="bf16" if out.dtype == torch.bfloat16 else "f32")
    try:
        s = torch.cuda.current_stream(Q.device) if stream is None else stream
        with torch.cuda.device(Q.device):
            need = ae_recurrent_workspace_bytes(h)
            if workspace is None:
                workspace = torch.empty(need, dtype=torch.uint8, device=Q.device)
            if h_in is not None and (h_in.dtype != torch.float32 or tuple(h_in.shape) != (B, H, D_qk, D_v)
                                     or not h_in.is_contiguous() or not h_in.is_cuda):
                raise ValueError("h_in must be a contiguous fp32 device tensor [B, H, D_qk, D_v]")
            h_out = torch.empty((B, H, D_qk, D_v), dtype=torch.float32, device=Q.device) if return_state else None
            ae_recurrent_forward_state(h, Q.data_ptr(), K.data_ptr(), V.data_ptr(), 0 if h_in is None else h_in.data_ptr(),
                                       out.data_ptr(), 0 if h_out is None else h_out.data_ptr(), workspace.data_ptr(),
                                       workspace.numel(), s.cuda_stream)
    finally:
        ae_recurrent_destroy(h)
    return (out, h_out) if return_state else out


def attention_forward(Q, K, V, *, scale, score_mod="none", bias=0.0, gamma=None, norm="softmax",
                      mask="none", out=None, stream=None, out_dtype=None, stats=None, window=0, kv_splits=0,
                      workspace=None, bias_tensor=None):
    """Runs the HIP operator on CUDA/HIP bf16 tensors laid out [B, H, L, D]
    (last dim contiguous) and returns O [B, H_q, L_q, D_v]: fp32, or bf16 if `out` is a
    bf16 tensor or out_dtype is torch.bfloat16.  stats: optional contiguous fp32 device
    tensor [B, H_q, L_q] that receives the row statistic of the normalization.  window: keys
    per query for mask="sliding_window".  kv_splits > 1: the keys are cut into that many ranges
    (few query rows, many keys); `workspace` is then a device byte tensor of at least
    ae_attn_workspace_bytes() bytes (allocated here if not given).  bias_tensor: for score_mod
    "bias_tensor", a bf16 device tensor [B or 1, H_q or 1, L_q, L_k] (last dimension contiguous)."""
    import torch

    if not (Q.is_cuda and K.is_cuda and V.is_cuda):
        raise ValueError("attention_forward needs device tensors; there is no CPU path")
    for t in (Q, K, V):
        if t.dtype != torch.bfloat16 or t.dim() != 4 or t.stride(3) != 1:
            raise ValueError("Q, K, V must be 4-D bf16 with a contiguous last dimension")
    B, H_q, L_q, D_qk = Q.shape
    _, H_kv, L_k, D_v = V.shape
    if K.shape != (B, H_kv, L_k, D_qk):
        raise ValueError("K shape does not match Q / V")
    if out is None:
        out = torch.empty((B, H_q, L_q, D_v), dtype=out_dtype or torch.float32, device=Q.device)
    if out.dtype not in (torch.float32, torch.bfloat16) or out.stride(3) != 1:
        raise ValueError("O must be fp32 or bf16 with a contiguous last dimension")
    h = ae_attn_create(B=B, H_q=H_q, H_kv=H_kv, L_q=L_q, L_k=L_k, D_qk=D_qk, D_v=D_v, scale=scale,
                       score_mod=score_mod, bias=bias, gamma=gamma, norm=norm, mask=mask,
                       q_stride=Q.stride()[:3], k_stride=K.stride()[:3], v_stride=V.stride()[:3],
                       o_stride=out.stride()[:3], out_dtype="bf16" if out.dtype == torch.bfloat16 else "f32",
                       window=window, kv_splits=kv_splits, bias_stride=_bias_strides(bias_tensor, B, H_q, L_q, L_k))
    try:
        s = torch.cuda.current_stream(Q.device) if stream is None else stream
        with torch.cuda.device(Q.device):
            if stats is not None and (stats.dtype != torch.float32 or tuple(stats.shape) != (B, H_q, L_q)
                                      or not stats.is_contiguous()):
                raise ValueError("stats must be a contiguous fp32 tensor [B, H_q, L_q]")
            need = ae_attn_workspace_bytes(h)
            if bias_tensor is not None:
                ae_attn_forward_bias(h, Q.data_ptr(), K.data_ptr(), V.data_ptr(), bias_tensor.data_ptr(), out.data_ptr(),
                                     0 if stats is None else stats.data_ptr(), s.cuda_stream)
            elif need:
                if workspace is None:
                    workspace = torch.empty(need, dtype=torch.uint8, device=Q.device)
                ae_attn_forward_split(h, Q.data_ptr(), K.data_ptr(), V.data_ptr(), out.data_ptr(),
                                      0 if stats is None else stats.data_ptr(), workspace.data_ptr(),
                                      workspace.numel() * workspace.element_size(), s.cuda_stream)
            elif stats is None:
                ae_attn_forward(h, Q.data_ptr(), K.data_ptr(), V.data_ptr(), out.data_ptr(), s.cuda_stream)
            else:
                if stats.dtype != torch.float32 or tuple(stats.shape) != (B, H_q, L_q) or not stats.is_contiguous():
                    raise ValueError("stats must be a contiguous fp32 tensor [B, H_q, L_q]")
                ae_attn_forward_stats(h, Q.data_ptr(), K.data_ptr(), V.data_ptr(), out.data_ptr(), stats.data_ptr(),
                                      s.cuda_stream)
    finally:
        ae_attn_destroy(h)
    return out


def _bias_strides(bias_tensor, B, H_q, L_q, L_k):
    """Element strides {batch, head, row} of a bias tensor [B or 1, H_q or 1, L_q, L_k]; a dimension of size 1 is
    shared (stride 0)."""
    if bias_tensor is None:
        return (0, 0, 0)
    import torch
    t = bias_tensor
    if (t.dtype != torch.bfloat16 or t.dim() != 4 or t.shape[0] not in (1, B) or t.shape[1] not in (1, H_q)
            or tuple(t.shape[2:]) != (L_q, L_k) or t.stride(3) != 1 or not t.is_cuda):
        raise ValueError("bias_tensor must be a bf16 device tensor [B or 1, H_q or 1, L_q, L_k] with a contiguous last dimension")
    return (0 if t.shape[0] == 1 else t.stride(0), 0 if t.shape[1] == 1 else t.stride(1), t.stride(2))


def attention_backward(Q, K, V, O, dO, stats, *, scale, score_mod="none", bias=0.0, gamma=None, norm="softmax",
                       mask="none", window=0, stream=None, workspace=None, bias_tensor=None, want_dbias=False):
    """Runs the HIP backward pass on device tensors: Q, K, V bf16 [B, H, L, D] (last dim contiguous), O the
    forward output (fp32 or bf16), dO bf16 contiguous, stats the fp32 row statistic of the forward pass (O and
    stats may be None for sigmoid and no normalization); window: keys per query for mask="sliding_window".  Returns (dQ, dK, dV)
    as contiguous fp32 tensors; with want_dbias also the bias gradient, bf16 [B, H_q, L_q, L_k] (per batch and head)."""
    import torch

    if not (Q.is_cuda and K.is_cuda and V.is_cuda and dO.is_cuda):
        raise ValueError("attention_backward needs device tensors; there is no CPU path")
    B, H_q, L_q, D_qk = Q.shape
    _, H_kv, L_k, D_v = V.shape
    if dO.dtype != torch.bfloat16 or tuple(dO.shape) != (B, H_q, L_q, D_v) or not dO.is_contiguous():
        raise ValueError("dO must be a contiguous bf16 tensor [B, H_q, L_q, D_v]")
    if stats is not None and (stats.dtype != torch.float32 or tuple(stats.shape) != (B, H_q, L_q) or not stats.is_contiguous()):
        raise ValueError("stats must be a contiguous fp32 tensor [B, H_q, L_q]")
    o_dtype, o_stride = ("f32", (0, 0, 0)) if O is None else ("bf16" if O.dtype == torch.bfloat16 else "f32", O.stride()[:3])
    h = ae_attn_create(B=B, H_q=H_q, H_kv=H_kv, L_q=L_q, L_k=L_k, D_qk=D_qk, D_v=D_v, scale=scale,
                       score_mod=score_mod, bias=bias, gamma=gamma, norm=norm, mask=mask, q_stride=Q.stride()[:3],
                       k_stride=K.stride()[:3], v_stride=V.stride()[:3], o_stride=o_stride, out_dtype=o_dtype,
                       window=window, bias_stride=_bias_strides(bias_tensor, B, H_q, L_q, L_k))
    try:
        s = torch.cuda.current_stream(Q.device) if stream is None else stream
        with torch.cuda.device(Q.device):
            dQ = torch.empty((B, H_q, L_q, D_qk), dtype=torch.float32, device=Q.device)
            dK = torch.empty((B, H_kv, L_k, D_qk), dtype=torch.float32, device=Q.device)
            dV = torch.empty((B, H_kv, L_k, D_v), dtype=torch.float32, device=Q.device)
            need = ae_attn_backward_workspace_bytes(h)
            if workspace is None:
                workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=Q.device)
            tail = (0 if O is None else O.data_ptr(), dO.data_ptr(), 0 if stats is None else stats.data_ptr(), dQ.data_ptr(),
                    dK.data_ptr(), dV.data_ptr(), workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                    s.cuda_stream)
            dB = None
            if bias_tensor is not None:
                ld = (L_k + 3) // 4 * 4
                if want_dbias:
                    dB = torch.zeros((B, H_q, L_q, ld), dtype=torch.bfloat16, device=Q.device)
                ae_attn_backward_bias(h, Q.data_ptr(), K.data_ptr(), V.data_ptr(), bias_tensor.data_ptr(), *tail[:6],
                                      0 if dB is None else dB.data_ptr(), ld, *tail[6:])
            else:
                ae_attn_backward(h, Q.data_ptr(), K.data_ptr(), V.data_ptr(), *tail)
    finally:
        ae_attn_destroy(h)
    if want_dbias:
        return dQ, dK, dV, dB[..., :L_k]
    return dQ, dK, dV


def run_workload(w, Q, K, V, out=None, out_dtype=None, stats=None, kv_splits=0, bias_tensor=None):
    """attention_forward with the parameters of a workloads.Workload."""
    return attention_forward(Q, K, V, scale=w.scale_value, score_mod=w.score_mod, bias=w.bias,
                             gamma=w.gamma(), norm=w.norm, mask=w.mask, out=out, out_dtype=out_dtype, stats=stats,
                             window=w.window, kv_splits=kv_splits, bias_tensor=bias_tensor)


# ---- recurrent pattern with per-token gates (gated retention, Mamba2 SSM) ------------------------------------
class ae_gated_desc_t(C.Structure):
    _fields_ = [("B", C.c_int32), ("H", C.c_int32), ("H_qk", C.c_int32), ("L", C.c_int32), ("D_qk", C.c_int32),
                ("D_v", C.c_int32), ("scale", C.c_float), ("out_dtype", C.c_int)]


_lib.ae_gated_create.argtypes = [C.POINTER(ae_gated_desc_t), C.POINTER(C.c_void_p)]
_lib.ae_gated_create.restype = C.c_int
_lib.ae_gated_forward.argtypes = [C.c_void_p] * 10
_lib.ae_gated_forward.restype = C.c_int
_lib.ae_gated_destroy.argtypes = [C.c_void_p]
_lib.ae_gated_destroy.restype = C.c_int
_lib.ae_gated_workspace_bytes.argtypes = [C.c_void_p, C.POINTER(C.c_size_t)]
_lib.ae_gated_workspace_bytes.restype = C.c_int
_lib.ae_gated_forward_segmented.argtypes = [C.c_void_p] * 10 + [C.c_size_t, C.c_void_p]
_lib.ae_gated_forward_segmented.restype = C.c_int
_lib.ae_gated_backward_workspace_bytes.argtypes = [C.c_void_p, C.POINTER(C.c_size_t)]
_lib.ae_gated_backward_workspace_bytes.restype = C.c_int
_lib.ae_gated_backward.argtypes = [C.c_void_p] * 13 + [C.c_size_t, C.c_void_p]
_lib.ae_gated_backward.restype = C.c_int


def ae_gated_create(*, B: int, H: int, L: int, D_qk: int, D_v: int, scale: float, H_qk: Optional[int] = None,
                    out_dtype="f32") -> int:
    d = ae_gated_desc_t()
    d.B, d.H, d.H_qk, d.L, d.D_qk, d.D_v = B, H, H if H_qk is None else H_qk, L, D_qk, D_v
    d.scale = float(scale)
    d.out_dtype = OUT_DTYPES[out_dtype] if isinstance(out_dtype, str) else int(out_dtype)
    h = C.c_void_p()
    _check(_lib.ae_gated_create(C.byref(d), C.byref(h)))
    return h.value


def ae_gated_forward(handle: int, Q: int, K: int, V: int, log_decay: int, key_gate: int, h_in: int, O: int, h_out: int,
                     stream: int = 0) -> None:
    """Device pointers as ints; key_gate, h_in, h_out may be 0."""
    _check(_lib.ae_gated_forward(handle, Q, K, V, log_decay, key_gate, h_in, O, h_out, stream))


def ae_gated_destroy(handle: Optional[int]) -> None:
    _check(_lib.ae_gated_destroy(handle))


def ae_gated_workspace_bytes(handle: int) -> int:
    n = C.c_size_t()
    _check(_lib.ae_gated_workspace_bytes(handle, C.byref(n)))
    return n.value


def ae_gated_forward_segmented(handle: int, Q: int, K: int, V: int, log_decay: int, key_gate: int, h_in: int, O: int, h_out: int,
                               workspace: int, workspace_bytes: int, stream: int = 0) -> None:
    _check(_lib.ae_gated_forward_segmented(handle, Q, K, V, log_decay, key_gate, h_in, O, h_out, workspace, workspace_bytes, stream))


def ae_gated_backward_workspace_bytes(handle: int) -> int:
    n = C.c_size_t()
    _check(_lib.ae_gated_backward_workspace_bytes(handle, C.byref(n)))
    return n.value


def ae_gated_backward(handle: int, Q: int, K: int, V: int, log_decay: int, key_gate: int, dO: int, dQ: int, dK: int, dV: int,
                      dlog_decay: int, dkey_gate: int, workspace: int, workspace_bytes: int, stream: int = 0) -> None:
    """Device pointers as ints; key_gate and dkey_gate are 0 together."""
    _check(_lib.ae_gated_backward(handle, Q, K, V, log_decay, key_gate, dO, dQ, dK, dV, dlog_decay, dkey_gate, workspace,
                                  workspace_bytes, stream))


def gated_recurrent(Q, K, V, log_decay, key_gate=None, *, scale, h_in=None, want_state=False, out_dtype=None, stream=None,
                    segmented=False):
    """Runs the gated recurrent pattern on device tensors: Q, K bf16 [B, H_qk, L, D_qk], V bf16 [B, H, L, D_v],
    log_decay / key_gate fp32 [B, H, L] (all contiguous), h_in fp32 [B, H, D_qk, D_v] or None.  Returns O
    [B, H, L, D_v] (fp32, or bf16 with out_dtype=torch.bfloat16), and the final state when want_state.  segmented: through
    ae_gated_forward_segmented (the walks cut into segments where few heads meet a long sequence)."""
    import torch

    for t in (Q, K, V, log_decay) + (() if key_gate is None else (key_gate,)) + (() if h_in is None else (h_in,)):
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError("gated_recurrent needs contiguous device tensors; there is no CPU path")
    B, H_qk, L, D_qk = Q.shape
    _, H, _, D_v = V.shape
    out = torch.empty((B, H, L, D_v), dtype=out_dtype or torch.float32, device=Q.device)
    h_out = torch.empty((B, H, D_qk, D_v), dtype=torch.float32, device=Q.device) if want_state else None
    h = ae_gated_create(B=B, H=H, H_qk=H_qk, L=L, D_qk=D_qk, D_v=D_v, scale=scale,
                        out_dtype="bf16" if out.dtype == torch.bfloat16 else "f32")
    try:
        s = torch.cuda.current_stream(Q.device) if stream is None else stream
        nbytes = ae_gated_workspace_bytes(h) if segmented else 0
        ws = torch.empty(nbytes, dtype=torch.uint8, device=Q.device) if nbytes else None
        with torch.cuda.device(Q.device):
            args = (h, Q.data_ptr(), K.data_ptr(), V.data_ptr(), log_decay.data_ptr(),
                    0 if key_gate is None else key_gate.data_ptr(), 0 if h_in is None else h_in.data_ptr(),
                    out.data_ptr(), 0 if h_out is None else h_out.data_ptr())
            if segmented:
                ae_gated_forward_segmented(*args, 0 if ws is None else ws.data_ptr(), nbytes, s.cuda_stream)
            else:
                ae_gated_forward(*args, s.cuda_stream)
    finally:
        ae_gated_destroy(h)
    return (out, h_out) if want_state else out


def gated_recurrent_backward(Q, K, V, log_decay, key_gate, dO, *, scale, stream=None):
    """Backward pass of gated_recurrent on device tensors (layouts as there, dO bf16 [B, H, L, D_v], contiguous).
    Returns (dQ, dK, dV, dlog_decay, dkey_gate or None), all fp32; dQ and dK have the shape of Q."""
    import torch

    for t in (Q, K, V, log_decay, dO) + (() if key_gate is None else (key_gate,)):
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError("gated_recurrent_backward needs contiguous device tensors; there is no CPU path")
    B, H_qk, L, D_qk = Q.shape
    _, H, _, D_v = V.shape
    f32 = dict(dtype=torch.float32, device=Q.device)
    dQ, dK, dV = torch.empty(Q.shape, **f32), torch.empty(K.shape, **f32), torch.empty(V.shape, **f32)
    dla = torch.empty((B, H, L), **f32)
    dkg = None if key_gate is None else torch.empty((B, H, L), **f32)
    h = ae_gated_create(B=B, H=H, H_qk=H_qk, L=L, D_qk=D_qk, D_v=D_v, scale=scale)
    try:
        nbytes = ae_gated_backward_workspace_bytes(h)
        ws = torch.empty(nbytes, dtype=torch.uint8, device=Q.device)
        s = torch.cuda.current_stream(Q.device) if stream is None else stream
        with torch.cuda.device(Q.device):
            ae_gated_backward(h, Q.data_ptr(), K.data_ptr(), V.data_ptr(), log_decay.data_ptr(),
                              0 if key_gate is None else key_gate.data_ptr(), dO.data_ptr(), dQ.data_ptr(), dK.data_ptr(),
                              dV.data_ptr(), dla.data_ptr(), 0 if dkg is None else dkg.data_ptr(), ws.data_ptr(), nbytes,
                              s.cuda_stream)
    finally:
        ae_gated_destroy(h)
    return dQ, dK, dV, dla, dkg

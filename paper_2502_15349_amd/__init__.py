"""MI355X-native fused parallel-pattern attention (forward).

`workloads` (synthetic input recipes) is importable anywhere.  The operator
itself lives in `paper_2502_15349_amd.ae_attn`, which loads the in-tree HIP
library `libae_attn.so` on import and raises if it has not been built: there
is no CPU or PyTorch fallback.
"""
__all__ = ["workloads"]

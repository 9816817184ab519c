"""CPU oracle for the fused parallel-pattern attention path (forward, and its backward pass).

TEST INFRASTRUCTURE ONLY.  Nothing in the product package may import this
package; only tests/, __graft_entry__.smoke() and the cpu_baseline leg of
bench.py do.  It shares no code with the HIP kernels or their Python binding.
"""
from .attention_backward_oracle import attention_backward, attention_backward_head  # noqa: F401
from .attention_oracle import (  # noqa: F401
    attention,
    attention_head,
    brute,
    row_stats_head,
    weights_head,
)

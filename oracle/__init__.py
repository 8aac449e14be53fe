"""CPU oracle for the RADAR hot path -- TEST INFRASTRUCTURE, not the product.

Only ``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s cpu_baseline leg
may import this package.  It wraps ``radar_oracle.c`` (plain C, fp64 arithmetic)
with ctypes and takes / returns numpy arrays.  It imports nothing from the HIP
package.
"""
from .radar_oracle import (  # noqa: F401
    build,
    sanitizer_runtime,
    num_threads,
    set_threads,
    round_bf16,
    tree_attention,
    draft_expand,
    draft_rerank,
    verify_accept,
    accept_length_distribution,
    accept_margins,
    policy_step,
    verify_accept_q,
    OracleError,
)

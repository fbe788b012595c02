"""fp64 CPU oracle for sliced causal attention (test infrastructure only).

Nothing in the product package may import this; only tests, the smoke check and
the CPU-baseline leg of the benchmark use it.
"""
from .slimpipe_oracle import attn_fwd, attn_bwd, attn_merge  # noqa: F401

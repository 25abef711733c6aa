"""CPU oracle for the SparseK attention hot path -- TEST INFRASTRUCTURE ONLY.

A thin numpy/ctypes face over ``sparsek_oracle.c`` (plain C, fp64, written from the
paper's definitions).  Nothing in the product package imports this; only the tests,
the smoke check and the benchmark's ``cpu_baseline`` leg do.  It shares no code with
the HIP library.
"""
from .ref import (  # noqa: F401
    build,
    sparsek,
    tau_prefixes,
    select_prefix,
    death,
    attn_query_bydef,
    attn_rows,
    attn_fwd,
    mask_bwd,
    attn_bwd,
    mask_all,
    decode_bydef,
    tau_incremental,
    decode_incremental,
    max_threads,
    scores,
)

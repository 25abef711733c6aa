"""SparseK attention hot path for MI355X: thin Python binding over libsparsek (C ABI).

All computation happens in the HIP library; this package only marshals arguments.
torch is used for device memory and streams.  There is no CPU fallback: if the
library has not been built, every call raises.
"""
from .binding import (  # noqa: F401
    SparsekCfg,
    SparsekDecodeCfg,
    DecodeState,
    lib,
    lib_path,
    check,
    sparsek_mask,
    sparsek_mask_workspace,
    sparsek_mask_status,
    sparsek_mask_static,
    sparsek_materialize,
    sparsek_attn_fwd,
    sparsek_mask_bwd,
    sparsek_attn_bwd,
    sparsek_bwd,
    sparsek_scores,
    ChunkState,
    sparsek_chunk_prefill,
    sparsek_chunk_bwd,
    sparsek_chunk_status,
    sparsek_chunk_to_decode,
    sparsek_decode_init,
    sparsek_decode_load,
    sparsek_decode_step,
    sparsek_decode_status,
    F32,
    BF16,
)

"""fea: paged decode attention over prefix-aliased KV blocks on MI355X (gfx950).

Thin ctypes binding of libfea.so (see include/fea.h).  Every step of the path -
chunk hashing, block-table construction, alias detection, the KV sweep and the
merge - runs inside the library; this package only marshals arguments.  There is
no fallback: if the library is not built, importing the binding functions fails.
"""
from .fea import (  # noqa: F401
    FEA_DTYPE_BF16, FEA_DTYPE_F32, FEA_FLAG_REUSE_PLAN, FEA_FLAG_PLAN_ONLY, FEA_FLAG_REFRESH_PLAN, FeaError, KVPool, AttnParams,
    fea_build_block_tables, fea_chunk_hashes, fea_decode_attention, fea_decode_plan_info,
    fea_decode_workspace_bytes, fea_kv_alloc, fea_kv_free, fea_kv_stats, fea_release,
    fea_validate_block_tables, fea_profile_enable, fea_profile_read, library_path, load_library,
    Cht, StopPolicy, fea_kv_extend, fea_kv_append, Policy, PolicyParams,
    FEA_ADD, FEA_STOP, FEA_POLICY_UCB, FEA_POLICY_QLEARN, FEA_HASH_CHAINED, FEA_HASH_XXH64,
    fea_chunk_hashes_xxh64, fea_kv_set_hash, fea_chunk_hashes_device, fea_decode_attention_static, fea_stream_read_gbs,
)

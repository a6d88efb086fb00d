"""libquoka: QuoKA chunk-prefill sparse attention on one AMD MI355X (HIP kernels behind a C ABI)."""
from .binding import (  # noqa: F401
    QuokaError,
    QuokaShape,
    QUOKA_F32,
    QUOKA_BF16,
    load_library,
    library_path,
    make_shape,
    quoka_workspace_bytes,
    quoka_select_queries,
    quoka_score_keys,
    quoka_topk_keys,
    quoka_sparse_attn,
    quoka_dense_attn,
    quoka_chunk_attn,
    quoka_version,
    ChunkBuffers,
)

"""MI355X-native rolling-KV-cache chunk attention (hand-written HIP behind a C ABI)."""
from .binding import (  # noqa: F401
    ASTRO_BF16,
    ASTRO_F32,
    AstroError,
    KVCache,
    astro_chunk_attn_bwd,
    astro_chunk_attn_fwd,
    astro_chunk_attn_workspace_bytes,
    astro_kvcache_append,
    astro_kvcache_bytes,
    astro_kvcache_create,
    astro_kvcache_destroy,
    astro_kvcache_reset,
    astro_kvcache_tables,
    astro_strerror,
    make_desc,
)

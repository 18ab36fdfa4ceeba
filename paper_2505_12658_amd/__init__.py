"""MI355X-native packed variable-length attention, paged KV-cache write and attention over the paged cache (gfx950 HIP kernels
behind a C ABI; this package is only the thin Python binding)."""
from .binding import (  # noqa: F401
    HydraError,
    hydra_attn_build_worklist,
    hydra_attn_paged_fwd,
    hydra_attn_paged_workspace_bytes,
    hydra_attn_varlen_fwd,
    hydra_attn_varlen_fwd_prebuilt,
    hydra_attn_varlen_fwd_shared,
    hydra_attn_varlen_fwd_static,
    hydra_attn_workspace_bytes,
    hydra_kv_cache_write,
    hydra_page_cache_gather,
    hydra_page_cache_write,
    hydra_status_string,
    library_path,
    load_library,
)

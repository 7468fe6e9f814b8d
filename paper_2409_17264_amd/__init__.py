"""MI355X-native paged attention for chunked prefill, split-KV decode and the
log-sum-exp merge of KV-cache parallelism (hand-written HIP behind a C ABI).

The Python layer only marshals arguments; every step runs in the HIP library.
The library is loaded on first use and a missing library is an error.
"""
from .binding import (  # noqa: F401
    MedhaError,
    chunk_partial_attn,
    chunk_partial_workspace_bytes,
    chunked_prefill_attn,
    chunked_prefill_attn_noalloc,
    chunked_prefill_workspace_bytes,
    decode_partial_attn,
    decode_partial_workspace_bytes,
    describe_plan,
    describe_slot,
    kv_append,
    library_path,
    load_library,
    lse_merge,
)

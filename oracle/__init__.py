"""CPU oracle for the paged KV-cache data path (test infrastructure only).

Only the tests, the smoke check and the bench's CPU-baseline leg may import
this package; the product package never does.
"""
from .kv_oracle import (  # noqa: F401
    OracleError,
    append_packed,
    append_tokens,
    bitmap_words,
    build,
    collect_dirty,
    decode_attn,
    gather_tokens,
    pack_blocks,
    prefill_attn,
    restore_blocks,
)

"""Float64 CPU checker (test infrastructure only; never imported by the product path)."""
from .attention import (E4M3FN_TABLE, attn_partial_dense, attn_partial_paged, decode_bf16, decode_elems,  # noqa: F401
                        decode_q, gather_kv, local_partials, merge, merge_requests, remote_partials,
                        request_full_attention)

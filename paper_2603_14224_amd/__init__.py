"""Self-Indexing KV cache decode path for AMD MI355X (gfx950): Python binding of libsik.so."""
from .binding import (EXPORTS, SIK_BF16, SIK_F16, SIK_F32, SIK_Q_ENCODE, SIK_Q_FIT, Layout, SikError,  # noqa: F401
                      alloc_kvq, alloc_workspace, lib, make_layout, sik_kvq_bytes, sik_quantize_kv, sik_sparse_attn_q2, sik_decode_step_q2, sik_decode_step_ex, DecodeArgs, sik_decode_step, sik_decode_step_profiled, sik_quantize_keys, sik_score,
                      sik_sparse_attn, sik_strerror, sik_topk, sik_workspace_bytes)

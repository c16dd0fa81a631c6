"""Self-Indexing KV cache decode path for AMD MI355X (gfx950): Python binding of libsik.so."""
from .binding import (EXPORTS, SIK_BF16, SIK_F16, SIK_F32, SIK_Q_ENCODE, SIK_Q_FIT, DecodeArgs, Layout,  # noqa: F401
                      SikError, alloc_kvq, alloc_workspace, lib, make_layout, sik_decode_step, sik_decode_step_ex,
                      sik_decode_step_profiled, sik_decode_step_q2, sik_decode_step_static, SIK_STATIC_SCRATCH_BYTES, sik_kvq_bytes, sik_plan_info, sik_prefill_compress, sik_quantize_keys,
                      sik_quantize_kv, sik_score, sik_sparse_attn, sik_sparse_attn_q2, sik_strerror, sik_topk,
                      sik_workspace_bytes, sik_workspace_init, sik_workspace_status)

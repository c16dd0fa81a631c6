"""Thin ctypes binding of libsik.so (C ABI in include/sik.h).

Argument marshalling only: every step of the path runs in the HIP kernels.  torch is used for
device memory and streams; tensors are passed as raw device pointers.  There is no CPU fallback:
if the shared library is missing or a call fails, an exception is raised.
"""
import ctypes
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsik.so")

SIK_F16, SIK_BF16, SIK_F32 = 0, 1, 2
SIK_Q_FIT, SIK_Q_ENCODE = 1, 2
_TORCH2SIK = {torch.float16: SIK_F16, torch.bfloat16: SIK_BF16, torch.float32: SIK_F32}

EXPORTS = ("sik_strerror", "sik_version", "sik_plan_info", "sik_workspace_bytes", "sik_workspace_init",
           "sik_workspace_status", "sik_quantize_keys", "sik_score",
           "sik_topk", "sik_sparse_attn", "sik_decode_step", "sik_decode_step_static", "sik_decode_step_profiled", "sik_kvq_bytes",
           "sik_quantize_kv", "sik_prefill_compress", "sik_sparse_attn_q2", "sik_decode_step_q2", "sik_decode_step_ex")


class SikError(RuntimeError):
    def __init__(self, status, text):
        super().__init__(f"sik status {status}: {text}")
        self.status = status


class DecodeArgs(ctypes.Structure):
    """sik_decode_args of include/sik.h."""
    _fields_ = [("q", ctypes.c_void_p), ("k_new", ctypes.c_void_p), ("v_new", ctypes.c_void_p),
                ("K", ctypes.c_void_p), ("V", ctypes.c_void_p), ("kvq", ctypes.c_void_p), ("alpha", ctypes.c_void_p),
                ("seq_len", ctypes.c_void_p), ("mu", ctypes.c_void_p), ("codebook", ctypes.c_void_p),
                ("codes", ctypes.c_void_p), ("k", ctypes.c_int32), ("k_per_mille", ctypes.c_int32),
                ("group_shared", ctypes.c_int32), ("softmax_scale", ctypes.c_float),
                ("forced_idx", ctypes.c_void_p), ("n_forced", ctypes.c_int32), ("forced_K", ctypes.c_void_p),
                ("forced_V", ctypes.c_void_p), ("out", ctypes.c_void_p), ("idx_out", ctypes.c_void_p),
                ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t), ("stream", ctypes.c_void_p),
                ("kernel_us", ctypes.POINTER(ctypes.c_float)), ("launches", ctypes.c_int32),
                ("spin_limit", ctypes.c_int32)]


class Layout(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32), ("n_q_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("max_len", ctypes.c_int32), ("kv_dtype", ctypes.c_int32),
                ("out_dtype", ctypes.c_int32)]


_lib = None


def lib():
    """Load libsik.so (built in-tree by paper_2603_14224_amd/build.py); raises if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} not built: run `python -m paper_2603_14224_amd.build` "
                              "(or __graft_entry__.build()) first; there is no fallback path")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, sz, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t, ctypes.c_float
        lp = ctypes.POINTER(Layout)
        L.sik_strerror.restype = ctypes.c_char_p
        L.sik_strerror.argtypes = [ctypes.c_int]
        L.sik_version.restype = ctypes.c_int
        L.sik_plan_info.restype = ctypes.c_int
        L.sik_plan_info.argtypes = [lp, ctypes.POINTER(i32)]
        L.sik_workspace_bytes.restype = sz
        L.sik_workspace_init.restype = ctypes.c_int
        L.sik_workspace_init.argtypes = [lp, i32, vp, sz, vp]
        L.sik_workspace_status.restype = ctypes.c_int
        L.sik_workspace_status.argtypes = [vp, vp, ctypes.POINTER(ctypes.c_uint32)]
        L.sik_workspace_bytes.argtypes = [lp, i32]
        L.sik_quantize_keys.restype = ctypes.c_int
        L.sik_quantize_keys.argtypes = [lp, vp, vp, i32, i32, ctypes.c_int, vp, vp, vp, vp, vp, sz, vp]
        L.sik_score.restype = ctypes.c_int
        L.sik_score.argtypes = [lp, vp, vp, vp, vp, vp, vp]
        L.sik_topk.restype = ctypes.c_int
        L.sik_topk.argtypes = [lp, vp, vp, i32, vp, vp, sz, vp]
        L.sik_sparse_attn.restype = ctypes.c_int
        L.sik_sparse_attn.argtypes = [lp, vp, vp, vp, vp, i32, f32, vp, vp, sz, vp]
        L.sik_decode_step.restype = ctypes.c_int
        L.sik_decode_step.argtypes = [lp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, f32, vp, vp, vp, sz, vp]
        L.sik_decode_step_static.restype = ctypes.c_int
        L.sik_decode_step_static.argtypes = [lp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, f32, vp, vp, vp]
        L.sik_decode_step_profiled.restype = ctypes.c_int
        L.sik_decode_step_profiled.argtypes = L.sik_decode_step.argtypes + [ctypes.POINTER(ctypes.c_float)]
        L.sik_kvq_bytes.restype = sz
        L.sik_kvq_bytes.argtypes = [lp]
        L.sik_quantize_kv.restype = ctypes.c_int
        L.sik_quantize_kv.argtypes = [lp, vp, vp, vp, i32, i32, ctypes.c_int, vp, vp, vp, vp]
        L.sik_prefill_compress.restype = ctypes.c_int
        L.sik_prefill_compress.argtypes = [lp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.sik_sparse_attn_q2.restype = ctypes.c_int
        L.sik_sparse_attn_q2.argtypes = [lp, vp, vp, vp, vp, i32, f32, vp, vp, sz, vp]
        L.sik_decode_step_ex.restype = ctypes.c_int
        L.sik_decode_step_ex.argtypes = [lp, ctypes.POINTER(DecodeArgs)]
        L.sik_decode_step_q2.restype = ctypes.c_int
        L.sik_decode_step_q2.argtypes = [lp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, f32, vp, vp, vp, sz, vp,
                                         ctypes.POINTER(ctypes.c_float)]
        _lib = L
    return _lib


def _check(rc):
    if rc != 0:
        raise SikError(rc, lib().sik_strerror(rc).decode())


def _ptr(t):
    if t is None:
        return None
    assert t.is_contiguous(), "sik tensors must be contiguous"
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    # Without a GPU the C side still validates arguments first; any launch then reports SIK_ERR_LAUNCH.
    if not torch.cuda.is_available():
        return None
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def make_layout(batch, n_kv_heads, n_q_heads, head_dim, max_len, kv_dtype, out_dtype=None) -> Layout:
    kd = _TORCH2SIK[kv_dtype] if isinstance(kv_dtype, torch.dtype) else int(kv_dtype)
    od = kd if out_dtype is None else (_TORCH2SIK[out_dtype] if isinstance(out_dtype, torch.dtype) else int(out_dtype))
    return Layout(batch, n_kv_heads, n_q_heads, head_dim, max_len, kd, od)


def sik_strerror(status: int) -> str:
    return lib().sik_strerror(status).decode()


def sik_plan_info(layout: Layout):
    """Launch geometry of a layout (SIK_PLAN_INFO_LEN ints, see include/sik.h); raises on a bad layout."""
    info = (ctypes.c_int32 * 8)()
    _check(lib().sik_plan_info(ctypes.byref(layout), info))
    return [int(x) for x in info]


def sik_workspace_bytes(layout: Layout, k: int) -> int:
    return int(lib().sik_workspace_bytes(ctypes.byref(layout), int(k)))


def alloc_workspace(layout: Layout, k: int, device="cuda") -> torch.Tensor:
    """Device buffer of sik_workspace_bytes, initialised with sik_workspace_init."""
    n = sik_workspace_bytes(layout, k)
    if n == 0:
        raise SikError(-2, "sik_workspace_bytes rejected the layout / k")
    ws = torch.empty(n, dtype=torch.uint8, device=device)
    sik_workspace_init(layout, k, ws)
    return ws


def sik_workspace_init(layout: Layout, k: int, workspace):
    _check(lib().sik_workspace_init(ctypes.byref(layout), int(k), _ptr(workspace), workspace.numel(), _stream()))


def sik_workspace_status(workspace) -> int:
    """Status word of the workspace after waiting for the current stream (0 = every step completed)."""
    st = ctypes.c_uint32(0)
    _check(lib().sik_workspace_status(_ptr(workspace), _stream(), ctypes.byref(st)))
    return int(st.value)


def sik_quantize_keys(layout, K, seq_len, t0, n, mode, mu, codebook, counts, codes, workspace):
    _check(lib().sik_quantize_keys(ctypes.byref(layout), _ptr(K), _ptr(seq_len), int(t0), int(n), int(mode),
                                   _ptr(mu), _ptr(codebook), _ptr(counts), _ptr(codes), _ptr(workspace),
                                   workspace.numel() if workspace is not None else 0, _stream()))


def sik_score(layout, q, codebook, codes, seq_len, scores):
    _check(lib().sik_score(ctypes.byref(layout), _ptr(q), _ptr(codebook), _ptr(codes), _ptr(seq_len),
                           _ptr(scores), _stream()))


def sik_topk(layout, scores, seq_len, k, idx, workspace):
    _check(lib().sik_topk(ctypes.byref(layout), _ptr(scores), _ptr(seq_len), int(k), _ptr(idx),
                          _ptr(workspace), workspace.numel() if workspace is not None else 0, _stream()))


def sik_sparse_attn(layout, q, K, V, idx, k, softmax_scale, out, workspace):
    _check(lib().sik_sparse_attn(ctypes.byref(layout), _ptr(q), _ptr(K), _ptr(V), _ptr(idx), int(k),
                                 float(softmax_scale), _ptr(out), _ptr(workspace),
                                 workspace.numel() if workspace is not None else 0, _stream()))


def sik_kvq_bytes(layout: Layout) -> int:
    return int(lib().sik_kvq_bytes(ctypes.byref(layout)))


def alloc_kvq(layout: Layout, device="cuda") -> torch.Tensor:
    """Zeroed record plane [B, Hkv, max_len, 128] uint8 of the 2-bit K/V format."""
    n = sik_kvq_bytes(layout)
    if n == 0:
        raise SikError(-2, "sik_kvq_bytes rejected the layout")
    return torch.zeros(layout.batch, layout.n_kv_heads, layout.max_len, 128, dtype=torch.uint8, device=device)


def sik_quantize_kv(layout, K, V, seq_len, t0, n, mode, mu, alpha, kvq):
    _check(lib().sik_quantize_kv(ctypes.byref(layout), _ptr(K), _ptr(V), _ptr(seq_len), int(t0), int(n), int(mode),
                                 _ptr(mu), _ptr(alpha), _ptr(kvq), _stream()))


def sik_prefill_compress(layout, K, V, seq_len, mu, codebook, counts, codes, alpha, kvq, workspace):
    """mu, codes, codebook, counts, alpha and records of the fitted tokens in two passes over K and one over V."""
    _check(lib().sik_prefill_compress(ctypes.byref(layout), _ptr(K), _ptr(V), _ptr(seq_len), _ptr(mu), _ptr(codebook),
                                      _ptr(counts), _ptr(codes), _ptr(alpha), _ptr(kvq), _ptr(workspace),
                                      workspace.numel() if workspace is not None else 0, _stream()))


def sik_sparse_attn_q2(layout, q, kvq, alpha, idx, k, softmax_scale, out, workspace):
    _check(lib().sik_sparse_attn_q2(ctypes.byref(layout), _ptr(q), _ptr(kvq), _ptr(alpha), _ptr(idx), int(k),
                                    float(softmax_scale), _ptr(out), _ptr(workspace),
                                    workspace.numel() if workspace is not None else 0, _stream()))


def sik_decode_step_q2(layout, q, k_new, v_new, kvq, seq_len, mu, alpha, codebook, codes, k, softmax_scale, out,
                       idx_out, workspace, profiled=False):
    """Decode step on the 2-bit cache; with profiled=True returns the SIK_N_KERNELS + 1 event intervals (us)."""
    us = (ctypes.c_float * 5)() if profiled else None
    _check(lib().sik_decode_step_q2(ctypes.byref(layout), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(kvq),
                                    _ptr(seq_len), _ptr(mu), _ptr(alpha), _ptr(codebook), _ptr(codes), int(k),
                                    float(softmax_scale), _ptr(out), _ptr(idx_out), _ptr(workspace),
                                    workspace.numel() if workspace is not None else 0, _stream(), us))
    return [float(x) for x in us] if profiled else None


def sik_decode_step_ex(layout, *, q, seq_len, codebook, codes, k, out, workspace, k_new=None, v_new=None, K=None,
                       V=None, kvq=None, alpha=None, mu=None, softmax_scale=0.0, forced_idx=None, forced_K=None,
                       forced_V=None, idx_out=None, k_per_mille=0, group_shared=False, profiled=False,
                       launches=0, spin_limit=0):
    """General decode step (argument block of include/sik.h): either cache format, optional forced set."""
    us = (ctypes.c_float * 5)() if profiled else None

    def vp(t):
        return None if t is None else _ptr(t).value

    st = _stream()

    a = DecodeArgs(q=vp(q), k_new=vp(k_new), v_new=vp(v_new), K=vp(K), V=vp(V), kvq=vp(kvq), alpha=vp(alpha),
                   seq_len=vp(seq_len), mu=vp(mu), codebook=vp(codebook), codes=vp(codes), k=int(k),
                   k_per_mille=int(k_per_mille), group_shared=1 if group_shared else 0, softmax_scale=float(softmax_scale), forced_idx=vp(forced_idx),
                   n_forced=0 if forced_idx is None else int(forced_idx.shape[-1]), forced_K=vp(forced_K),
                   forced_V=vp(forced_V), out=vp(out), idx_out=vp(idx_out), workspace=vp(workspace),
                   workspace_bytes=workspace.numel() if workspace is not None else 0,
                   stream=None if st is None else st.value, kernel_us=us, launches=int(launches),
                   spin_limit=int(spin_limit))
    _check(lib().sik_decode_step_ex(ctypes.byref(layout), ctypes.byref(a)))
    return [float(x) for x in us] if profiled else None


def sik_decode_step(layout, q, k_new, v_new, K, V, seq_len, mu, codebook, codes, k, softmax_scale, out, idx_out,
                    workspace):
    _check(lib().sik_decode_step(ctypes.byref(layout), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(K), _ptr(V),
                                 _ptr(seq_len), _ptr(mu), _ptr(codebook), _ptr(codes), int(k),
                                 float(softmax_scale), _ptr(out), _ptr(idx_out), _ptr(workspace),
                                 workspace.numel() if workspace is not None else 0, _stream()))


SIK_STATIC_SCRATCH_BYTES = 32 << 20


def sik_decode_step_static(layout, q, k_new, v_new, K, V, seq_len, mu, codebook, codes, k, softmax_scale, out, idx_out):
    """sik_decode_step on the library's built-in scratch buffer (no workspace argument, nothing allocated)."""
    _check(lib().sik_decode_step_static(ctypes.byref(layout), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(K), _ptr(V),
                                        _ptr(seq_len), _ptr(mu), _ptr(codebook), _ptr(codes), int(k),
                                        float(softmax_scale), _ptr(out), _ptr(idx_out), _stream()))


def sik_decode_step_profiled(layout, q, k_new, v_new, K, V, seq_len, mu, codebook, codes, k, softmax_scale, out,
                             idx_out, workspace):
    """Runs one decode step with per-kernel HIP events; returns the 4 event-to-event intervals and the
    empty-interval cost of an event pair, in microseconds."""
    us = (ctypes.c_float * 5)()
    _check(lib().sik_decode_step_profiled(ctypes.byref(layout), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(K),
                                          _ptr(V), _ptr(seq_len), _ptr(mu), _ptr(codebook), _ptr(codes), int(k),
                                          float(softmax_scale), _ptr(out), _ptr(idx_out), _ptr(workspace),
                                          workspace.numel() if workspace is not None else 0, _stream(), us))
    return list(us)

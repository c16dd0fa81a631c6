"""ctypes front end of the CPU oracle (oracle/sik_oracle.c).

TEST INFRASTRUCTURE, NOT THE PRODUCT: only tests, the smoke check and the
benchmark's CPU-baseline leg may import this module.  It does not import the
HIP package and the HIP package does not import it.

All tensors are numpy arrays; 16-bit floats travel as raw uint16 bit patterns
with dtype "fp16" or "bf16".  Shapes follow the C file's header.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_DT = {"fp16": 0, "bf16": 1}
_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        _lib = ctypes.CDLL(path)
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dt):
    a = np.ascontiguousarray(a, dtype=dt)
    return a


def set_threads(n: int) -> int:
    return lib().sik_oracle_set_threads(int(n))


def widen(x_bits, dtype):
    x = _c(x_bits, np.uint16)
    out = np.empty(x.shape, np.float64)
    rc = lib().sik_oracle_widen(_p(x), _DT[dtype], ctypes.c_int64(x.size), _p(out))
    assert rc == 0
    return out


def mean(K, dtype, seq_len):
    K = _c(K, np.uint16)
    B, Hkv, Lmax, D = K.shape
    sl = _c(seq_len, np.int32)
    mu = np.empty((B, Hkv, D), np.float32)
    rc = lib().sik_oracle_mean(_p(K), _DT[dtype], B, Hkv, Lmax, D, _p(sl), _p(mu))
    assert rc == 0
    return mu


def encode(K, dtype, mu, t0, n, codes=None):
    """Encode tokens [t0, t0+n) of every (b, h) against mu; returns codes."""
    K = _c(K, np.uint16)
    B, Hkv, Lmax, D = K.shape
    mu = _c(mu, np.float32)
    if codes is None:
        codes = np.zeros((B, Hkv, Lmax, D // 8), np.uint8)
    assert codes.dtype == np.uint8 and codes.flags.c_contiguous
    rc = lib().sik_oracle_encode(_p(K), _DT[dtype], B, Hkv, Lmax, D, int(t0), int(n), _p(mu), _p(codes))
    assert rc == 0
    return codes


def codebook(K, dtype, seq_len, mu, codes):
    K = _c(K, np.uint16)
    B, Hkv, Lmax, D = K.shape
    sl = _c(seq_len, np.int32)
    mu = _c(mu, np.float32)
    codes = _c(codes, np.uint8)
    cb = np.empty((B, Hkv, D // 4, 16, 4), np.float32)
    cnt = np.empty((B, Hkv, D // 4, 16), np.int32)
    rc = lib().sik_oracle_codebook(_p(K), _DT[dtype], B, Hkv, Lmax, D, _p(sl), _p(mu), _p(codes),
                                   _p(cb), _p(cnt))
    assert rc == 0
    return cb, cnt


def fit(K, dtype, seq_len):
    """Prefill-side quantiser: mu, codes of tokens [0, seq_len), codebook, counts."""
    K = _c(K, np.uint16)
    B, Hkv, Lmax, D = K.shape
    sl = _c(seq_len, np.int32)
    mu = mean(K, dtype, sl)
    codes = np.zeros((B, Hkv, Lmax, D // 8), np.uint8)
    for b in range(B):
        encode(K[b:b + 1], dtype, mu[b:b + 1], 0, int(sl[b]), codes[b:b + 1])
    cb, cnt = codebook(K, dtype, sl, mu, codes)
    return mu, codes, cb, cnt


def table(q, dtype, cb):
    q = _c(q, np.uint16)
    B, Hq, D = q.shape
    cb = _c(cb, np.float32)
    Hkv = cb.shape[1]
    T = np.empty((B, Hq, D // 4, 16), np.float64)
    rc = lib().sik_oracle_table(_p(q), _DT[dtype], B, Hkv, Hq, D, _p(cb), _p(T))
    assert rc == 0
    return T


def score(q, dtype, cb, codes, seq_len):
    """fp64 scores [B, Hq, Lmax]; entries at or beyond seq_len[b] are -inf."""
    T = table(q, dtype, cb)
    codes = _c(codes, np.uint8)
    B, Hkv, Lmax, D8 = codes.shape
    Hq = T.shape[1]
    sl = _c(seq_len, np.int32)
    s = np.full((B, Hq, Lmax), -np.inf, np.float64)
    rc = lib().sik_oracle_score(_p(T), _p(codes), B, Hkv, Hq, Lmax, D8 * 8, _p(sl), _p(s))
    assert rc == 0
    return s


def topk(scores, seq_len, k):
    s = _c(scores, np.float64)
    B, Hq, Lmax = s.shape
    sl = _c(seq_len, np.int32)
    idx = np.empty((B, Hq, int(k)), np.int32)
    rc = lib().sik_oracle_topk(_p(s), B, Hq, Lmax, _p(sl), int(k), _p(idx))
    assert rc == 0
    return idx


def sparse_attn(q, K, V, dtype, idx, scale=0.0):
    q = _c(q, np.uint16)
    K = _c(K, np.uint16)
    V = _c(V, np.uint16)
    idx = _c(idx, np.int32)
    B, Hkv, Lmax, D = K.shape
    Hq = q.shape[1]
    k = idx.shape[2]
    out = np.empty((B, Hq, D), np.float64)
    rc = lib().sik_oracle_sparse_attn(_p(q), _p(K), _p(V), _DT[dtype], B, Hkv, Hq, Lmax, D, _p(idx), k,
                                      ctypes.c_double(float(scale)), _p(out))
    assert rc == 0
    return out


def decode_step(q, k_new, v_new, K, V, dtype, seq_len, mu, cb, codes, k, scale=0.0):
    """One decode step.  With k_new/v_new given, the new row is first written
    to row seq_len[b] of K and V (in place), encoded against the frozen mu (in
    place in codes), and seq_len (in place) grows by one; the new token then
    competes in the selection like any other.  Returns (out fp64, idx)."""
    assert K.dtype == np.uint16 and K.flags.c_contiguous
    assert V.dtype == np.uint16 and V.flags.c_contiguous
    B, Hkv, Lmax, D = K.shape
    if k_new is not None:
        kn = _c(k_new, np.uint16)
        vn = _c(v_new, np.uint16)
        rc = lib().sik_oracle_append_rows(_p(K), _p(V), _p(kn), _p(vn), B, Hkv, Lmax, D, _p(seq_len))
        assert rc == 0
        for b in range(B):
            encode(K[b:b + 1], dtype, mu[b:b + 1], int(seq_len[b]), 1, codes[b:b + 1])
        seq_len += 1
    s = score(q, dtype, cb, codes, seq_len)
    idx = topk(s, seq_len, k)
    out = sparse_attn(q, K, V, dtype, idx, scale)
    return out, idx

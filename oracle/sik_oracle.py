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


# --------------------------------------------------------------------------- 2-bit token-wise K/V format
def to_fp16(x):
    """binary32 -> IEEE binary16 bit patterns (round to nearest even), the oracle's own conversion."""
    x = _c(x, np.float32)
    out = np.empty(x.shape, np.uint16)
    rc = lib().sik_oracle_to_fp16(_p(x), ctypes.c_int64(x.size), _p(out))
    assert rc == 0
    return out


def f64_to_fp16(x):
    """fp64 -> IEEE binary16 bit patterns in one rounding (nearest even): how the stored parameters are rounded."""
    x = _c(x, np.float64)
    out = np.empty(x.shape, np.uint16)
    rc = lib().sik_oracle_f64_to_fp16(_p(x), ctypes.c_int64(x.size), _p(out))
    assert rc == 0
    return out


def alpha(K, dtype, seq_len, mu):
    """Per-channel max |K - mu| over the tokens below seq_len (fp64, stored as fp32): [B, Hkv, D]."""
    K = _c(K, np.uint16)
    B, Hkv, Lmax, D = K.shape
    sl = _c(seq_len, np.int32)
    mu = _c(mu, np.float32)
    a = np.empty((B, Hkv, D), np.float32)
    rc = lib().sik_oracle_alpha(_p(K), _DT[dtype], B, Hkv, Lmax, D, _p(sl), _p(mu), _p(a))
    assert rc == 0
    return a


class QuantKV:
    """Logical fields of the 2-bit format: kq, vq [B,Hkv,Lmax,D] uint8 in 0..3; kpar, vpar
    [B,Hkv,Lmax,D/32,2] uint16 = fp16 bits of (qs, zp)."""

    def __init__(self, B, Hkv, Lmax, D):
        self.kq = np.zeros((B, Hkv, Lmax, D), np.uint8)
        self.vq = np.zeros((B, Hkv, Lmax, D), np.uint8)
        self.kpar = np.zeros((B, Hkv, Lmax, D // 32, 2), np.uint16)
        self.vpar = np.zeros((B, Hkv, Lmax, D // 32, 2), np.uint16)


def quantize_kv(K, V, dtype, mu, alpha_, t0, n, qkv=None):
    """Quantise tokens [t0, t0+n) of every (b, h) in place in qkv (created when None)."""
    K = _c(K, np.uint16)
    V = _c(V, np.uint16)
    B, Hkv, Lmax, D = K.shape
    if qkv is None:
        qkv = QuantKV(B, Hkv, Lmax, D)
    mu = _c(mu, np.float32)
    al = _c(alpha_, np.float32)
    rc = lib().sik_oracle_quantize_kv(_p(K), _p(V), _DT[dtype], B, Hkv, Lmax, D, int(t0), int(n), _p(mu), _p(al),
                                      _p(qkv.kq), _p(qkv.kpar), _p(qkv.vq), _p(qkv.vpar))
    assert rc == 0
    return qkv


def dequant_kv(codes, qkv, alpha_, t0, n):
    """fp64 (K', V) reconstructed from the fields for tokens [t0, t0+n); other rows are zero."""
    codes = _c(codes, np.uint8)
    B, Hkv, Lmax, D = qkv.kq.shape
    al = _c(alpha_, np.float32)
    Kd = np.zeros((B, Hkv, Lmax, D), np.float64)
    Vd = np.zeros((B, Hkv, Lmax, D), np.float64)
    rc = lib().sik_oracle_dequant_kv(_p(codes), _p(qkv.kq), _p(qkv.kpar), _p(qkv.vq), _p(qkv.vpar), _p(al), B, Hkv,
                                     Lmax, D, int(t0), int(n), _p(Kd), _p(Vd))
    assert rc == 0
    return Kd, Vd


def sparse_attn_q2(q, dtype, codes, qkv, alpha_, idx, scale=0.0):
    q = _c(q, np.uint16)
    codes = _c(codes, np.uint8)
    idx = _c(idx, np.int32)
    B, Hkv, Lmax, D = qkv.kq.shape
    Hq, k = q.shape[1], idx.shape[2]
    al = _c(alpha_, np.float32)
    out = np.empty((B, Hq, D), np.float64)
    rc = lib().sik_oracle_sparse_attn_q2(_p(q), _DT[dtype], _p(codes), _p(qkv.kq), _p(qkv.kpar), _p(qkv.vq),
                                         _p(qkv.vpar), _p(al), B, Hkv, Hq, Lmax, D, _p(idx), k,
                                         ctypes.c_double(float(scale)), _p(out))
    assert rc == 0
    return out


def pack_records(codes, qkv):
    """The 128-byte per-token record of the library's 2-bit format, built from the fields: 16 slots of 8
    bytes, slot p covering channels 8p..8p+7: byte 0 = sign byte p of the 1-bit code, byte 1 = 0, bytes 2-3 =
    K codes (little-endian, code of channel 8p+e in bits 2e+1:2e), bytes 4-5 = V codes likewise, bytes 6-7 =
    one fp16 parameter of 32-channel group p/4: K qs, K zp, V qs, V zp for p mod 4 = 0, 1, 2, 3."""
    B, Hkv, Lmax, D = qkv.kq.shape
    assert D == 128
    rec = np.zeros((B, Hkv, Lmax, 16, 8), np.uint8)
    rec[..., 0] = codes
    sh = (2 * np.arange(8)).astype(np.uint16)
    kw = (qkv.kq.reshape(B, Hkv, Lmax, 16, 8).astype(np.uint16) << sh).sum(axis=-1).astype(np.uint16)
    vw = (qkv.vq.reshape(B, Hkv, Lmax, 16, 8).astype(np.uint16) << sh).sum(axis=-1).astype(np.uint16)
    par = np.concatenate([qkv.kpar, qkv.vpar], axis=-1).reshape(B, Hkv, Lmax, 16)  # group-major: Kqs Kzp Vqs Vzp
    for word, at in ((kw, 2), (vw, 4), (par, 6)):
        rec[..., at] = (word & 0xff).astype(np.uint8)
        rec[..., at + 1] = (word >> 8).astype(np.uint8)
    return rec.reshape(B, Hkv, Lmax, 128)


def unpack_records(rec):
    """Inverse of pack_records: (codes, QuantKV) from [B,Hkv,Lmax,128] uint8 records."""
    rec = np.ascontiguousarray(rec, np.uint8)
    B, Hkv, Lmax, _ = rec.shape
    r = rec.reshape(B, Hkv, Lmax, 16, 8)
    codes = r[..., 0].copy()
    out = QuantKV(B, Hkv, Lmax, 128)
    sh = (2 * np.arange(8)).astype(np.uint16)
    kw = r[..., 2].astype(np.uint16) | (r[..., 3].astype(np.uint16) << 8)
    vw = r[..., 4].astype(np.uint16) | (r[..., 5].astype(np.uint16) << 8)
    out.kq = ((kw[..., None] >> sh) & 3).astype(np.uint8).reshape(B, Hkv, Lmax, 128)
    out.vq = ((vw[..., None] >> sh) & 3).astype(np.uint8).reshape(B, Hkv, Lmax, 128)
    par = (r[..., 6].astype(np.uint16) | (r[..., 7].astype(np.uint16) << 8)).reshape(B, Hkv, Lmax, 4, 4)
    out.kpar = np.ascontiguousarray(par[..., 0:2])
    out.vpar = np.ascontiguousarray(par[..., 2:4])
    return codes, out


def fit_q2(K, V, dtype, seq_len, mu):
    """Prefill-side 2-bit quantiser: alpha from the fitted tokens, then their fields."""
    K = _c(K, np.uint16)
    B = K.shape[0]
    sl = _c(seq_len, np.int32)
    al = alpha(K, dtype, sl, mu)
    qkv = None
    for b in range(B):
        part = quantize_kv(K[b:b + 1], V[b:b + 1], dtype, mu[b:b + 1], al[b:b + 1], 0, int(sl[b]))
        if qkv is None:
            qkv = QuantKV(*K.shape)
        for f in ("kq", "vq", "kpar", "vpar"):
            getattr(qkv, f)[b] = getattr(part, f)[0]
    return al, qkv


def decode_step_q2(q, k_new, v_new, dtype, seq_len, mu, alpha_, cb, codes, qkv, k, scale=0.0):
    """One decode step on the 2-bit cache.  With k_new/v_new [B,Hkv,D] given, the new token is encoded
    (sign code against the frozen mu, magnitudes against the frozen alpha) into row seq_len[b] in place and
    seq_len grows by one.  Returns (out fp64, idx)."""
    B, Hkv, Lmax, D = qkv.kq.shape
    if k_new is not None:
        kn = _c(k_new, np.uint16).reshape(B, Hkv, 1, D)
        vn = _c(v_new, np.uint16).reshape(B, Hkv, 1, D)
        for b in range(B):
            t = int(seq_len[b])
            assert t < Lmax
            codes[b, :, t] = encode(kn[b:b + 1], dtype, mu[b:b + 1], 0, 1)[0, :, 0]
            one = quantize_kv(kn[b:b + 1], vn[b:b + 1], dtype, mu[b:b + 1], alpha_[b:b + 1], 0, 1)
            for f in ("kq", "vq", "kpar", "vpar"):
                getattr(qkv, f)[b, :, t] = getattr(one, f)[0, :, 0]
        seq_len += 1
    s = score(q, dtype, cb, codes, seq_len)
    idx = topk(s, seq_len, k)
    out = sparse_attn_q2(q, dtype, codes, qkv, alpha_, idx, scale)
    return out, idx


# --------------------------------------------------------------------------- forced-inclusion sets (sink tokens)
def forced_valid(forced_idx, seq_len):
    """Which entries of forced_idx [B,Hkv,nf] name a token: 0 <= idx < seq_len[b]."""
    f = np.asarray(forced_idx, np.int32)
    sl = np.asarray(seq_len, np.int32).reshape(-1, 1, 1)
    return (f >= 0) & (f < sl)


def budget(k, seq_len_b, k_per_mille):
    """Tokens sequence b attends: k, or with k_per_mille > 0 the smaller of k and ceil(L * k_per_mille / 1000)
    (a fraction of the context such as the paper's 7.5 %), at least 1."""
    if k_per_mille <= 0:
        return int(k)
    return min(int(k), max(1, (int(seq_len_b) * int(k_per_mille) + 999) // 1000))


def topk_with_forced(scores, seq_len, k, forced_idx, R, k_per_mille=0):
    """Selection with a forced set: per (b, KV head) the valid forced tokens always take part and never
    compete; every query head of the group then takes the budget - (number of valid forced tokens) best of
    the others (none if the forced tokens fill the budget).  Returns idx [B,Hq,k]: forced tokens first, then
    the dynamic picks, then -1."""
    s = np.array(scores, np.float64, copy=True)
    B, Hq, Lmax = s.shape
    valid = forced_valid(forced_idx, seq_len)
    idx = np.full((B, Hq, int(k)), -1, np.int32)
    for b in range(B):
        for h in range(Hq // R):
            f = np.asarray(forced_idx)[b, h][valid[b, h]].astype(np.int32)
            assert len(set(f.tolist())) == len(f), "forced tokens must be distinct"
            assert len(f) < k, "the budget k must exceed the forced set"
            rows = slice(h * R, (h + 1) * R)
            s[b, rows][:, f] = -np.inf
            idx[b, rows, :len(f)] = f
            kd = budget(k, seq_len[b], k_per_mille) - len(f)
            if kd <= 0:
                continue
            dyn = topk(s[b:b + 1, rows], np.asarray(seq_len, np.int32)[b:b + 1], kd)[0]
            # a dynamic pick can never be a forced token: there are seq_len - len(f) others and kd of them exist
            kd_eff = min(kd, int(seq_len[b]) - len(f))
            dyn[:, kd_eff:] = -1
            idx[b, rows, len(f):len(f) + kd] = dyn
    return idx


def sparse_attn_q2_forced(q, dtype, codes, qkv, alpha_, mu, fK, fV, fvalid, idx, scale=0.0):
    """Attention over records (idx) plus full-precision forced rows fK, fV [B,Hkv,nf,D] (valid where fvalid)."""
    q = _c(q, np.uint16)
    codes = _c(codes, np.uint8)
    idx = _c(idx, np.int32)
    fK, fV = _c(fK, np.uint16), _c(fV, np.uint16)
    fv = _c(fvalid, np.uint8)
    B, Hkv, Lmax, D = qkv.kq.shape
    Hq, k, nf = q.shape[1], idx.shape[2], fK.shape[2]
    out = np.empty((B, Hq, D), np.float64)
    rc = lib().sik_oracle_sparse_attn_q2_forced(_p(q), _DT[dtype], _p(codes), _p(qkv.kq), _p(qkv.kpar), _p(qkv.vq),
                                                _p(qkv.vpar), _p(_c(alpha_, np.float32)), _p(_c(mu, np.float32)),
                                                _p(fK), _p(fV), _p(fv), nf, B, Hkv, Hq, Lmax, D, _p(idx), k,
                                                ctypes.c_double(float(scale)), _p(out))
    assert rc == 0
    return out


def decode_step_forced(q, k_new, v_new, K, V, dtype, seq_len, mu, cb, codes, k, forced_idx, scale=0.0,
                       k_per_mille=0):
    """decode_step with a forced set (and optionally a budget that follows the context length) on the 16-bit
    cache: forced tokens are read from the cache like the others."""
    B, Hkv, Lmax, D = K.shape
    if k_new is not None:
        decode_step(q, k_new, v_new, K, V, dtype, seq_len, mu, cb, codes, 1, scale)  # append only; result unused
    s = score(q, dtype, cb, codes, seq_len)
    idx = topk_with_forced(s, seq_len, k, forced_idx, q.shape[1] // Hkv, k_per_mille)
    return sparse_attn(q, K, V, dtype, idx, scale), idx


def decode_step_q2_forced(q, k_new, v_new, dtype, seq_len, mu, alpha_, cb, codes, qkv, k, forced_idx, fK=None,
                          fV=None, scale=0.0):
    """decode_step_q2 with a forced set.  With fK, fV (16-bit rows of the forced tokens, slot by slot) the forced
    tokens are attended in full precision and only the dynamic picks come from records; otherwise all from
    records.  Returns (out, idx) with idx = forced tokens, dynamic picks, -1."""
    Hkv = qkv.kq.shape[1]
    if k_new is not None:
        decode_step_q2(q, k_new, v_new, dtype, seq_len, mu, alpha_, cb, codes, qkv, 1, scale)  # append only
    s = score(q, dtype, cb, codes, seq_len)
    idx = topk_with_forced(s, seq_len, k, forced_idx, q.shape[1] // Hkv)
    if fK is None:
        return sparse_attn_q2(q, dtype, codes, qkv, alpha_, idx, scale), idx
    valid = forced_valid(forced_idx, seq_len)
    R = q.shape[1] // Hkv
    dyn = idx.copy()
    for b in range(idx.shape[0]):
        for h in range(Hkv):
            dyn[b, h * R:(h + 1) * R, :int(valid[b, h].sum())] = -1   # the forced ones come from fK, fV instead
    out = sparse_attn_q2_forced(q, dtype, codes, qkv, alpha_, mu, fK, fV, valid.astype(np.uint8), dyn, scale)
    return out, idx


# --------------------------------------------------------------------------- group-shared selection
def shared_scores(q, dtype, cb, codes, seq_len):
    """Scores of a KV head = sum of the scores of its R query heads: [B, Hkv, Lmax] fp64 (-inf beyond seq_len)."""
    s = score(q, dtype, cb, codes, seq_len)
    B, Hq, Lmax = s.shape
    Hkv = codes.shape[1]
    return s.reshape(B, Hkv, Hq // Hkv, Lmax).sum(axis=2)


def decode_step_shared(q, k_new, v_new, K, V, dtype, seq_len, mu, cb, codes, k, scale=0.0):
    """Decode step with ONE index set per KV head, shared by the R query heads of its group: the k tokens with
    the largest summed score (ties to the smaller index).  Each query head then attends over that set with its
    own query.  Returns (out [B,Hq,D] fp64, idx [B,Hkv,k])."""
    if k_new is not None:
        decode_step(q, k_new, v_new, K, V, dtype, seq_len, mu, cb, codes, 1, scale)   # append only
    idx_kv = topk(shared_scores(q, dtype, cb, codes, seq_len), seq_len, k)
    R = q.shape[1] // K.shape[1]
    return sparse_attn(q, K, V, dtype, np.repeat(idx_kv, R, axis=1), scale), idx_kv

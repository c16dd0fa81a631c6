"""The near-tie rule of the 2-bit record parity tests (helpers.records_agree), checked on the CPU.

The oracle evaluates the quantisation function of "Token-Wise Quantization Format" in fp64 with true divisions.
An implementation that decides in binary32 (subtraction of mu, product with a rounded reciprocal of alpha,
subtraction of zp, product with a rounded reciprocal of qs) must agree with it everywhere except inside the
stated error band around a half-integer of t = (x - zp) / qs, or around an fp16 rounding boundary of a stored
parameter.  Here that binary32 evaluation is written in numpy and run through the rule, so that the rule itself
(and the size of the exception set it admits) is pinned without a GPU; a deliberately wrong evaluation must fail.
"""
import numpy as np
import pytest

import sik_workloads as W
from helpers import records_agree


def binary32_records(oracle, K, V, dtype, mu, alpha, codes, L, third_bias=0.0):
    """Records of tokens [0, L) of every (b, h), decided in binary32 with reciprocals (numpy)."""
    B, H, Lmax, D = K.shape
    K32, V32 = W.from_bits(K, dtype).astype(np.float32), W.from_bits(V, dtype).astype(np.float32)
    qkv = oracle.QuantKV(B, H, Lmax, D)
    with np.errstate(divide="ignore", invalid="ignore"):
        ral = np.where(alpha > 0, np.float32(1) / alpha, np.float32(0)).astype(np.float32)
    Kp = (K32[:, :, :L] - mu[:, :, None, :]).astype(np.float32)
    khat = (np.abs(Kp) * ral[:, :, None, :]).astype(np.float32)
    for x, q, par in ((khat, qkv.kq, qkv.kpar), (V32[:, :, :L], qkv.vq, qkv.vpar)):
        g = x.reshape(B, H, L, 4, 32)
        lo, hi = g.min(-1) + np.float32(0), g.max(-1)
        third = ((hi - lo).astype(np.float32) / np.float32(3)).astype(np.float32) * np.float32(1 + third_bias)
        par[:, :, :L, :, 0] = third.astype(np.float16).view(np.uint16)
        par[:, :, :L, :, 1] = lo.astype(np.float16).view(np.uint16)
        qs = par[:, :, :L, :, 0].view(np.float16).astype(np.float32)[..., None]
        zp = par[:, :, :L, :, 1].view(np.float16).astype(np.float32)[..., None]
        with np.errstate(divide="ignore", invalid="ignore"):
            rqs = (np.float32(1) / qs).astype(np.float32)
            t = ((g - zp).astype(np.float32) * rqs).astype(np.float32)
            q[:, :, :L] = np.where(qs > 0, np.clip(np.rint(t), 0, 3), 0).astype(np.uint8).reshape(B, H, L, D)
    return oracle.pack_records(codes, qkv)


@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
def test_binary32_decisions_stay_inside_the_band(oracle, dtype):
    cfg = W.scaled(W.CONFIGS["C2"], batch=2, n_kv_heads=2, n_q_heads=4, context=6000, top_k=16, dtype=dtype, seed=77)
    K, V = W.make_cache(cfg, channel_offset_std=1.0)
    sl = np.array([6000, 6000], np.int32)
    mu, codes, _, _ = oracle.fit(K, dtype, sl)
    al, qkv = oracle.fit_q2(K, V, dtype, sl, mu)
    rec = binary32_records(oracle, K, V, dtype, mu, al, codes, 6000)
    tot = np.zeros(4, np.int64)
    for b in range(2):
        tot += records_agree(oracle, rec, K, V, dtype, mu, al, codes, qkv, b, 0, 6000)
    n_par, n_code, tot_par, tot_code = tot
    print(f"{dtype}: {n_par} of {tot_par} parameters and {n_code} of {tot_code} codes differ inside the band")
    # the band admits only a sliver: under one parameter in a thousand and one code in twenty thousand
    assert n_par <= tot_par // 1000 and n_code <= tot_code // 20000
    # byte-identical records pass with no exception at all
    same = oracle.pack_records(codes, qkv)
    assert records_agree(oracle, same, K, V, dtype, mu, al, codes, qkv, 0, 0, 6000)[:2] == (0, 0)


def test_the_rule_rejects_a_wrong_quantiser(oracle):
    cfg = W.scaled(W.CONFIGS["C2"], batch=1, n_kv_heads=2, n_q_heads=4, context=500, top_k=16, seed=78)
    K, V = W.make_cache(cfg, channel_offset_std=1.0)
    sl = np.array([500], np.int32)
    mu, codes, _, _ = oracle.fit(K, cfg.dtype, sl)
    al, qkv = oracle.fit_q2(K, V, cfg.dtype, sl, mu)
    # a scale that is off by one part in a thousand is far outside the band
    rec = binary32_records(oracle, K, V, cfg.dtype, mu, al, codes, 500, third_bias=1e-3)
    with pytest.raises(AssertionError):
        records_agree(oracle, rec, K, V, cfg.dtype, mu, al, codes, qkv, 0, 0, 500)
    # one flipped code bit in an otherwise identical record
    rec = oracle.pack_records(codes, qkv)
    t = 0.0
    for tok in range(500):                       # find a code that is not near a tie and flip it
        bad = rec.copy()
        bad[0, 0, tok, 2] ^= 1
        try:
            records_agree(oracle, bad, K, V, cfg.dtype, mu, al, codes, qkv, 0, 0, 500)
        except AssertionError:
            t += 1
    assert t == 500
    # a wrong sign byte
    bad = rec.copy()
    bad[0, 1, 7, 8] ^= 0x10
    with pytest.raises(AssertionError):
        records_agree(oracle, bad, K, V, cfg.dtype, mu, al, codes, qkv, 0, 0, 500)

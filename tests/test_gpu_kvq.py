"""Parity of the 2-bit token-wise K/V path (records, attention on records, decode step on records) against the
CPU oracle, through the C ABI.

Bars: alpha bit-equal (a maximum of binary32 values); records byte-for-byte equal to the oracle's fields packed
into the documented layout (the codes are integer decisions taken in binary32 on both sides); attention within
the same bars as the 16-bit path (1e-5 relative for fp32 output) against the oracle's fp64 attention over the
dequantised rows; top-k sets as in the 16-bit decode step (scoring does not depend on the K/V format).
"""
import numpy as np
import pytest
import torch

import sik_workloads as W
from helpers import dev, topk_sets_agree
from test_gpu_parity import TDT, check_attention, cfg_small, sync

pytestmark = pytest.mark.gpu

import paper_2603_14224_amd as sik  # noqa: E402


class Q2State:
    """One layer's cache quantised by the oracle (fields + packed records) and mirrored on the device."""

    def __init__(self, cfg, oracle, capacity=None, seq_len=None, offset_std=0.0, out_dtype=None, K=None, V=None):
        self.cfg, self.o = cfg, oracle
        if K is None:
            K, V = W.make_cache(cfg, capacity=capacity, channel_offset_std=offset_std)
        self.K, self.V = K, V
        B, H, cap, D = K.shape
        self.sl = np.full(B, cfg.context, np.int32) if seq_len is None else np.asarray(seq_len, np.int32)
        self.mu, self.codes, self.cb, _ = oracle.fit(K, cfg.dtype, self.sl)
        self.alpha, self.qkv = oracle.fit_q2(K, V, cfg.dtype, self.sl, self.mu)
        self.layout = sik.make_layout(B, H, cfg.n_q_heads, D, cap, TDT[cfg.dtype], out_dtype)
        self.dK, self.dV = dev(K, cfg.dtype), dev(V, cfg.dtype)
        self.dsl = torch.from_numpy(self.sl.copy()).cuda()
        self.dmu = torch.from_numpy(self.mu).cuda()
        self.dcb = torch.from_numpy(self.cb).cuda()
        self.dcodes = torch.from_numpy(self.codes).cuda()
        self.ws = sik.alloc_workspace(self.layout, min(cfg.top_k, cap))

    def records(self):
        return self.o.pack_records(self.codes, self.qkv)


def gpu_fit(st):
    dal = torch.full(st.mu.shape, -1.0, device="cuda")
    kvq = sik.alloc_kvq(st.layout)
    sik.sik_quantize_kv(st.layout, st.dK, st.dV, st.dsl, 0, 0, sik.SIK_Q_FIT, st.dmu, dal, kvq)
    sync()
    return dal, kvq


@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
@pytest.mark.parametrize("offset", [0.0, 1.5])
def test_fit_alpha_and_records_bit_exact(oracle, dtype, offset):
    cfg = cfg_small(batch=2, n_kv_heads=3, n_q_heads=6, context=1337, top_k=64, dtype=dtype, seed=41)
    st = Q2State(cfg, oracle, capacity=1400, seq_len=[1337, 801], offset_std=offset)
    dal, kvq = gpu_fit(st)
    assert np.array_equal(dal.cpu().numpy(), st.alpha)
    got, want = kvq.cpu().numpy(), st.records()
    for b, L in enumerate(st.sl):
        assert np.array_equal(got[b, :, :L], want[b, :, :L])
        assert not got[b, :, L:].any()            # records beyond seq_len are not written
    assert sik.sik_kvq_bytes(st.layout) == got.nbytes


def test_encode_range_against_frozen_parameters(oracle):
    # tokens appended later may exceed the fitted range (|K - mu| > alpha): their groups adapt per token
    cfg = cfg_small(batch=2, n_kv_heads=2, n_q_heads=4, context=500, top_k=32, seed=42)
    st = Q2State(cfg, oracle, capacity=640, offset_std=1.0)
    dal, kvq = gpu_fit(st)
    rng = np.random.default_rng(0)
    K2, V2 = st.K.copy(), st.V.copy()
    new = W.make_cache(cfg, capacity=640, channel_offset_std=1.0, layer=3)
    K2[:, :, 500:633] = W.to_bits(W.from_bits(new[0][:, :, 500:633], cfg.dtype) * 3.0, cfg.dtype)
    V2[:, :, 500:633] = new[1][:, :, 500:633]
    qkv = oracle.quantize_kv(K2, V2, cfg.dtype, st.mu, st.alpha, 500, 133, st.qkv)
    codes = oracle.encode(K2, cfg.dtype, st.mu, 500, 133, st.codes)
    sik.sik_quantize_kv(st.layout, dev(K2, cfg.dtype), dev(V2, cfg.dtype), None, 500, 133, sik.SIK_Q_ENCODE, st.dmu,
                        dal, kvq)
    sync()
    got, want = kvq.cpu().numpy(), oracle.pack_records(codes, qkv)
    assert np.array_equal(got[:, :, :633], want[:, :, :633]) and not got[:, :, 633:].any()
    assert np.array_equal(dal.cpu().numpy(), st.alpha)      # frozen
    # empty range: nothing happens
    sik.sik_quantize_kv(st.layout, st.dK, st.dV, None, 10, 0, sik.SIK_Q_ENCODE, st.dmu, dal, kvq)
    sync()
    assert np.array_equal(kvq.cpu().numpy(), got)
    del rng


def test_degenerate_groups_and_channels(oracle):
    cfg = cfg_small(batch=1, n_kv_heads=2, n_q_heads=2, context=130, top_k=16, dtype="fp16", seed=43)
    K, V = W.make_cache(cfg)
    Kf, Vf = W.from_bits(K, "fp16").copy(), W.from_bits(V, "fp16").copy()
    Kf[0, 0, :, 5] = 0.75                    # a constant channel: K = mu there, alpha = 0
    Kf[0, 1, 7] = 0.0                        # a zero key row
    Vf[0, 0, 3] = 2.5                        # constant value row: qs = 0 in all four groups
    Vf[0, 1, 9, 32:64] = 0.0                 # an all-zero group
    Vf[0, 1, 11, 0:32] = np.where(np.arange(32) % 2 == 0, 0.0, -0.0)   # zeros of both signs only
    Vf[0, 1, 12, 0:32] = np.linspace(0, 3, 32)                         # exact ties at .5 do occur here
    K, V = W.to_bits(Kf, "fp16"), W.to_bits(Vf, "fp16")
    st = Q2State(cfg, oracle, K=K, V=V)
    assert st.alpha[0, 0, 5] == 0.0
    dal, kvq = gpu_fit(st)
    assert np.array_equal(dal.cpu().numpy(), st.alpha)
    assert np.array_equal(kvq.cpu().numpy(), st.records())


@pytest.mark.parametrize("dtype,out_f32", [("bf16", True), ("fp16", True), ("bf16", False), ("fp16", False)])
def test_attention_on_records_matches_oracle(oracle, dtype, out_f32):
    cfg = cfg_small(batch=2, n_kv_heads=2, n_q_heads=8, context=3000, top_k=333, dtype=dtype, seed=44)
    st = Q2State(cfg, oracle, seq_len=[3000, 1777], offset_std=0.5, out_dtype=torch.float32 if out_f32 else None)
    kvq = torch.from_numpy(st.records()).cuda()
    dal = torch.from_numpy(st.alpha).cuda()
    q, _, _ = W.make_step_inputs(cfg, 0)
    idx = oracle.topk(oracle.score(q, dtype, st.cb, st.codes, st.sl), st.sl, 333)
    idx[0, 0, 5] = idx[0, 0, 6]              # a repeated entry counts twice
    idx[1, 3, 100:] = -1                     # padding is skipped
    out = torch.empty(2, 8, 128, dtype=torch.float32 if out_f32 else TDT[dtype], device="cuda")
    sik.sik_sparse_attn_q2(st.layout, dev(q, dtype), kvq, dal, torch.from_numpy(idx).cuda(), 333, 0.0, out, st.ws)
    sync()
    ref = oracle.sparse_attn_q2(q, dtype, st.codes, st.qkv, st.alpha, idx)
    check_attention(out.float().cpu().numpy().astype(np.float64), ref, out_f32, dtype)


def test_attention_on_records_all_tokens_and_small_selections(oracle):
    cfg = cfg_small(batch=1, n_kv_heads=2, n_q_heads=4, context=1100, top_k=1100, seed=45)
    st = Q2State(cfg, oracle, out_dtype=torch.float32)
    kvq = torch.from_numpy(st.records()).cuda()
    dal = torch.from_numpy(st.alpha).cuda()
    q, _, _ = W.make_step_inputs(cfg, 1)
    out = torch.empty(1, 4, 128, device="cuda")
    for k, idx in ((1100, np.tile(np.arange(1100, dtype=np.int32), (1, 4, 1))),
                   (1, np.full((1, 4, 1), 17, np.int32)),
                   (40, np.tile(np.arange(1060, 1100, dtype=np.int32)[::-1].copy(), (1, 4, 1))),
                   (5, np.full((1, 4, 5), -1, np.int32))):
        sik.sik_sparse_attn_q2(st.layout, dev(q, cfg.dtype), kvq, dal, torch.from_numpy(idx).cuda(), k, 0.09, out,
                               st.ws)
        sync()
        ref = oracle.sparse_attn_q2(q, cfg.dtype, st.codes, st.qkv, st.alpha, idx, scale=0.09)
        check_attention(out.cpu().numpy().astype(np.float64), ref, True)

"""Parity of the 2-bit token-wise K/V path (records, attention on records, decode step on records) against the
CPU oracle, through the C ABI.

Bars: alpha bit-equal; records against the oracle's fields (the quantisation function in fp64 with true
divisions) under the rule of helpers.records_agree: sign bytes equal, stored parameters and 2-bit codes equal
except where the exact value lies within the library's binary32 rounding error of an fp16 rounding boundary /
of a half-integer of t = (x - zp) / qs (the exceptions are counted and printed; where nothing is near a tie the
records are byte-for-byte the oracle's); attention within the same bars as the 16-bit path (1e-5 relative for
fp32 output) against the oracle's fp64 attention over the dequantised rows of THE SAME records; top-k sets as in
the 16-bit decode step (scoring does not depend on the K/V format).
"""
import numpy as np
import pytest
import torch

import sik_workloads as W
from helpers import dev, records_agree, topk_sets_agree
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


def check_records(st, got, K, V, qkv, codes, ranges, label):
    """got against the oracle's fields on token ranges [(b, t0, t1)]; prints the near-tie exceptions."""
    exc = np.zeros(4, np.int64)
    for b, t0, t1 in ranges:
        exc += records_agree(st.o, got, K, V, st.cfg.dtype, st.mu, st.alpha, codes, qkv, b, t0, t1)
    print(f"{label}: {exc[0]} of {exc[2]} parameters and {exc[1]} of {exc[3]} codes inside the near-tie band")
    return exc


def adopt_appended_records(oracle, kvq, kn, vn, dtype, mu, alpha, codes, qkv, sl):
    """After a decode step that appended token sl[b] - 1 on both sides: the library's record of that token must
    match the oracle's (already in qkv) under the near-tie rule; the oracle then takes over the library's own row,
    so that attention is compared on identical records."""
    B, Hkv = kn.shape[0], kn.shape[1]
    for b in range(B):
        t = int(sl[b]) - 1
        row = np.zeros((B, Hkv, 1, 128), np.uint8)
        row[b] = kvq[b, :, t:t + 1].cpu().numpy()
        records_agree(oracle, row, kn[:, :, None, :], vn[:, :, None, :], dtype, mu, alpha, codes, qkv, b, t, t + 1,
                      base=t)
        _, one = oracle.unpack_records(row[b:b + 1])
        for f in ("kq", "vq", "kpar", "vpar"):
            getattr(qkv, f)[b, :, t] = getattr(one, f)[0, :, 0]


def gpu_fit(st):
    dal = torch.full(st.mu.shape, -1.0, device="cuda")
    kvq = sik.alloc_kvq(st.layout)
    sik.sik_quantize_kv(st.layout, st.dK, st.dV, st.dsl, 0, 0, sik.SIK_Q_FIT, st.dmu, dal, kvq)
    sync()
    return dal, kvq


@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
@pytest.mark.parametrize("offset", [0.0, 1.5])
def test_fit_alpha_and_records_match_oracle(oracle, dtype, offset):
    cfg = cfg_small(batch=2, n_kv_heads=3, n_q_heads=6, context=1337, top_k=64, dtype=dtype, seed=41)
    st = Q2State(cfg, oracle, capacity=1400, seq_len=[1337, 801], offset_std=offset)
    dal, kvq = gpu_fit(st)
    assert np.array_equal(dal.cpu().numpy(), st.alpha)
    got = kvq.cpu().numpy()
    exc = check_records(st, got, st.K, st.V, st.qkv, st.codes, [(b, 0, int(L)) for b, L in enumerate(st.sl)],
                        f"fit {dtype} offset {offset}")
    assert exc[0] <= exc[2] // 500 and exc[1] <= exc[3] // 10000     # a sliver, not a systematic difference
    for b, L in enumerate(st.sl):
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
    got = kvq.cpu().numpy()
    check_records(st, got, K2, V2, qkv, codes, [(0, 0, 633), (1, 0, 633)], "encode range")
    assert not got[:, :, 633:].any()
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
    got = kvq.cpu().numpy()
    check_records(st, got, K, V, st.qkv, st.codes, [(0, 0, 130)], "degenerate groups")
    # the planted groups are exact in any precision: constant row, zero group, zeros of both signs, the ramp with
    # its exact ties
    _, g = oracle.unpack_records(got)
    for (h, t, sl_) in ((0, 3, slice(0, 128)), (1, 9, slice(32, 64)), (1, 11, slice(0, 32)), (1, 12, slice(0, 32))):
        assert np.array_equal(g.vq[0, h, t, sl_], st.qkv.vq[0, h, t, sl_])
        gs = slice(sl_.start // 32, sl_.stop // 32)
        assert np.array_equal(g.vpar[0, h, t, gs], st.qkv.vpar[0, h, t, gs])
    assert not g.vpar[0, 0, 3, :, 0].any() and not g.vq[0, 0, 3].any()      # qs = 0 -> Q = 0
    assert not g.kq[0, 0, :, 5].any()        # dead channel: x = 0


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


# --------------------------------------------------------------------------- decode step on records
# launches = 1: the one-launch step on records whenever its plan allows (the library picks it for large launches only)
BOTH_PATHS = pytest.mark.parametrize("launches", [0, 1], ids=["auto", "one_launch"])


def run_decode_q2_and_check(oracle, cfg, capacity, steps, append, offset_std=0.0, seq_len=None, out_f32=True,
                            launches=0):
    st = Q2State(cfg, oracle, capacity=capacity, seq_len=seq_len, offset_std=offset_std,
                 out_dtype=torch.float32 if out_f32 else None)
    B, Hq, k = cfg.batch, cfg.n_q_heads, min(cfg.top_k, capacity)
    kvq = torch.from_numpy(st.records()).cuda()
    dal = torch.from_numpy(st.alpha).cuda()
    sl, codes, qkv = st.sl.copy(), st.codes, st.qkv
    out = torch.empty(B, Hq, 128, dtype=torch.float32 if out_f32 else TDT[cfg.dtype], device="cuda")
    idx = torch.empty(B, Hq, k, dtype=torch.int32, device="cuda")
    total_diff = 0
    for step in range(steps):
        q, kn, vn = W.make_step_inputs(cfg, step)
        dkn = dev(kn, cfg.dtype) if append else None
        dvn = dev(vn, cfg.dtype) if append else None
        if launches == 0:
            sik.sik_decode_step_q2(st.layout, dev(q, cfg.dtype), dkn, dvn, kvq, st.dsl, st.dmu, dal, st.dcb, st.dcodes,
                                   k, 0.0, out, idx, st.ws)
        else:
            sik.sik_decode_step_ex(st.layout, q=dev(q, cfg.dtype), k_new=dkn, v_new=dvn, kvq=kvq, alpha=dal,
                                   seq_len=st.dsl, mu=st.dmu, codebook=st.dcb, codes=st.dcodes, k=k, out=out,
                                   idx_out=idx, workspace=st.ws, launches=launches)
        sync()
        assert sik.sik_workspace_status(st.ws) == 0
        ref_out, ref_idx = oracle.decode_step_q2(q, kn if append else None, vn if append else None, cfg.dtype, sl,
                                                 st.mu, st.alpha, st.cb, codes, qkv, k)
        assert np.array_equal(st.dsl.cpu().numpy(), sl)
        if append:
            adopt_appended_records(oracle, kvq, kn, vn, cfg.dtype, st.mu, st.alpha, codes, qkv, sl)
            for b in range(B):
                t = int(sl[b]) - 1
                assert np.array_equal(st.dcodes[b, :, t].cpu().numpy(), codes[b, :, t])
        g_idx = idx.cpu().numpy()
        s_ref = oracle.score(q, cfg.dtype, st.cb, codes, sl)
        for b in range(B):
            for hq in range(Hq):
                total_diff += topk_sets_agree(g_idx[b, hq], ref_idx[b, hq], s_ref[b, hq], int(sl[b]), k)
        ref_on_gpu_set = oracle.sparse_attn_q2(q, cfg.dtype, codes, qkv, st.alpha, g_idx)
        check_attention(out.float().cpu().numpy().astype(np.float64), ref_on_gpu_set, out_f32, cfg.dtype)
    return total_diff


@BOTH_PATHS
def test_decode_q2_c1_full(oracle, launches):
    run_decode_q2_and_check(oracle, W.CONFIGS["C1"], capacity=4096, steps=2, append=False, launches=launches)


@BOTH_PATHS
def test_decode_q2_c1_16bit_out(oracle, launches):
    run_decode_q2_and_check(oracle, W.CONFIGS["C1"], capacity=4096, steps=1, append=False, out_f32=False, launches=launches)


@BOTH_PATHS
def test_decode_q2_c2_shape_reduced(oracle, launches):
    run_decode_q2_and_check(oracle, cfg_small("C2", context=8192, top_k=256), capacity=8192, steps=2, append=False,
                            offset_std=1.0, launches=launches)


@BOTH_PATHS
def test_decode_q2_c3_shape_reduced_with_append(oracle, launches):
    run_decode_q2_and_check(oracle, cfg_small("C3", context=9000, top_k=300), capacity=9004, steps=3, append=True,
                            offset_std=1.0, launches=launches)


@BOTH_PATHS
def test_decode_q2_c4_shape_reduced_ragged_batch(oracle, launches):
    run_decode_q2_and_check(oracle, cfg_small("C4", batch=4, context=2048, top_k=512), capacity=2050, steps=1,
                            append=True, seq_len=[2048, 1, 511, 700], launches=launches)


@BOTH_PATHS
def test_decode_q2_c5_shape_reduced_gqa8_fp16(oracle, launches):
    cfg = cfg_small("C5", batch=2, n_kv_heads=2, n_q_heads=16, context=6000, top_k=1536, dtype="fp16")
    run_decode_q2_and_check(oracle, cfg, capacity=6016, steps=3, append=True, launches=launches)


@BOTH_PATHS
def test_decode_q2_dense_selection_and_k_above_context(oracle, launches):
    run_decode_q2_and_check(oracle, cfg_small("C2", context=20000, top_k=20000), capacity=20000, steps=1, append=False, launches=launches)
    run_decode_q2_and_check(oracle, cfg_small("C2", n_kv_heads=2, n_q_heads=8, context=700, top_k=1024),
                            capacity=1100, steps=1, append=True, launches=launches)


@BOTH_PATHS
def test_decode_q2_empty_and_single_token_sequences(oracle, launches):
    cfg = cfg_small("C2", batch=3, n_kv_heads=2, n_q_heads=4, context=300, top_k=16)
    run_decode_q2_and_check(oracle, cfg, capacity=320, steps=2, append=True, seq_len=[0, 1, 300], launches=launches)


def test_decode_q2_graph_replay_and_profiled(oracle):
    cfg = cfg_small("C2", context=20000, top_k=600)
    st = Q2State(cfg, oracle, capacity=20008, out_dtype=torch.float32)
    kvq = torch.from_numpy(st.records()).cuda()
    dal = torch.from_numpy(st.alpha).cuda()
    q, kn, vn = W.make_step_inputs(cfg, 0)
    dq, dkn, dvn = dev(q, cfg.dtype), dev(kn, cfg.dtype), dev(vn, cfg.dtype)
    out = torch.empty(1, 32, 128, device="cuda")
    idx = torch.empty(1, 32, 600, dtype=torch.int32, device="cuda")

    def body(prof=False):
        st.dsl.fill_(20000)
        return sik.sik_decode_step_q2(st.layout, dq, dkn, dvn, kvq, st.dsl, st.dmu, dal, st.dcb, st.dcodes, 600, 0.0,
                                      out, idx, st.ws, profiled=prof)

    body()
    sync()
    eager_out, eager_idx = out.clone(), torch.sort(idx, dim=-1).values.clone()
    assert int(st.dsl[0]) == 20001
    us = body(prof=True)
    assert len(us) == 5 and us[1] > 0 and us[3] > 0 and torch.equal(out, eager_out)
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        body()
        sync()
        with torch.cuda.graph(g, stream=side):
            body()
    sync()
    for r in range(3):
        out.zero_()
        idx.fill_(-3)
        st.dsl.fill_(123)
        torch.randn(1 << 20, device="cuda").sum().item()
        g.replay()
        sync()
        assert int(st.dsl[0]) == 20001
        assert torch.equal(out, eager_out), r
        assert torch.equal(torch.sort(idx, dim=-1).values, eager_idx), r


@pytest.mark.parametrize("forced", [False, True])
def test_decode_q2_one_launch_graph_replay_with_append(oracle, forced):
    # the one-launch step on records (and with a forced set that names the appended token) under graph replay: its
    # counters are left at zero by every replay, the appended record and the published length are the eager ones
    cfg = cfg_small("C3", context=20000, top_k=600)
    st = Q2State(cfg, oracle, capacity=20008, out_dtype=torch.float32)
    kvq0 = torch.from_numpy(st.records()).cuda()
    kvq, dal = kvq0.clone(), torch.from_numpy(st.alpha).cuda()
    q, kn, vn = W.make_step_inputs(cfg, 0)
    dq, dkn, dvn = dev(q, cfg.dtype), dev(kn, cfg.dtype), dev(vn, cfg.dtype)
    out = torch.empty(1, 32, 128, device="cuda")
    idx = torch.empty(1, 32, 600, dtype=torch.int32, device="cuda")
    fidx = None
    if forced:
        f = np.tile(np.arange(0, 64 * 300, 300, dtype=np.int32), (1, 8, 1))
        f[:, :, 0] = 20000                       # the token being appended
        fidx = torch.from_numpy(f).cuda()

    def body(launches=1):
        st.dsl.fill_(20000)
        sik.sik_decode_step_ex(st.layout, q=dq, k_new=dkn, v_new=dvn, kvq=kvq, alpha=dal, seq_len=st.dsl, mu=st.dmu,
                               codebook=st.dcb, codes=st.dcodes, k=600, out=out, idx_out=idx, workspace=st.ws,
                               forced_idx=fidx, launches=launches)

    body(launches=2)
    sync()
    ref_out, ref_idx, ref_rec = out.clone(), torch.sort(idx, dim=-1).values.clone(), kvq[:, :, 20000].clone()
    kvq.copy_(kvq0)
    body()
    sync()
    assert sik.sik_workspace_status(st.ws) == 0 and int(st.dsl[0]) == 20001
    eager_out = out.clone()
    assert torch.equal(torch.sort(idx, dim=-1).values, ref_idx) and torch.equal(kvq[:, :, 20000], ref_rec)
    assert float((eager_out - ref_out).abs().max()) <= 2e-5 * float(ref_out.abs().max())
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        body()
        sync()
        with torch.cuda.graph(g, stream=side):
            body()
    sync()
    for r in range(3):
        out.zero_()
        idx.fill_(-3)
        kvq.copy_(kvq0)
        torch.randn(1 << 20, device="cuda").sum().item()
        g.replay()
        sync()
        assert sik.sik_workspace_status(st.ws) == 0 and int(st.dsl[0]) == 20001
        assert torch.equal(out, eager_out), r
        assert torch.equal(torch.sort(idx, dim=-1).values, ref_idx), r
        assert torch.equal(kvq[:, :, 20000], ref_rec), r


def test_decode_q2_rejects_contexts_without_a_fused_plan(oracle):
    lay = sik.make_layout(1, 1, 1, 128, 600000, torch.bfloat16, torch.float32)
    ws = sik.alloc_workspace(lay, 16)
    t = torch.zeros(16, device="cuda")
    with pytest.raises(sik.SikError) as e:
        sik.sik_decode_step_q2(lay, t, None, None, t, t, t, t, t, t, 16, 0.0, t, None, ws)
    assert e.value.status == -2


# --------------------------------------------------------------------------- prefill-compress in one call
@pytest.mark.parametrize("dtype,seq_len", [("bf16", [5000, 1337, 1, 0]), ("fp16", [4099, 4100, 777, 64])])
def test_prefill_compress_equals_the_separate_calls_and_the_oracle(oracle, dtype, seq_len):
    # one call, two passes over K and one over V: every output has the bits of sik_quantize_keys FIT followed by
    # sik_quantize_kv FIT, and agrees with the oracle as those do
    cfg = cfg_small(batch=4, n_kv_heads=3, n_q_heads=6, context=max(seq_len), top_k=64, dtype=dtype, seed=47)
    st = Q2State(cfg, oracle, capacity=max(seq_len) + 20, seq_len=seq_len, offset_std=1.2)
    B, H, cap = 4, 3, max(seq_len) + 20

    def fresh():
        return (torch.full((B, H, 128), -3.0, device="cuda"), torch.full((B, H, 32, 16, 4), -3.0, device="cuda"),
                torch.full((B, H, 32, 16), -3, dtype=torch.int32, device="cuda"),
                torch.zeros(B, H, cap, 16, dtype=torch.uint8, device="cuda"), torch.full((B, H, 128), -3.0, device="cuda"),
                sik.alloc_kvq(st.layout))

    mu1, cb1, cnt1, codes1, al1, rec1 = fresh()
    sik.sik_quantize_keys(st.layout, st.dK, st.dsl, 0, 0, sik.SIK_Q_FIT, mu1, cb1, cnt1, codes1, st.ws)
    sik.sik_quantize_kv(st.layout, st.dK, st.dV, st.dsl, 0, 0, sik.SIK_Q_FIT, mu1, al1, rec1)
    mu2, cb2, cnt2, codes2, al2, rec2 = fresh()
    sik.sik_prefill_compress(st.layout, st.dK, st.dV, st.dsl, mu2, cb2, cnt2, codes2, al2, rec2, st.ws)
    sync()
    for name, a, b in (("mu", mu1, mu2), ("codebook", cb1, cb2), ("counts", cnt1, cnt2), ("codes", codes1, codes2),
                       ("alpha", al1, al2), ("records", rec1, rec2)):
        assert torch.equal(a, b), name
    assert np.array_equal(mu2.cpu().numpy(), st.mu) and np.array_equal(al2.cpu().numpy(), st.alpha)
    assert np.array_equal(cnt2.cpu().numpy(), oracle.fit(st.K, dtype, st.sl)[3])
    got = rec2.cpu().numpy()
    check_records(st, got, st.K, st.V, st.qkv, st.codes, [(b, 0, int(L)) for b, L in enumerate(st.sl)],
                  f"prefill-compress {dtype}")
    for b, L in enumerate(st.sl):
        assert np.array_equal(codes2[b, :, :L].cpu().numpy(), st.codes[b, :, :L])
        assert not got[b, :, L:].any() and not codes2[b, :, L:].any()


def test_prefill_compress_argument_errors():
    lay = sik.make_layout(1, 2, 4, 128, 512, torch.bfloat16)
    ws = sik.alloc_workspace(lay, 0)
    t = torch.zeros(16, device="cuda")
    with pytest.raises(sik.SikError) as e:
        sik.sik_prefill_compress(lay, t, None, t, t, t, t, t, t, t, ws)
    assert e.value.status == -1
    with pytest.raises(sik.SikError) as e:
        sik.sik_prefill_compress(lay, t, t, t, t, t, t, t, t, t, torch.zeros(256, dtype=torch.uint8, device="cuda"))
    assert e.value.status == -6

"""Parity of the HIP library (through the C ABI) against the CPU oracle, stage by stage and fused.

Bars (written here as the tests use them):
  codes            byte-for-byte equal given the same mu
  mu               |mu_gpu - mu_ref| <= 1e-6 * max(1, max|K_d|)
  codebook         |c_gpu - c_ref| <= 1e-5 * max_i |K'_{i,d}| per channel, counts equal
  scores           |s_gpu - s_ref| <= 1e-5 * max(|s_ref|, RMS(s_ref))
  top-k            identical sets except oracle ties within 1e-5 relative of the k-th score
  attention fp32   max|d| / max|out_ref| <= 1e-5 per (b, hq)
  attention 16-bit max|d| <= 2e-3, or the correctly rounded 16-bit value where the 16-bit grid is
                   coarser than 2e-3 (bf16 half-ulp is 3.9e-3 at |x| = 1): |d| <= half-ulp + 1e-5 max|ref|
"""
import numpy as np
import pytest
import torch

import sik_workloads as W
from helpers import bits_of_tensor, check_attention, dev, f64, half_ulp, topk_sets_agree  # noqa: F401

pytestmark = pytest.mark.gpu

import paper_2603_14224_amd as sik  # noqa: E402

TDT = {"fp16": torch.float16, "bf16": torch.bfloat16}


def cfg_small(name="C2", **kw):
    return W.scaled(W.CONFIGS[name], **kw)


class GpuState:
    """Device mirror of one layer's cache plus the oracle's quantiser state for it."""

    def __init__(self, cfg, oracle, capacity=None, seq_len=None, offset_std=0.0, out_dtype=None):
        self.cfg, self.o = cfg, oracle
        self.K, self.V = W.make_cache(cfg, capacity=capacity, channel_offset_std=offset_std)
        B, H, cap, D = self.K.shape
        self.cap = cap
        self.sl = np.full(B, cfg.context, np.int32) if seq_len is None else np.asarray(seq_len, np.int32)
        self.mu, self.codes, self.cb, self.cnt = oracle.fit(self.K, cfg.dtype, self.sl)
        self.layout = sik.make_layout(B, H, cfg.n_q_heads, D, cap, TDT[cfg.dtype], out_dtype)
        self.dK, self.dV = dev(self.K, cfg.dtype), dev(self.V, cfg.dtype)
        self.dsl = torch.from_numpy(self.sl.copy()).cuda()
        self.dmu = torch.from_numpy(self.mu).cuda()
        self.dcb = torch.from_numpy(self.cb).cuda()
        self.dcodes = torch.from_numpy(self.codes).cuda()
        self.ws = sik.alloc_workspace(self.layout, min(cfg.top_k, cap))


def sync():
    torch.cuda.synchronize()


# --------------------------------------------------------------------------- quantiser
@pytest.mark.parametrize("dtype", ["fp16", "bf16"])
def test_encode_codes_bit_exact(oracle, dtype):
    cfg = cfg_small(batch=2, n_kv_heads=3, n_q_heads=6, context=1237, dtype=dtype, seed=21)
    K, _ = W.make_cache(cfg, capacity=1300, channel_offset_std=2.0)
    sl = np.array([1237, 1237], np.int32)
    mu = oracle.mean(K, dtype, sl)
    lay = sik.make_layout(2, 3, 6, 128, 1300, TDT[dtype])
    dK, dmu = dev(K, dtype), torch.from_numpy(mu).cuda()
    for t0, n in ((0, 1237), (5, 1), (100, 999), (1299, 1), (17, 0)):
        want = np.full((2, 3, 1300, 16), 0x5A, np.uint8)
        oracle.encode(K, dtype, mu, t0, n, want)
        got = torch.full((2, 3, 1300, 16), 0x5A, dtype=torch.uint8, device="cuda")
        sik.sik_quantize_keys(lay, dK, None, t0, n, sik.SIK_Q_ENCODE, dmu, None, None, got, None)
        sync()
        assert np.array_equal(got.cpu().numpy(), want), (t0, n)


@pytest.mark.parametrize("dtype,offset", [("bf16", 0.0), ("bf16", 2.0), ("fp16", 2.0)])
def test_fit_mu_codes_codebook(oracle, dtype, offset):
    cfg = cfg_small(batch=2, n_kv_heads=4, n_q_heads=8, context=5000, dtype=dtype, seed=22)
    K, _ = W.make_cache(cfg, capacity=5003, channel_offset_std=offset)
    sl = np.array([5000, 1531], np.int32)
    mu, codes, cb, cnt = oracle.fit(K, dtype, sl)
    lay = sik.make_layout(2, 4, 8, 128, 5003, TDT[dtype])
    ws = sik.alloc_workspace(lay, 0)
    dK, dsl = dev(K, dtype), torch.from_numpy(sl).cuda()
    dmu = torch.empty(2, 4, 128, device="cuda")
    dcb = torch.empty(2, 4, 32, 16, 4, device="cuda")
    dcnt = torch.empty(2, 4, 32, 16, dtype=torch.int32, device="cuda")
    dcodes = torch.zeros(2, 4, 5003, 16, dtype=torch.uint8, device="cuda")
    sik.sik_quantize_keys(lay, dK, dsl, 0, 0, sik.SIK_Q_FIT, dmu, dcb, dcnt, dcodes, ws)
    sync()
    Kd = f64(K, dtype)
    gmu = dmu.cpu().numpy()
    assert np.abs(gmu - mu).max() <= 1e-6 * max(1.0, np.abs(Kd).max())
    # fp64 accumulation on both sides: the fp32 means are expected to be the same bits
    n_mu_diff = int((gmu != mu).sum())
    gcodes = dcodes.cpu().numpy()
    mism = 0
    for b in range(2):
        mism += int((gcodes[b, :, :sl[b]] != codes[b, :, :sl[b]]).sum())
        assert not gcodes[b, :, sl[b]:].any()  # tokens beyond seq_len untouched
    print(f"fit: mu entries differing {n_mu_diff}, code bytes differing {mism}")
    assert n_mu_diff == 0 and mism == 0
    assert np.array_equal(dcnt.cpu().numpy(), cnt)
    gcb = dcb.cpu().numpy()
    for b in range(2):
        Kp = np.abs(Kd[b, :, :sl[b]] - mu[b][:, None, :]).max(axis=1)  # [H, D] max |K'|
        tol = 1e-5 * Kp.reshape(4, 32, 1, 4)
        assert np.all(np.abs(gcb[b] - cb[b]) <= tol)


# --------------------------------------------------------------------------- scores
@pytest.mark.parametrize("name,kw", [
    ("C1", dict(context=4096)),
    ("C2", dict(batch=2, n_kv_heads=2, n_q_heads=8, context=3001)),
    ("C5", dict(batch=1, n_kv_heads=2, n_q_heads=16, context=2500)),      # GQA 8:1 -> two tables
    ("C2", dict(batch=1, n_kv_heads=2, n_q_heads=6, context=777)),        # R = 3: padded head block
    ("C2", dict(batch=1, n_kv_heads=1, n_q_heads=12, context=600)),       # R = 12: two head blocks
])
def test_scores(oracle, name, kw):
    cfg = cfg_small(name, **kw)
    B = cfg.batch
    sl = np.full(B, cfg.context, np.int32)
    if B > 1:
        sl[1] = cfg.context // 3
    st = GpuState(cfg, oracle, capacity=cfg.context + 5, seq_len=sl, offset_std=1.0)
    q, _, _ = W.make_step_inputs(cfg, 0)
    ref = oracle.score(q, cfg.dtype, st.cb, st.codes, sl)
    got = torch.full((B, cfg.n_q_heads, st.cap), 123.0, device="cuda")
    sik.sik_score(st.layout, dev(q, cfg.dtype), st.dcb, st.dcodes, st.dsl, got)
    sync()
    got = got.cpu().numpy()
    for b in range(B):
        for hq in range(cfg.n_q_heads):
            r = ref[b, hq, :sl[b]]
            tol = 1e-5 * np.maximum(np.abs(r), np.sqrt(np.mean(r * r)))
            assert np.all(np.abs(got[b, hq, :sl[b]] - r) <= tol)
            assert np.all(got[b, hq, sl[b]:] == 123.0)  # not written beyond seq_len


# --------------------------------------------------------------------------- top-k
def run_topk(scores_np, sl, k):
    B, Hq, Lmax = scores_np.shape
    lay = sik.make_layout(B, 1, Hq, 128, Lmax, torch.bfloat16)
    ws = sik.alloc_workspace(lay, k)
    idx = torch.full((B, Hq, k), -7, dtype=torch.int32, device="cuda")
    sik.sik_topk(lay, torch.from_numpy(scores_np).cuda(), torch.from_numpy(np.asarray(sl, np.int32)).cuda(), k, idx, ws)
    sync()
    return idx.cpu().numpy()


@pytest.mark.parametrize("L,k", [(5000, 128), (5000, 1), (5000, 4999), (5000, 5000), (300, 512), (70001, 2048)])
def test_topk_random_scores(oracle, L, k):
    rng = np.random.default_rng(L + k)
    Lmax = max(L, k) + 3
    s = rng.normal(size=(2, 3, Lmax)).astype(np.float32)
    s[0, 1] *= 1e-3
    s[1, 2] = s[1, 2] * 50 + 1000      # far from zero: bins must resolve a narrow relative range
    sl = [L, max(1, L // 2)]
    got = run_topk(s, sl, k)
    ref = oracle.topk(s.astype(np.float64), np.asarray(sl, np.int32), k)
    for b in range(2):
        for h in range(3):
            # identical fp32 scores on both sides: the sets must be identical
            assert sorted(got[b, h].tolist()) == sorted(ref[b, h].tolist())


def test_topk_ties_and_degenerate_rows(oracle):
    rng = np.random.default_rng(77)
    L, k = 6000, 200
    s = rng.normal(size=(1, 6, L)).astype(np.float32)
    s[0, 0] = 1.25                                   # all equal: threshold bin holds everything
    s[0, 1] = np.where(rng.random(L) < 0.5, 2.0, -1.0)  # two values, thousands of ties at the cut
    s[0, 2, :] = np.round(s[0, 2] * 4) / 4           # heavy quantisation: many exact ties
    s[0, 3, 100:1500] = s[0, 3].max() + 1.0          # a plateau of 1400 ties above everything else
    s[0, 4] = 0.0
    s[0, 4, ::7] = -0.0                              # signed zeros compare equal
    s[0, 5, :] = np.arange(L, dtype=np.float32)      # strictly increasing
    got = run_topk(s, [L], k)
    ref = oracle.topk(s.astype(np.float64), np.array([L], np.int32), k)
    for h in range(6):
        assert sorted(got[0, h].tolist()) == sorted(ref[0, h].tolist()), h


def test_topk_is_deterministic(oracle):
    rng = np.random.default_rng(5)
    s = rng.normal(size=(1, 4, 40000)).astype(np.float32)
    a = np.sort(run_topk(s, [40000], 1024), axis=-1)
    for _ in range(3):
        assert np.array_equal(np.sort(run_topk(s, [40000], 1024), axis=-1), a)


def test_topk_many_rows_long_context_crowded_bins(oracle):
    # 512 rows of 70000 scores: enough rows for one histogram workgroup per row, whose range must still be cut
    # into chunks of at most 64512 tokens (the chunk histograms count in 16 bits): all scores equal, and all
    # but one equal with the bins spread by an outlier, put 70000 tokens into one bin
    L, k = 70000, 300
    assert sik.sik_plan_info(sik.make_layout(64, 1, 8, 128, L, torch.bfloat16))[3:5] == [2, 64512]
    rng = np.random.default_rng(11)
    s = np.zeros((64, 8, L), np.float32)
    s[0, 1] = 3.5
    s[0, 2, 69999] = 100.0
    s[0, 3, 5] = -100.0
    s[1] = rng.normal(size=(8, L)).astype(np.float32)
    s[2:] = np.round(rng.normal(size=(1, 8, L)) * 8).astype(np.float32)       # a few dozen distinct values
    sl = np.full(64, L, np.int32)
    sl[5], sl[6] = 64513, 65536
    got = run_topk(s, sl.tolist(), k)
    ref = oracle.topk(s.astype(np.float64), sl, k)
    assert np.array_equal(np.sort(got, -1), np.sort(ref, -1))


def test_topk_empty_sequence(oracle):
    s = np.zeros((2, 2, 64), np.float32)
    got = run_topk(s, [0, 64], 16)
    assert np.all(got[0] == -1)
    assert sorted(got[1, 0].tolist()) == list(range(16))


# --------------------------------------------------------------------------- attention
@pytest.mark.parametrize("dtype,out_f32", [("bf16", True), ("fp16", True), ("bf16", False), ("fp16", False)])
def test_sparse_attention_on_oracle_indices(oracle, dtype, out_f32):
    cfg = cfg_small(batch=2, n_kv_heads=2, n_q_heads=8, context=3000, top_k=333, dtype=dtype, seed=31)
    st = GpuState(cfg, oracle, capacity=3010, out_dtype=torch.float32 if out_f32 else None)
    q, _, _ = W.make_step_inputs(cfg, 0)
    rng = np.random.default_rng(2)
    k = 333
    idx = np.stack([[rng.permutation(3000)[:k] for _ in range(8)] for _ in range(2)]).astype(np.int32)
    idx[0, 1, 300:] = -1          # padded row
    idx[1, 0, :] = -1             # empty selection
    idx[1, 2, 5] = idx[1, 2, 6]   # a repeated entry counts twice
    ref = oracle.sparse_attn(q, st.K, st.V, dtype, idx)
    out = torch.empty(2, 8, 128, dtype=torch.float32 if out_f32 else TDT[dtype], device="cuda")
    sik.sik_sparse_attn(st.layout, dev(q, dtype), st.dK, st.dV, torch.from_numpy(idx).cuda(), k, 0.0, out, st.ws)
    sync()
    got = out.float().cpu().numpy().astype(np.float64)
    check_attention(got, ref, out_f32, dtype)
    assert np.all(got[1, 0] == 0)


def test_sparse_attention_all_tokens_matches_dense(oracle):
    # k = L: the sparse kernel must reproduce dense attention (oracle pinned to the textbook form)
    cfg = cfg_small(batch=1, n_kv_heads=2, n_q_heads=4, context=1500, top_k=1500, seed=32)
    st = GpuState(cfg, oracle, out_dtype=torch.float32)
    q, _, _ = W.make_step_inputs(cfg, 0)
    idx = np.tile(np.arange(1500, dtype=np.int32), (1, 4, 1))
    ref = oracle.sparse_attn(q, st.K, st.V, cfg.dtype, idx, scale=0.11)
    out = torch.empty(1, 4, 128, device="cuda")
    sik.sik_sparse_attn(st.layout, dev(q, cfg.dtype), st.dK, st.dV, torch.from_numpy(idx).cuda(), 1500, 0.11, out, st.ws)
    sync()
    check_attention(out.cpu().numpy().astype(np.float64), ref, True)


# --------------------------------------------------------------------------- fused decode step
# launches = 0: the path the library picks for the layout (small launches: scoring, then selection + attention);
# launches = 1: the one-launch step whenever its plan allows, so that the reduced shapes below exercise it too;
# launches = 3: the one-launch step with its first scoring pass in 16-bit fixed point.
BOTH_PATHS = pytest.mark.parametrize("launches", [0, 1, 3], ids=["auto", "one_launch", "one_launch_16bit"])


def decode_step(layout, q, k_new, v_new, K, V, seq_len, mu, cb, codes, k, out, idx, ws, launches=0):
    if launches == 0:
        sik.sik_decode_step(layout, q, k_new, v_new, K, V, seq_len, mu, cb, codes, k, 0.0, out, idx, ws)
    else:
        sik.sik_decode_step_ex(layout, q=q, k_new=k_new, v_new=v_new, K=K, V=V, seq_len=seq_len, mu=mu, codebook=cb,
                               codes=codes, k=k, out=out, idx_out=idx, workspace=ws, launches=launches)


def run_decode_and_check(oracle, cfg, capacity, steps, append, offset_std=0.0, seq_len=None, out_f32=True,
                         sample_rows=None, launches=0):
    st = GpuState(cfg, oracle, capacity=capacity, seq_len=seq_len, offset_std=offset_std,
                  out_dtype=torch.float32 if out_f32 else None)
    B, Hq, k = cfg.batch, cfg.n_q_heads, min(cfg.top_k, capacity)
    K, V, codes, sl = st.K, st.V, st.codes, st.sl.copy()
    out = torch.empty(B, Hq, 128, dtype=torch.float32 if out_f32 else TDT[cfg.dtype], device="cuda")
    idx = torch.empty(B, Hq, k, dtype=torch.int32, device="cuda")
    total_diff = 0
    for step in range(steps):
        q, kn, vn = W.make_step_inputs(cfg, step)
        dq = dev(q, cfg.dtype)
        dkn = dev(kn, cfg.dtype) if append else None
        dvn = dev(vn, cfg.dtype) if append else None
        decode_step(st.layout, dq, dkn, dvn, st.dK, st.dV, st.dsl, st.dmu, st.dcb, st.dcodes, k, out, idx, st.ws,
                    launches)
        sync()
        assert sik.sik_workspace_status(st.ws) == 0
        # oracle: same step on the host copies (appends in place)
        if append:
            ref_out, ref_idx = oracle.decode_step(q, kn, vn, K, V, cfg.dtype, sl, st.mu, st.cb, codes, k)
        else:
            ref_out, ref_idx = oracle.decode_step(q, None, None, K, V, cfg.dtype, sl, st.mu, st.cb, codes, k)
        assert np.array_equal(st.dsl.cpu().numpy(), sl)
        if append:
            for b in range(B):
                t = sl[b] - 1
                assert np.array_equal(bits_of_tensor(st.dK[b, :, t]), K[b, :, t])
                assert np.array_equal(bits_of_tensor(st.dV[b, :, t]), V[b, :, t])
                assert np.array_equal(st.dcodes[b, :, t].cpu().numpy(), codes[b, :, t])
        g_idx = idx.cpu().numpy()
        s_ref = oracle.score(q, cfg.dtype, st.cb, codes, sl)
        for b in range(B):
            for hq in range(Hq):
                total_diff += topk_sets_agree(g_idx[b, hq], ref_idx[b, hq], s_ref[b, hq], int(sl[b]), k)
        # attention is compared on the GPU's own (tie-legal) index set
        ref_on_gpu_set = oracle.sparse_attn(q, K, V, cfg.dtype, g_idx)
        check_attention(out.float().cpu().numpy().astype(np.float64), ref_on_gpu_set, out_f32, cfg.dtype)
    return total_diff


@BOTH_PATHS
def test_decode_step_c1_full(oracle, launches):
    cfg = W.CONFIGS["C1"]
    run_decode_and_check(oracle, cfg, capacity=4096, steps=2, append=False, launches=launches)


@BOTH_PATHS
def test_decode_step_c1_16bit_out(oracle, launches):
    run_decode_and_check(oracle, W.CONFIGS["C1"], capacity=4096, steps=1, append=False, out_f32=False, launches=launches)


@BOTH_PATHS
def test_decode_step_c2_shape_reduced(oracle, launches):
    cfg = cfg_small("C2", context=8192, top_k=256)
    run_decode_and_check(oracle, cfg, capacity=8192, steps=2, append=False, offset_std=1.0, launches=launches)


@BOTH_PATHS
def test_decode_step_c3_shape_reduced_with_append(oracle, launches):
    cfg = cfg_small("C3", context=9000, top_k=300)
    run_decode_and_check(oracle, cfg, capacity=9004, steps=3, append=True, offset_std=1.0, launches=launches)


@BOTH_PATHS
def test_decode_step_c4_shape_reduced_ragged_batch(oracle, launches):
    cfg = cfg_small("C4", batch=4, context=2048, top_k=512)
    run_decode_and_check(oracle, cfg, capacity=2050, steps=1, append=True, seq_len=[2048, 1, 511, 700], launches=launches)


@BOTH_PATHS
def test_decode_step_c5_shape_reduced_gqa8(oracle, launches):
    cfg = cfg_small("C5", batch=2, n_kv_heads=2, n_q_heads=16, context=6000, top_k=1536)
    run_decode_and_check(oracle, cfg, capacity=6016, steps=3, append=True, launches=launches)


@BOTH_PATHS
def test_decode_step_k_not_below_context(oracle, launches):
    # k >= L: everything is selected and the result is dense attention
    cfg = cfg_small("C2", n_kv_heads=2, n_q_heads=8, context=700, top_k=1024)
    run_decode_and_check(oracle, cfg, capacity=1100, steps=1, append=True, launches=launches)


@BOTH_PATHS
def test_decode_step_dense_selection_flushes_the_wave_lists(oracle, launches):
    # k = L with 4096-token chunks: every wavefront selects all 1024 tokens of its share, far more than
    # its 512-slot list holds, so the list is gathered and refilled several times
    cfg = cfg_small("C2", context=40000, top_k=40000)
    run_decode_and_check(oracle, cfg, capacity=40000, steps=1, append=False, launches=launches)


@BOTH_PATHS
def test_decode_step_half_selected(oracle, launches):
    # k = L / 2: the threshold sits in the middle of the score distribution
    cfg = cfg_small("C2", n_kv_heads=2, n_q_heads=8, context=30000, top_k=15000)
    run_decode_and_check(oracle, cfg, capacity=30008, steps=1, append=True, launches=launches)


@BOTH_PATHS
def test_decode_step_zero_query_all_scores_equal(oracle, launches):
    # q = 0 makes every score equal: the selector must still return k distinct smallest indices
    cfg = cfg_small("C2", n_kv_heads=1, n_q_heads=4, context=3000, top_k=100)
    st = GpuState(cfg, oracle, out_dtype=torch.float32)
    q = np.zeros((1, 4, 128), np.uint16)
    out = torch.empty(1, 4, 128, device="cuda")
    idx = torch.empty(1, 4, 100, dtype=torch.int32, device="cuda")
    decode_step(st.layout, dev(q, cfg.dtype), None, None, st.dK, st.dV, st.dsl, st.dmu, st.dcb, st.dcodes, 100, out,
                idx, st.ws, launches)
    sync()
    g = idx.cpu().numpy()
    for hq in range(4):
        assert sorted(g[0, hq].tolist()) == list(range(100))
    ref = oracle.sparse_attn(q, st.K, st.V, cfg.dtype, g)
    check_attention(out.cpu().numpy().astype(np.float64), ref, True)


@BOTH_PATHS
@pytest.mark.parametrize("ndup", [40, 300])
def test_decode_step_duplicate_keys_at_threshold(oracle, ndup, launches):
    # identical keys in a row have identical scores; with k chosen so that the cut falls inside that plateau,
    # one wavefront's share of the threshold bin (40 keys), or the shares of wavefronts of two workgroups (300
    # keys), exceed the per-wavefront candidate slots: the surplus travels through the head's overflow pool and
    # the exact ranking must take the smallest indices of the plateau
    cfg = cfg_small("C2", n_kv_heads=1, n_q_heads=4, context=12000, top_k=64)
    K, V = W.make_cache(cfg)
    K[0, 0, 5000:5000 + ndup] = K[0, 0, 5000]
    sl = np.array([12000], np.int32)
    mu, codes, cb, cnt = oracle.fit(K, cfg.dtype, sl)
    q, _, _ = W.make_step_inputs(cfg, 0)
    s_ref = oracle.score(q, cfg.dtype, cb, codes, sl)
    # rank of the first duplicate under each query head; the head that ranks the plateau best sets k
    r0s = [int(np.where(np.lexsort((np.arange(12000), -s_ref[0, h])) == 5000)[0][0]) for h in range(4)]
    hsel = int(np.argmin(r0s))
    k = r0s[hsel] + 20
    assert 20 < k < 12000 - ndup
    lay = sik.make_layout(1, 1, 4, 128, 12000, torch.bfloat16, torch.float32)
    ws = sik.alloc_workspace(lay, k)
    out = torch.empty(1, 4, 128, device="cuda")
    idx = torch.empty(1, 4, k, dtype=torch.int32, device="cuda")
    dsl = torch.from_numpy(sl.copy()).cuda()
    decode_step(lay, dev(q, cfg.dtype), None, None, dev(K, cfg.dtype), dev(V, cfg.dtype), dsl,
                torch.from_numpy(mu).cuda(), torch.from_numpy(cb).cuda(), torch.from_numpy(codes).cuda(), k, out, idx, ws,
                launches)
    sync()
    g = idx.cpu().numpy()
    ref_idx = oracle.topk(s_ref, sl, k)
    # exact, smallest indices of the plateau
    assert sorted(g[0, hsel].tolist()) == sorted(ref_idx[0, hsel].tolist())
    assert set(range(5000, 5020)) <= set(g[0, hsel].tolist()) and 5020 not in set(g[0, hsel].tolist())
    for hq in range(4):
        topk_sets_agree(g[0, hq], ref_idx[0, hq], s_ref[0, hq], 12000, k)
    check_attention(out.cpu().numpy().astype(np.float64), oracle.sparse_attn(q, K, V, cfg.dtype, g), True)


def test_decode_step_very_long_context_takes_the_unfused_path(oracle):
    # above 512K tokens the fused select + attention kernel would need more than 64 chunks of 8192:
    # the decode step then runs select_kernel + attn_kernel (also the 64-chunk limit of the histograms)
    cfg = cfg_small("C2", n_kv_heads=1, n_q_heads=2, context=530000, top_k=3000)
    run_decode_and_check(oracle, cfg, capacity=530004, steps=1, append=True)


@BOTH_PATHS
def test_decode_step_long_context_fused_many_chunks(oracle, launches):
    # 300K tokens: 37 chunks of 8192 in the fused kernel, more than the 32 whose partials the last
    # arriver prefetches; 64 scoring chunks
    cfg = cfg_small("C2", n_kv_heads=1, n_q_heads=4, context=300000, top_k=2048)
    run_decode_and_check(oracle, cfg, capacity=300000, steps=1, append=False, launches=launches)


@BOTH_PATHS
def test_decode_step_empty_and_single_token_sequences(oracle, launches):
    cfg = cfg_small("C2", batch=3, n_kv_heads=2, n_q_heads=4, context=1500, top_k=8)
    st = GpuState(cfg, oracle, capacity=1504, seq_len=[0, 1, 1500], out_dtype=torch.float32)
    q, _, _ = W.make_step_inputs(cfg, 0)
    out = torch.full((3, 4, 128), 7.0, device="cuda")
    idx = torch.full((3, 4, 8), -5, dtype=torch.int32, device="cuda")
    decode_step(st.layout, dev(q, cfg.dtype), None, None, st.dK, st.dV, st.dsl, st.dmu, st.dcb, st.dcodes, 8, out, idx,
                st.ws, launches)
    sync()
    g, o = idx.cpu().numpy(), out.cpu().numpy().astype(np.float64)
    assert np.all(g[0] == -1) and np.all(o[0] == 0)                      # empty sequence: zero rows
    assert np.all(np.sort(g[1], axis=-1)[:, -1] == 0) and np.all(np.sort(g[1], axis=-1)[:, :-1] == -1)
    Vd = W.from_bits(st.V, cfg.dtype).astype(np.float64)
    for hq in range(4):
        assert np.allclose(o[1, hq], Vd[1, hq // 2, 0], rtol=1e-6, atol=1e-7)  # one token: its V row
    ref = oracle.sparse_attn(q, st.K, st.V, cfg.dtype, g)
    check_attention(o[2:3], ref[2:3], True)


@BOTH_PATHS
def test_decode_step_output_is_bit_reproducible(oracle, launches):
    # fixed-order merges and rank-ordered candidates: the same inputs give the same output bits and the
    # same index set on every run, whatever the arrival order of the workgroups
    cfg = cfg_small("C2", context=20000, top_k=700)
    st = GpuState(cfg, oracle, out_dtype=torch.float32)
    q, _, _ = W.make_step_inputs(cfg, 3)
    dq = dev(q, cfg.dtype)
    outs, sets = [], []
    for _ in range(4):
        o = torch.empty(1, 32, 128, device="cuda")
        idx = torch.empty(1, 32, 700, dtype=torch.int32, device="cuda")
        decode_step(st.layout, dq, None, None, st.dK, st.dV, st.dsl, st.dmu, st.dcb, st.dcodes, 700, o, idx, st.ws,
                    launches)
        sync()
        outs.append(o.clone())
        sets.append(torch.sort(idx, dim=-1).values.clone())
    for o, s_ in zip(outs[1:], sets[1:]):
        assert torch.equal(o, outs[0]) and torch.equal(s_, sets[0])


@BOTH_PATHS
def test_decode_step_graph_replay_matches_eager(oracle, launches):
    # the step is captured into a HIP graph (kernels only, no memset nodes) and replayed several times with
    # eager work and synchronisations in between; every replay must reproduce the eager result, including the
    # device-side append (the graph resets the length first, as bench.py does)
    cfg = cfg_small("C3", context=20000, top_k=600)
    st = GpuState(cfg, oracle, capacity=20008, out_dtype=torch.float32)
    q, kn, vn = W.make_step_inputs(cfg, 0)
    dq, dkn, dvn = dev(q, cfg.dtype), dev(kn, cfg.dtype), dev(vn, cfg.dtype)
    out = torch.empty(1, 32, 128, device="cuda")
    idx = torch.empty(1, 32, 600, dtype=torch.int32, device="cuda")

    def body():
        st.dsl.fill_(20000)
        decode_step(st.layout, dq, dkn, dvn, st.dK, st.dV, st.dsl, st.dmu, st.dcb, st.dcodes, 600, out, idx, st.ws,
                    launches)

    body()
    sync()
    eager_out, eager_idx = out.clone(), torch.sort(idx, dim=-1).values.clone()
    assert int(st.dsl[0]) == 20001
    side = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        body()
        sync()
        with torch.cuda.graph(g, stream=side):
            body()
    sync()
    for r in range(4):
        out.zero_()
        idx.fill_(-3)
        st.dsl.fill_(123)                      # eager work between replays
        torch.randn(1 << 20, device="cuda").sum().item()
        g.replay()
        sync()
        assert int(st.dsl[0]) == 20001
        assert torch.equal(out, eager_out), r
        assert torch.equal(torch.sort(idx, dim=-1).values, eager_idx), r


def test_profiled_decode_step_same_result_and_five_intervals(oracle):
    cfg = cfg_small("C2", n_kv_heads=2, n_q_heads=8, context=6000, top_k=128)
    st = GpuState(cfg, oracle, out_dtype=torch.float32)
    q, _, _ = W.make_step_inputs(cfg, 0)
    dq = dev(q, cfg.dtype)
    a, b, c, d = (torch.empty(1, 8, 128, device="cuda") for _ in range(4))
    kw = dict(q=dq, K=st.dK, V=st.dV, seq_len=st.dsl, mu=st.dmu, codebook=st.dcb, codes=st.dcodes, k=128,
              workspace=st.ws)
    sik.sik_decode_step(st.layout, dq, None, None, st.dK, st.dV, st.dsl, st.dmu, st.dcb, st.dcodes, 128, 0.0, a, None, st.ws)
    us = sik.sik_decode_step_profiled(st.layout, dq, None, None, st.dK, st.dV, st.dsl, st.dmu, st.dcb, st.dcodes, 128,
                                      0.0, b, None, st.ws)
    sync()
    # a launch this small runs as scoring, then fused selection + attention (no prep, no stand-alone selector)
    assert len(us) == 5 and us[0] == 0 and us[2] == 0 and 0.5 < us[1] < 1000 and 0.5 < us[3] < 1000
    assert us[1] + us[3] <= us[4] * 1.001         # (the gap may hold the one-time loading of the second kernel)
    assert torch.equal(a, b)
    us2 = sik.sik_decode_step_ex(st.layout, out=c, launches=2, profiled=True, **kw)
    assert us2[0] == 0 and us2[2] == 0 and us2[1] > 0.5 and us2[3] > 0.5 and torch.equal(a, c)
    # forced into one launch: one kernel, reported in the last slot; the span is that kernel
    assert sik.sik_plan_info(st.layout)[7] > 0
    us1 = sik.sik_decode_step_ex(st.layout, out=d, launches=1, profiled=True, **kw)
    assert us1[0] == 0 and us1[1] == 0 and us1[2] == 0 and 0.5 < us1[3] < 1000
    assert abs(us1[4] - us1[3]) <= 0.01 * us1[3] + 0.1
    assert float((a - d).abs().max()) <= 2e-5 * float(a.abs().max())   # each within 1e-5 of the exact result
    assert sik.sik_workspace_status(st.ws) == 0


def test_one_launch_append_with_more_workgroups_than_compute_units(oracle):
    # one chunk per head block: nothing waits, so the grid (40 x 8 = 320 workgroups) may exceed the compute units even
    # when a row is appended; the last workgroup of a sequence to leave publishes its new length
    cfg = cfg_small("C4", batch=40, n_kv_heads=8, n_q_heads=32, context=3000, top_k=128, seed=12)
    st = GpuState(cfg, oracle, capacity=3008, seq_len=[3000 - 7 * (i % 5) for i in range(40)], out_dtype=torch.float32)
    assert sik.sik_plan_info(st.layout)[7] > 0
    q, kn, vn = W.make_step_inputs(cfg, 0)
    dq, dkn, dvn = dev(q, cfg.dtype), dev(kn, cfg.dtype), dev(vn, cfg.dtype)
    res = {}
    for launches in (2, 1):
        dK, dV, dcodes = st.dK.clone(), st.dV.clone(), st.dcodes.clone()
        dsl = torch.from_numpy(st.sl.copy()).cuda()
        out = torch.empty(40, 32, 128, device="cuda")
        idx = torch.empty(40, 32, 128, dtype=torch.int32, device="cuda")
        sik.sik_decode_step_ex(st.layout, q=dq, k_new=dkn, v_new=dvn, K=dK, V=dV, seq_len=dsl, mu=st.dmu,
                               codebook=st.dcb, codes=dcodes, k=128, out=out, idx_out=idx, workspace=st.ws,
                               launches=launches)
        sync()
        assert sik.sik_workspace_status(st.ws) == 0
        res[launches] = (out, torch.sort(idx, dim=-1).values, dK, dV, dcodes, dsl)
    a, b = res[2], res[1]
    assert np.array_equal(b[5].cpu().numpy(), st.sl + 1) and torch.equal(a[5], b[5])
    assert torch.equal(a[1], b[1]) and torch.equal(a[2], b[2]) and torch.equal(a[3], b[3]) and torch.equal(a[4], b[4])
    assert float((a[0] - b[0]).abs().max()) <= 2e-5 * float(a[0].abs().max())


def test_one_launch_bounded_wait_gives_up_and_reports(oracle):
    # The one-launch step waits, inside the kernel, for the histograms of a head's other chunks.  The wait is bounded:
    # with a spin limit of one poll it gives up (forced from the host, every workgroup still runs to its end), the
    # status word of the workspace says so, and after sik_workspace_init the same workspace serves normal steps again.
    cfg = cfg_small("C3", context=20000, top_k=600)
    st = GpuState(cfg, oracle, capacity=20008, out_dtype=torch.float32)
    assert sik.sik_plan_info(st.layout)[7] > 0
    q, kn, vn = W.make_step_inputs(cfg, 0)
    dq, dkn, dvn = dev(q, cfg.dtype), dev(kn, cfg.dtype), dev(vn, cfg.dtype)
    ref = torch.empty(1, 32, 128, device="cuda")
    ref_idx = torch.empty(1, 32, 600, dtype=torch.int32, device="cuda")
    out = torch.empty(1, 32, 128, device="cuda")
    idx = torch.empty(1, 32, 600, dtype=torch.int32, device="cuda")
    kw = dict(q=dq, k_new=dkn, v_new=dvn, K=st.dK, V=st.dV, seq_len=st.dsl, mu=st.dmu, codebook=st.dcb,
              codes=st.dcodes, k=600, workspace=st.ws)
    sik.sik_decode_step_ex(st.layout, out=ref, idx_out=ref_idx, launches=2, **kw)
    sync()
    assert int(st.dsl[0]) == 20001 and sik.sik_workspace_status(st.ws) == 0
    for limit in (1, 0):
        st.dsl.fill_(20000)
        print(f"one-launch step, spin_limit={limit}", flush=True)
        sik.sik_decode_step_ex(st.layout, out=out, idx_out=idx, launches=1, spin_limit=limit, **kw)
        sync()
        status = sik.sik_workspace_status(st.ws)
        if limit == 1:
            assert status & 1, status         # a first arriver cannot see 20 chunks after one poll
            sik.sik_workspace_init(st.layout, 600, st.ws)
            assert sik.sik_workspace_status(st.ws) == 0
        else:
            assert status == 0 and int(st.dsl[0]) == 20001
            assert torch.equal(torch.sort(idx, dim=-1).values, torch.sort(ref_idx, dim=-1).values)
            assert float((out - ref).abs().max()) <= 2e-5 * float(ref.abs().max())


@pytest.mark.parametrize("case", ["plain", "offset", "tiny_range", "two_groups", "huge_offset"])
@pytest.mark.parametrize("shape", ["one_chunk", "five_chunks"])
def test_16bit_first_pass_selects_exactly_the_sets_of_the_fp32_paths(oracle, case, shape):
    # The first pass in 16-bit fixed point only sorts tokens into bins; every token within the guard band of the cut
    # is rescored in binary32 and ranked, so the selected SET must equal that of the other paths bit for bit (all
    # paths sum the same table entries in the same order).  Adversarial tables: a large common offset per group
    # (wide band: the fp32 rounding of the sums dwarfs the fixed-point step), entries that barely differ (every
    # token inside the band), a query that sees two groups only (256 distinct scores: plateaus at the cut).
    if shape == "one_chunk":
        cfg = cfg_small("C4", batch=2, n_kv_heads=2, n_q_heads=8, context=15000, top_k=512, seed=5)
    else:
        cfg = cfg_small("C2", n_kv_heads=2, n_q_heads=8, context=20000, top_k=700, seed=6)
    st = GpuState(cfg, oracle, out_dtype=torch.float32)
    B, Hq, k = cfg.batch, cfg.n_q_heads, cfg.top_k
    q, _, _ = W.make_step_inputs(cfg, 1)
    cb = st.cb.copy()
    if case == "offset":
        cb += 3.0
    elif case == "huge_offset":
        cb += 4000.0
    elif case == "tiny_range":
        m = cb.mean(axis=3, keepdims=True)
        cb = (m + 1e-4 * (cb - m)).astype(np.float32)
    elif case == "two_groups":
        qf = W.from_bits(q, cfg.dtype).copy()
        qf[..., 8:] = 0
        q = W.to_bits(qf, cfg.dtype)
    dq, dcb = dev(q, cfg.dtype), torch.from_numpy(cb).cuda()
    res = {}
    for launches in (2, 1, 3):
        out = torch.empty(B, Hq, 128, device="cuda")
        idx = torch.empty(B, Hq, k, dtype=torch.int32, device="cuda")
        sik.sik_decode_step_ex(st.layout, q=dq, K=st.dK, V=st.dV, seq_len=st.dsl, mu=st.dmu, codebook=dcb,
                               codes=st.dcodes, k=k, out=out, idx_out=idx, workspace=st.ws, launches=launches)
        sync()
        assert sik.sik_workspace_status(st.ws) == 0
        res[launches] = (out, torch.sort(idx, dim=-1).values)
    for launches in (1, 3):
        assert torch.equal(res[launches][1], res[2][1]), (case, launches)
        assert float((res[launches][0] - res[2][0]).abs().max()) <= 2e-5 * float(res[2][0].abs().max())
    # and that set is the oracle's, ties within 1e-5 of the k-th score aside (where the tables carry an offset far
    # above their spread that tolerance says nothing about binary32 sums, and the comparison above is the test)
    if case in ("plain", "two_groups"):
        s_ref = oracle.score(q, cfg.dtype, cb, st.codes, st.sl)
        ref_idx = oracle.topk(s_ref, st.sl, k)
        g = res[3][1].cpu().numpy()
        for b in range(B):
            for hq in range(Hq):
                topk_sets_agree(g[b, hq], ref_idx[b, hq], s_ref[b, hq], int(st.sl[b]), k)


@BOTH_PATHS
def test_decode_step_without_idx_out_matches(oracle, launches):
    cfg = cfg_small("C2", n_kv_heads=2, n_q_heads=8, context=5000, top_k=200)
    st = GpuState(cfg, oracle, out_dtype=torch.float32)
    q, _, _ = W.make_step_inputs(cfg, 0)
    dq = dev(q, cfg.dtype)
    a = torch.empty(1, 8, 128, device="cuda")
    b = torch.empty(1, 8, 128, device="cuda")
    idx = torch.empty(1, 8, 200, dtype=torch.int32, device="cuda")
    decode_step(st.layout, dq, None, None, st.dK, st.dV, st.dsl, st.dmu, st.dcb, st.dcodes, 200, a, idx, st.ws, launches)
    decode_step(st.layout, dq, None, None, st.dK, st.dV, st.dsl, st.dmu, st.dcb, st.dcodes, 200, b, None, st.ws, launches)
    sync()
    assert torch.allclose(a, b, rtol=1e-5, atol=1e-6)

"""Parity of the decode step with forced-inclusion sets (always-attended tokens that stay out of the top-k)
against the CPU oracle, on both cache formats, through sik_decode_step_ex.

Bars as in the plain decode step: every valid forced token is in the index set exactly once; the dynamic part is
the oracle's top-(k - forced) of the remaining tokens up to score ties within 1e-5 relative of its last pick;
attention within 1e-5 relative (fp32 output) of the oracle's on the GPU's own index set.
"""
import numpy as np
import pytest
import torch

import sik_workloads as W
from helpers import dev, topk_sets_agree
from test_gpu_kvq import Q2State, adopt_appended_records
from test_gpu_parity import GpuState, TDT, cfg_small, check_attention, sync

pytestmark = pytest.mark.gpu

import paper_2603_14224_amd as sik  # noqa: E402


def draw_forced(cfg, sl, n_forced, seed, spoil=True):
    rng = np.random.default_rng(seed)
    B, H = cfg.batch, cfg.n_kv_heads
    f = np.full((B, H, n_forced), -1, np.int32)
    for b in range(B):
        for h in range(H):
            m = min(n_forced, int(sl[b]))
            f[b, h, :m] = rng.choice(int(sl[b]), m, replace=False) if m else []
    if spoil and n_forced >= 4:
        f[0, 0, 1] = -1                       # an unused slot
        f[-1, -1, 2] = int(sl[-1]) + 5        # beyond the sequence: names no token
    return f


def check_sets(g_idx, ref_idx, s_ref, forced, sl, k, R):
    """Forced tokens present once; the dynamic part agrees with the oracle's up to ties at its cut."""
    B, Hq = g_idx.shape[:2]
    n_diff = 0
    for b in range(B):
        for hq in range(Hq):
            f = {int(i) for i in forced[b, hq // R] if 0 <= i < sl[b]}
            g = [int(i) for i in g_idx[b, hq] if i >= 0]
            r = [int(i) for i in ref_idx[b, hq] if i >= 0]
            assert len(g) == len(set(g)) == len(r), (b, hq, len(g), len(r))
            assert f <= set(g) and all(0 <= i < sl[b] for i in g)
            diff = (set(g) ^ set(r))
            if diff:
                assert not (diff & f)
                dyn_ref = [i for i in r if i not in f]
                cut = min(s_ref[b, hq, i] for i in dyn_ref)
                for i in diff:
                    assert abs(s_ref[b, hq, i] - cut) <= 1e-5 * abs(cut), (b, hq, i)
                n_diff += len(diff)
    return n_diff


# launches = 1: the one-launch step whenever its plan allows (the library takes it for large launches only)
BOTH_PATHS = pytest.mark.parametrize("launches", [0, 1], ids=["auto", "one_launch"])


def run_rows(oracle, cfg, capacity, steps, append, n_forced, seq_len=None, seed=1, launches=0):
    st = GpuState(cfg, oracle, capacity=capacity, seq_len=seq_len, offset_std=0.8, out_dtype=torch.float32)
    B, Hq, k = cfg.batch, cfg.n_q_heads, cfg.top_k
    R = Hq // cfg.n_kv_heads
    K, V, codes, sl = st.K, st.V, st.codes, st.sl.copy()
    out = torch.empty(B, Hq, 128, device="cuda")
    idx = torch.empty(B, Hq, k, dtype=torch.int32, device="cuda")
    for step in range(steps):
        q, kn, vn = W.make_step_inputs(cfg, step)
        forced = draw_forced(cfg, sl + (1 if append else 0), n_forced, seed + step)
        if append:
            forced[0, 0, 0] = sl[0]           # the token being appended may be forced too ("always included")
        sik.sik_decode_step_ex(st.layout, q=dev(q, cfg.dtype), k_new=dev(kn, cfg.dtype) if append else None,
                               v_new=dev(vn, cfg.dtype) if append else None, K=st.dK, V=st.dV, seq_len=st.dsl,
                               mu=st.dmu, codebook=st.dcb, codes=st.dcodes, k=k, out=out, idx_out=idx,
                               forced_idx=torch.from_numpy(forced).cuda(), workspace=st.ws, launches=launches)
        sync()
        assert sik.sik_workspace_status(st.ws) == 0
        ref_out, ref_idx = oracle.decode_step_forced(q, kn if append else None, vn if append else None, K, V,
                                                     cfg.dtype, sl, st.mu, st.cb, codes, k, forced)
        assert np.array_equal(st.dsl.cpu().numpy(), sl)
        g_idx = idx.cpu().numpy()
        check_sets(g_idx, ref_idx, oracle.score(q, cfg.dtype, st.cb, codes, sl), forced, sl, k, R)
        check_attention(out.cpu().numpy().astype(np.float64), oracle.sparse_attn(q, K, V, cfg.dtype, g_idx), True)


@BOTH_PATHS
def test_forced_rows_c1(oracle, launches):
    run_rows(oracle, W.CONFIGS["C1"], 4096, steps=2, append=False, n_forced=64, launches=launches)


@BOTH_PATHS
def test_forced_rows_c2_shape_with_append(oracle, launches):
    run_rows(oracle, cfg_small("C2", context=9000, top_k=160), 9004, steps=3, append=True, n_forced=64, launches=launches)


@BOTH_PATHS
def test_forced_rows_ragged_batch_gqa8_max_set(oracle, launches):
    cfg = cfg_small("C5", batch=3, n_kv_heads=2, n_q_heads=16, context=5000, top_k=300)
    run_rows(oracle, cfg, 5008, steps=2, append=True, n_forced=128, seq_len=[5000, 40, 777], launches=launches)


@BOTH_PATHS
def test_forced_rows_everything_selected_and_tiny_sequences(oracle, launches):
    # k above the context: forced plus all the others; sequences shorter than the forced set
    cfg = cfg_small("C2", batch=3, n_kv_heads=2, n_q_heads=4, context=600, top_k=700)
    run_rows(oracle, cfg, 704, steps=1, append=False, n_forced=16, seq_len=[600, 5, 0], launches=launches)


@BOTH_PATHS
def test_forced_rows_large_launch(oracle, launches):
    # more than 2 M keys in the launch: the scoring kernel's large-launch workgroups (512 threads, two per
    # compute unit) with the forced-token bitmap, ragged lengths, append
    cfg = cfg_small("C2", batch=5, n_kv_heads=8, n_q_heads=32, context=56000, top_k=300)
    run_rows(oracle, cfg, 56008, steps=1, append=True, n_forced=64, seq_len=[56000, 31000, 56000, 9, 44444], launches=launches)


def test_forced_empty_set_equals_plain_step(oracle):
    cfg = cfg_small("C2", n_kv_heads=2, n_q_heads=8, context=6000, top_k=128)
    st = GpuState(cfg, oracle, out_dtype=torch.float32)
    q, _, _ = W.make_step_inputs(cfg, 0)
    a, b_ = torch.empty(1, 8, 128, device="cuda"), torch.empty(1, 8, 128, device="cuda")
    none = torch.full((1, 2, 8), -1, dtype=torch.int32, device="cuda")
    # (the same kernels on both sides)
    sik.sik_decode_step_ex(st.layout, q=dev(q, cfg.dtype), K=st.dK, V=st.dV, seq_len=st.dsl, mu=st.dmu,
                           codebook=st.dcb, codes=st.dcodes, k=128, out=a, workspace=st.ws, launches=2)
    sik.sik_decode_step_ex(st.layout, q=dev(q, cfg.dtype), K=st.dK, V=st.dV, seq_len=st.dsl, mu=st.dmu,
                           codebook=st.dcb, codes=st.dcodes, k=128, out=b_, forced_idx=none, workspace=st.ws, launches=2)
    sync()
    assert torch.equal(a, b_)
    # the one-launch step selects the same tokens and differs only in the order of its fp32 sums
    sik.sik_decode_step(st.layout, dev(q, cfg.dtype), None, None, st.dK, st.dV, st.dsl, st.dmu, st.dcb, st.dcodes, 128,
                        0.0, b_, None, st.ws)
    sync()
    assert float((a - b_).abs().max()) <= 2e-5 * float(a.abs().max())   # each within 1e-5 of the exact result


def run_q2(oracle, cfg, capacity, steps, append, n_forced, side_rows, seq_len=None, seed=5, launches=0):
    st = Q2State(cfg, oracle, capacity=capacity, seq_len=seq_len, offset_std=0.8, out_dtype=torch.float32)
    B, Hkv, Hq, k = cfg.batch, cfg.n_kv_heads, cfg.n_q_heads, cfg.top_k
    R = Hq // Hkv
    kvq = torch.from_numpy(st.records()).cuda()
    dal = torch.from_numpy(st.alpha).cuda()
    sl, codes, qkv = st.sl.copy(), st.codes, st.qkv
    out = torch.empty(B, Hq, 128, device="cuda")
    idx = torch.empty(B, Hq, k, dtype=torch.int32, device="cuda")
    for step in range(steps):
        q, kn, vn = W.make_step_inputs(cfg, step)
        forced = draw_forced(cfg, sl, n_forced, seed + step)      # sinks are prefill tokens
        fK = np.zeros((B, Hkv, n_forced, 128), np.uint16)
        fV = np.zeros((B, Hkv, n_forced, 128), np.uint16)
        for b in range(B):
            for h in range(Hkv):
                for j, t in enumerate(forced[b, h]):
                    if 0 <= t < sl[b]:
                        fK[b, h, j], fV[b, h, j] = st.K[b, h, t], st.V[b, h, t]
        sik.sik_decode_step_ex(st.layout, q=dev(q, cfg.dtype), k_new=dev(kn, cfg.dtype) if append else None,
                               v_new=dev(vn, cfg.dtype) if append else None, kvq=kvq, alpha=dal, seq_len=st.dsl,
                               mu=st.dmu, codebook=st.dcb, codes=st.dcodes, k=k, out=out, idx_out=idx,
                               forced_idx=torch.from_numpy(forced).cuda(),
                               forced_K=dev(fK, cfg.dtype) if side_rows else None,
                               forced_V=dev(fV, cfg.dtype) if side_rows else None, workspace=st.ws,
                               launches=launches)
        sync()
        assert sik.sik_workspace_status(st.ws) == 0
        ref_out, ref_idx = oracle.decode_step_q2_forced(q, kn if append else None, vn if append else None, cfg.dtype,
                                                        sl, st.mu, st.alpha, st.cb, codes, qkv, k, forced,
                                                        fK if side_rows else None, fV if side_rows else None)
        assert np.array_equal(st.dsl.cpu().numpy(), sl)
        if append:
            adopt_appended_records(oracle, kvq, kn, vn, cfg.dtype, st.mu, st.alpha, codes, qkv, sl)
        g_idx = idx.cpu().numpy()
        check_sets(g_idx, ref_idx, oracle.score(q, cfg.dtype, st.cb, codes, sl), forced, sl, k, R)
        if side_rows:
            valid = oracle.forced_valid(forced, sl)
            dyn = g_idx.copy()
            for b in range(B):
                for hq in range(Hq):
                    f = {int(t) for t in forced[b, hq // R][valid[b, hq // R]]}
                    dyn[b, hq] = [-1 if int(t) in f else t for t in g_idx[b, hq]]
            ref = oracle.sparse_attn_q2_forced(q, cfg.dtype, codes, qkv, st.alpha, st.mu, fK, fV,
                                               valid.astype(np.uint8), dyn)
        else:
            ref = oracle.sparse_attn_q2(q, cfg.dtype, codes, qkv, st.alpha, g_idx)
        check_attention(out.cpu().numpy().astype(np.float64), ref, True)


@BOTH_PATHS
@pytest.mark.parametrize("side_rows", [False, True])
def test_forced_q2_c2_shape_with_append(oracle, side_rows, launches):
    run_q2(oracle, cfg_small("C2", context=9000, top_k=160), 9004, steps=3, append=True, n_forced=64,
           side_rows=side_rows, launches=launches)


@BOTH_PATHS
@pytest.mark.parametrize("side_rows", [False, True])
def test_forced_q2_ragged_batch_fp16(oracle, side_rows, launches):
    cfg = cfg_small("C4", batch=4, n_kv_heads=2, n_q_heads=8, context=2048, top_k=200, dtype="fp16")
    run_q2(oracle, cfg, 2052, steps=2, append=True, n_forced=100, side_rows=side_rows, seq_len=[2048, 3, 511, 0], launches=launches)


def test_forced_argument_errors(oracle):
    cfg = cfg_small("C2", n_kv_heads=2, n_q_heads=8, context=1000, top_k=64)
    st = GpuState(cfg, oracle, out_dtype=torch.float32)
    q, _, _ = W.make_step_inputs(cfg, 0)
    out = torch.empty(1, 8, 128, device="cuda")
    base = dict(q=dev(q, cfg.dtype), K=st.dK, V=st.dV, seq_len=st.dsl, mu=st.dmu, codebook=st.dcb, codes=st.dcodes,
                out=out, workspace=st.ws)
    f64_ = torch.full((1, 2, 64), -1, dtype=torch.int32, device="cuda")
    f200 = torch.full((1, 2, 200), -1, dtype=torch.int32, device="cuda")
    rows = torch.zeros(1, 2, 64, 128, dtype=torch.bfloat16, device="cuda")
    for kw, status in ((dict(k=64, forced_idx=f64_), -4),             # the budget must exceed the forced set
                       (dict(k=64, forced_idx=f200), -2),             # more than 128 forced slots
                       (dict(k=100, forced_idx=f64_, forced_K=rows, forced_V=rows), -8),   # side rows need the 2-bit cache
                       (dict(k=100, forced_idx=f64_, forced_K=rows), -1)):
        with pytest.raises(sik.SikError) as e:
            sik.sik_decode_step_ex(st.layout, **base, **kw)
        assert e.value.status == status, (kw.keys(), e.value.status)


# --------------------------------------------------------------------------- budgets that follow the context
@pytest.mark.parametrize("launches", [0, 1], ids=["auto", "one_launch"])
@pytest.mark.parametrize("per_mille,n_forced", [(75, 0), (75, 16), (4, 16), (1000, 0)])
def test_budget_per_mille_ragged_batch(oracle, per_mille, n_forced, launches):
    # 7.5 % of each sequence's own length; 0.4 %: the forced tokens fill (or exceed) the budget; 100 %: capped by k
    cfg = cfg_small("C2", batch=4, n_kv_heads=2, n_q_heads=8, context=6000, top_k=500)
    st = GpuState(cfg, oracle, capacity=6000, seq_len=[6000, 2500, 40, 0], offset_std=0.5, out_dtype=torch.float32)
    q, _, _ = W.make_step_inputs(cfg, 0)
    forced = draw_forced(cfg, st.sl, max(n_forced, 1), 3, spoil=False)
    if n_forced == 0:
        forced[:] = -1
    out = torch.empty(4, 8, 128, device="cuda")
    idx = torch.empty(4, 8, 500, dtype=torch.int32, device="cuda")
    sik.sik_decode_step_ex(st.layout, q=dev(q, cfg.dtype), K=st.dK, V=st.dV, seq_len=st.dsl, mu=st.dmu,
                           codebook=st.dcb, codes=st.dcodes, k=500, k_per_mille=per_mille, out=out, idx_out=idx,
                           forced_idx=torch.from_numpy(forced).cuda() if n_forced else None, workspace=st.ws,
                           launches=launches)
    sync()
    sl = st.sl.copy()
    ref_out, ref_idx = oracle.decode_step_forced(q, None, None, st.K, st.V, cfg.dtype, sl, st.mu, st.cb, st.codes, 500,
                                                 forced, k_per_mille=per_mille)
    g_idx = idx.cpu().numpy()
    for b in range(4):
        want = max(oracle.budget(500, sl[b], per_mille), int(((forced[b, 0] >= 0) & (forced[b, 0] < sl[b])).sum()))
        assert int((g_idx[b, 0] >= 0).sum()) == min(want, int(sl[b]))
    check_sets(g_idx, ref_idx, oracle.score(q, cfg.dtype, st.cb, st.codes, sl), forced, sl, 500, 4)
    check_attention(out.cpu().numpy().astype(np.float64), oracle.sparse_attn(q, st.K, st.V, cfg.dtype, g_idx), True)


def test_sign_only_retrieval_is_a_codebook_of_signs(oracle):
    # the ablation's "sign-only retrieval" (similarity from the sign bits alone) needs no kernel of its own: with
    # the centroid of Code j set to its sign pattern, the table lookup sums q_d * sign_d
    cfg = cfg_small("C2", batch=1, n_kv_heads=2, n_q_heads=8, context=3000, top_k=64)
    st = GpuState(cfg, oracle, out_dtype=torch.float32)
    j = np.arange(16)
    pattern = np.stack([2.0 * ((j >> (3 - e)) & 1) - 1.0 for e in range(4)], axis=-1).astype(np.float32)   # [16, 4]
    cb = np.broadcast_to(pattern, (1, 2, 32, 16, 4)).copy()
    q, _, _ = W.make_step_inputs(cfg, 0)
    scores = torch.empty(1, 8, 3000, device="cuda")
    sik.sik_score(st.layout, dev(q, cfg.dtype), torch.from_numpy(cb).cuda(), st.dcodes, st.dsl, scores)
    sync()
    signs = 2.0 * np.unpackbits(st.codes, axis=-1, bitorder="big").astype(np.float64) - 1.0     # [1, 2, 3000, 128]
    qf = W.from_bits(q, cfg.dtype).astype(np.float64)
    want = np.einsum("hd,hld->hl", qf[0], np.repeat(signs[0], 4, axis=0))
    assert np.abs(scores.cpu().numpy()[0] - want).max() <= 1e-5 * np.abs(want).max()


# --------------------------------------------------------------------------- group-shared selection
def run_shared(oracle, cfg, capacity, steps, append, q2=False, seq_len=None):
    B, Hkv, Hq, k = cfg.batch, cfg.n_kv_heads, cfg.n_q_heads, cfg.top_k
    R = Hq // Hkv
    if q2:
        st = Q2State(cfg, oracle, capacity=capacity, seq_len=seq_len, offset_std=0.7, out_dtype=torch.float32)
        kvq, dal = torch.from_numpy(st.records()).cuda(), torch.from_numpy(st.alpha).cuda()
    else:
        st = GpuState(cfg, oracle, capacity=capacity, seq_len=seq_len, offset_std=0.7, out_dtype=torch.float32)
    sl = st.sl.copy()
    out = torch.empty(B, Hq, 128, device="cuda")
    idx = torch.empty(B, Hkv, k, dtype=torch.int32, device="cuda")
    for step in range(steps):
        q, kn, vn = W.make_step_inputs(cfg, step)
        kw = dict(q=dev(q, cfg.dtype), k_new=dev(kn, cfg.dtype) if append else None,
                  v_new=dev(vn, cfg.dtype) if append else None, seq_len=st.dsl, mu=st.dmu, codebook=st.dcb,
                  codes=st.dcodes, k=k, out=out, idx_out=idx, workspace=st.ws, group_shared=True)
        kw.update(dict(kvq=kvq, alpha=dal) if q2 else dict(K=st.dK, V=st.dV))
        sik.sik_decode_step_ex(st.layout, **kw)
        sync()
        _, ref_idx = oracle.decode_step_shared(q, kn if append else None, vn if append else None, st.K, st.V,
                                               cfg.dtype, sl, st.mu, st.cb, st.codes, k)
        assert np.array_equal(st.dsl.cpu().numpy(), sl)
        s_kv = oracle.shared_scores(q, cfg.dtype, st.cb, st.codes, sl)
        g_idx = idx.cpu().numpy()
        for b in range(B):
            for h in range(Hkv):
                topk_sets_agree(g_idx[b, h], ref_idx[b, h], s_kv[b, h], int(sl[b]), k)
        full = np.repeat(g_idx, R, axis=1)
        if q2:
            ref = oracle.sparse_attn_q2(q, cfg.dtype, st.codes, st.qkv, st.alpha, full)
        else:
            ref = oracle.sparse_attn(q, st.K, st.V, cfg.dtype, full)
        check_attention(out.cpu().numpy().astype(np.float64), ref, True)


def test_shared_selection_c2_shape_with_append(oracle):
    run_shared(oracle, cfg_small("C2", context=9000, top_k=300), 9004, steps=3, append=True)


def test_shared_selection_gqa8_ragged_batch(oracle):
    cfg = cfg_small("C5", batch=3, n_kv_heads=2, n_q_heads=16, context=5000, top_k=700)
    run_shared(oracle, cfg, 5004, steps=2, append=True, seq_len=[5000, 300, 0])


def test_shared_selection_gqa3_fp16_k_above_context(oracle):
    cfg = cfg_small("C2", batch=2, n_kv_heads=2, n_q_heads=6, context=800, top_k=900, dtype="fp16")
    run_shared(oracle, cfg, 904, steps=1, append=False, seq_len=[800, 5])


def test_shared_selection_on_records(oracle):
    run_shared(oracle, cfg_small("C2", context=7000, top_k=256), 7000, steps=2, append=False, q2=True)


@pytest.mark.parametrize("q2", [False, True])
def test_shared_selection_with_forced_set_budget_and_append(oracle, q2):
    # everything at once: one index set per KV head, 20 forced tokens, a budget of 5 % of each sequence, append
    cfg = cfg_small("C2", batch=3, n_kv_heads=2, n_q_heads=8, context=4000, top_k=400)
    B, Hkv, Hq, k, R = 3, 2, 8, 400, 4
    cls = Q2State if q2 else GpuState
    st = cls(cfg, oracle, capacity=4004, seq_len=[4000, 900, 33], offset_std=0.6, out_dtype=torch.float32)
    if q2:
        kvq, dal = torch.from_numpy(st.records()).cuda(), torch.from_numpy(st.alpha).cuda()
    sl = st.sl.copy()
    out = torch.empty(B, Hq, 128, device="cuda")
    idx = torch.empty(B, Hkv, k, dtype=torch.int32, device="cuda")
    for step in range(2):
        q, kn, vn = W.make_step_inputs(cfg, step)
        forced = draw_forced(cfg, sl, 20, 9 + step)
        kw = dict(q=dev(q, cfg.dtype), k_new=dev(kn, cfg.dtype), v_new=dev(vn, cfg.dtype), seq_len=st.dsl, mu=st.dmu,
                  codebook=st.dcb, codes=st.dcodes, k=k, k_per_mille=50, out=out, idx_out=idx, workspace=st.ws,
                  group_shared=True, forced_idx=torch.from_numpy(forced).cuda())
        kw.update(dict(kvq=kvq, alpha=dal) if q2 else dict(K=st.dK, V=st.dV))
        sik.sik_decode_step_ex(st.layout, **kw)
        sync()
        if q2:
            oracle.decode_step_q2(q, kn, vn, cfg.dtype, sl, st.mu, st.alpha, st.cb, st.codes, st.qkv, 1)
            adopt_appended_records(oracle, kvq, kn, vn, cfg.dtype, st.mu, st.alpha, st.codes, st.qkv, sl)
        else:
            oracle.decode_step(q, kn, vn, st.K, st.V, cfg.dtype, sl, st.mu, st.cb, st.codes, 1)
        assert np.array_equal(st.dsl.cpu().numpy(), sl)
        s_kv = oracle.shared_scores(q, cfg.dtype, st.cb, st.codes, sl)
        ref_idx = oracle.topk_with_forced(s_kv, sl, k, forced, 1, 50)        # KV heads as rows
        g_idx = idx.cpu().numpy()
        check_sets(g_idx, ref_idx, s_kv, forced, sl, k, 1)
        for b in range(B):
            want = max(oracle.budget(k, sl[b], 50), int(((forced[b, 0] >= 0) & (forced[b, 0] < sl[b])).sum()))
            assert int((g_idx[b, 0] >= 0).sum()) == min(want, int(sl[b]))
        full = np.repeat(g_idx, R, axis=1)
        if q2:
            ref = oracle.sparse_attn_q2(q, cfg.dtype, st.codes, st.qkv, st.alpha, full)
        else:
            ref = oracle.sparse_attn(q, st.K, st.V, cfg.dtype, full)
        check_attention(out.cpu().numpy().astype(np.float64), ref, True)


def test_shared_selection_beyond_the_fused_plan(oracle):
    # contexts above 512K tokens take separate score / select / attention launches, also with one list per KV head
    cfg = cfg_small("C2", batch=1, n_kv_heads=1, n_q_heads=4, context=3000, top_k=64)
    st = GpuState(cfg, oracle, capacity=600000, out_dtype=torch.float32)
    q, _, _ = W.make_step_inputs(cfg, 0)
    out = torch.empty(1, 4, 128, device="cuda")
    idx = torch.empty(1, 1, 64, dtype=torch.int32, device="cuda")
    sik.sik_decode_step_ex(st.layout, q=dev(q, cfg.dtype), K=st.dK, V=st.dV, seq_len=st.dsl, mu=st.dmu,
                           codebook=st.dcb, codes=st.dcodes, k=64, out=out, idx_out=idx, workspace=st.ws,
                           group_shared=True)
    sync()
    sl = st.sl.copy()
    _, ref_idx = oracle.decode_step_shared(q, None, None, st.K, st.V, cfg.dtype, sl, st.mu, st.cb, st.codes, 64)
    s_kv = oracle.shared_scores(q, cfg.dtype, st.cb, st.codes, sl)
    g_idx = idx.cpu().numpy()
    topk_sets_agree(g_idx[0, 0], ref_idx[0, 0], s_kv[0, 0], 3000, 64)
    ref = oracle.sparse_attn(q, st.K, st.V, cfg.dtype, np.repeat(g_idx, 4, axis=1))
    check_attention(out.cpu().numpy().astype(np.float64), ref, True)


@pytest.mark.parametrize("R,q2", [(5, False), (4, True), (6, True)])
def test_shared_selection_large_launch_gathers_once(oracle, R, q2):
    # above 2 M keys the plain shared step selects once per KV head and the attention kernel feeds each gathered
    # row to the query heads of the group (blocks of 4: R = 5 leaves a block with a single head)
    cfg = cfg_small("C2", batch=8, n_kv_heads=8, n_q_heads=8 * R, context=33000, top_k=300)
    run_shared(oracle, cfg, 33000, steps=1, append=False, q2=q2, seq_len=[33000, 20000, 5, 33000, 1000, 0, 33000, 777])


def test_many_units_long_context_forced_set_and_equal_scores(oracle):
    """512 (sequence, KV head) units of 66000 tokens: a launch large enough for one scoring workgroup per unit,
    whose token range must still be cut into chunks of at most 64512 tokens (16-bit histogram counts, one forced
    bitmap bit per token of a chunk).  Forced tokens sit on both sides of token 65536; the first step has an
    all-zero query (every score equal: one histogram bin holds the whole context and the smaller index wins),
    the second a random one.  Every unit holds the same seeded cache, so the oracle computes one unit per distinct
    sequence length and every (b, query head) is compared with it."""
    B, Hkv, Hq, L, k, nf = 64, 8, 16, 66000, 256, 64
    R = Hq // Hkv
    cfg1 = cfg_small("C2", batch=1, n_kv_heads=1, n_q_heads=R, context=L, top_k=k, seed=91)
    dt = cfg1.dtype
    assert sik.sik_plan_info(sik.make_layout(B, Hkv, Hq, 128, L, TDT[dt], torch.float32))[:2] == [2, 64512]
    K1, V1 = W.make_cache(cfg1)
    mu1, codes1, cb1, _ = oracle.fit(K1, dt, np.array([L], np.int32))
    lens = np.full(B, L, np.int32)
    lens[3], lens[5], lens[9], lens[63] = 40000, 65536, 64513, 100
    rng = np.random.default_rng(7)
    forced1 = np.concatenate([rng.choice(64000, nf - 8, replace=False), 65500 + 7 * np.arange(8)]).astype(np.int32)
    lay = sik.make_layout(B, Hkv, Hq, 128, L, TDT[dt], torch.float32)
    ws = sik.alloc_workspace(lay, k)
    tile = lambda t, *shape: t.expand(*shape).contiguous()  # noqa: E731
    dK, dV = tile(dev(K1, dt), B, Hkv, L, 128), tile(dev(V1, dt), B, Hkv, L, 128)
    dcodes = tile(torch.from_numpy(codes1).cuda(), B, Hkv, L, 16)
    dmu, dcb = tile(torch.from_numpy(mu1).cuda(), B, Hkv, 128), tile(torch.from_numpy(cb1).cuda(), B, Hkv, 32, 16, 4)
    dsl = torch.from_numpy(lens).cuda()
    dforced = tile(torch.from_numpy(forced1).cuda().view(1, 1, nf), B, Hkv, nf)
    out = torch.empty(B, Hq, 128, device="cuda")
    idx = torch.empty(B, Hq, k, dtype=torch.int32, device="cuda")
    q_rand, _, _ = W.make_step_inputs(cfg1, 0)
    for step, q1 in enumerate((np.zeros_like(q_rand), q_rand)):
        dq = tile(dev(q1, dt).view(1, 1, R, 128), B, Hkv, R, 128).view(B, Hq, 128)
        sik.sik_decode_step_ex(lay, q=dq, K=dK, V=dV, seq_len=dsl, mu=dmu, codebook=dcb, codes=dcodes, k=k, out=out,
                               idx_out=idx, workspace=ws, forced_idx=dforced)
        sync()
        g_idx, g_out = idx.cpu().numpy(), out.cpu().numpy().astype(np.float64)
        ref = {}
        for Lb in sorted(set(lens.tolist())):
            sl1 = np.array([Lb], np.int32)
            _, r_idx = oracle.decode_step_forced(q1, None, None, K1, V1, dt, sl1, mu1, cb1, codes1, k,
                                                 forced1.reshape(1, 1, nf))
            ref[Lb] = (r_idx, oracle.score(q1, dt, cb1, codes1, sl1), sl1)
        for b in range(B):
            r_idx, s_ref, sl1 = ref[int(lens[b])]
            for h in range(Hkv):
                gi = g_idx[b:b + 1, h * R:(h + 1) * R]
                if step == 0:   # all scores equal: the library's own rule (smaller index first) decides, exactly
                    assert np.array_equal(np.sort(gi, -1), np.sort(r_idx, -1)), (b, h)
                else:
                    check_sets(gi, r_idx, s_ref, forced1.reshape(1, 1, nf), sl1, k, R)
        # attention over the library's own sets: all 1024 query heads as heads of the one oracle unit
        q_all = np.tile(q1, (1, B * Hkv, 1))
        att = oracle.sparse_attn(q_all, K1, V1, dt, g_idx.reshape(1, B * Hq, k))
        check_attention(g_out.reshape(1, B * Hq, 128), att, True)

"""Seeded random shapes through the general decode step against the CPU oracle: batch, GQA ratio, ragged lengths,
budget, cache format, append, forced sets, context-proportional budgets and the launch structure drawn together, a
few steps each.
Same bars as the hand-picked cases (tests/test_gpu_parity.py, tests/test_gpu_kvq.py, tests/test_gpu_forced.py)."""
import numpy as np
import pytest
import torch

import sik_workloads as W
from helpers import dev
from test_gpu_forced import check_sets
from test_gpu_kvq import Q2State, adopt_appended_records
from test_gpu_parity import GpuState, check_attention, cfg_small, sync

pytestmark = pytest.mark.gpu

import paper_2603_14224_amd as sik  # noqa: E402


def draw_case(seed):
    r = np.random.default_rng(1000 + seed)
    hkv = int(r.choice([1, 2, 3, 4]))
    R = int(r.choice([1, 2, 3, 4, 5, 8, 12]))
    B = int(r.choice([1, 1, 2, 3, 5]))
    L = int(r.choice([1, 70, 1000, 1024, 4097, 9000, 20011]))
    k = int(r.choice([1, 17, 256, 1000, 3000]))
    append = bool(r.integers(0, 2))
    cap = L + 4
    k = min(k, cap)
    nf = int(r.choice([0, 0, 3, 64]))
    if nf >= k:
        nf = 0
    return dict(seed=seed, hkv=hkv, R=R, B=B, L=L, k=k, append=append, cap=cap, nf=nf,
                q2=bool(r.integers(0, 2)), side=bool(r.integers(0, 2)), pm=int(r.choice([0, 0, 75, 500])),
                dtype=str(r.choice(["bf16", "fp16"])), lens=[int(x) for x in r.integers(0, L + 1, B)],
                # 0: the library's choice; 1: one launch whenever the plan allows; 3: with the 16-bit first pass
                launches=int(np.random.default_rng(5000 + seed).choice([0, 1, 1, 3])))


@pytest.mark.parametrize("seed", range(48))
def test_random_decode_cases(oracle, seed):
    c = draw_case(seed)
    print(c)
    cfg = cfg_small("C2", batch=c["B"], n_kv_heads=c["hkv"], n_q_heads=c["hkv"] * c["R"], context=c["L"],
                    top_k=c["k"], dtype=c["dtype"], seed=200 + seed)
    lens = c["lens"]
    lens[0] = c["L"]
    B, Hkv, Hq, k, R, nf = c["B"], c["hkv"], c["hkv"] * c["R"], c["k"], c["R"], c["nf"]
    q2, side = c["q2"], c["q2"] and c["side"] and nf > 0
    if q2:
        st = Q2State(cfg, oracle, capacity=c["cap"], seq_len=lens, offset_std=0.6, out_dtype=torch.float32)
        kvq, dal = torch.from_numpy(st.records()).cuda(), torch.from_numpy(st.alpha).cuda()
    else:
        st = GpuState(cfg, oracle, capacity=c["cap"], seq_len=lens, offset_std=0.6, out_dtype=torch.float32)
    sl = st.sl.copy()
    out = torch.empty(B, Hq, 128, device="cuda")
    idx = torch.empty(B, Hq, k, dtype=torch.int32, device="cuda")
    rng = np.random.default_rng(seed)
    for step in range(2):
        q, kn, vn = W.make_step_inputs(cfg, step)
        ap = c["append"]
        forced = np.full((B, Hkv, max(nf, 1)), -1, np.int32)
        fK = np.zeros((B, Hkv, max(nf, 1), 128), np.uint16)
        fV = np.zeros_like(fK)
        for b in range(B):
            for h in range(Hkv):
                m = min(nf, int(sl[b]))
                if m:
                    forced[b, h, :m] = rng.choice(int(sl[b]), m, replace=False)
                    fK[b, h, :m], fV[b, h, :m] = st.K[b, h, forced[b, h, :m]], st.V[b, h, forced[b, h, :m]]
        kw = dict(q=dev(q, cfg.dtype), k_new=dev(kn, cfg.dtype) if ap else None, v_new=dev(vn, cfg.dtype) if ap else None,
                  seq_len=st.dsl, mu=st.dmu, codebook=st.dcb, codes=st.dcodes, k=k, k_per_mille=c["pm"], out=out,
                  idx_out=idx, workspace=st.ws, forced_idx=torch.from_numpy(forced).cuda() if nf else None,
                  launches=c["launches"])
        if q2:
            kw.update(kvq=kvq, alpha=dal)
            if side:
                kw.update(forced_K=dev(fK, cfg.dtype), forced_V=dev(fV, cfg.dtype))
        else:
            kw.update(K=st.dK, V=st.dV)
        sik.sik_decode_step_ex(st.layout, **kw)
        sync()
        assert sik.sik_workspace_status(st.ws) == 0
        if q2:
            # the oracle's budget rule lives in decode_step_forced / topk_with_forced; reuse it for both formats
            if ap:
                oracle.decode_step_q2(q, kn, vn, cfg.dtype, sl, st.mu, st.alpha, st.cb, st.codes, st.qkv, 1)
                adopt_appended_records(oracle, kvq, kn, vn, cfg.dtype, st.mu, st.alpha, st.codes, st.qkv, sl)
            s_ref = oracle.score(q, cfg.dtype, st.cb, st.codes, sl)
            ref_idx = oracle.topk_with_forced(s_ref, sl, k, forced, R, c["pm"])
        else:
            _, ref_idx = oracle.decode_step_forced(q, kn if ap else None, vn if ap else None, st.K, st.V, cfg.dtype, sl,
                                                   st.mu, st.cb, st.codes, k, forced, k_per_mille=c["pm"])
            s_ref = oracle.score(q, cfg.dtype, st.cb, st.codes, sl)
        assert np.array_equal(st.dsl.cpu().numpy(), sl), "sequence lengths"
        g_idx = idx.cpu().numpy()
        check_sets(g_idx, ref_idx, s_ref, forced, sl, k, R)
        if q2 and side:
            valid = oracle.forced_valid(forced, sl)
            dyn = g_idx.copy()
            for b in range(B):
                for hq in range(Hq):
                    f = {int(t) for t in forced[b, hq // R][valid[b, hq // R]]}
                    dyn[b, hq] = [-1 if int(t) in f else t for t in g_idx[b, hq]]
            ref = oracle.sparse_attn_q2_forced(q, cfg.dtype, st.codes, st.qkv, st.alpha, st.mu, fK, fV,
                                               valid.astype(np.uint8), dyn)
        elif q2:
            ref = oracle.sparse_attn_q2(q, cfg.dtype, st.codes, st.qkv, st.alpha, g_idx)
        else:
            ref = oracle.sparse_attn(q, st.K, st.V, cfg.dtype, g_idx)
        check_attention(out.cpu().numpy().astype(np.float64), ref, True)

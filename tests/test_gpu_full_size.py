"""Full-size parity: the five benchmark configurations at their real shapes, in the launch configuration
bench.py times (sik_quantize_keys FIT, then sik_decode_step with bf16/fp16 outputs replaced by fp32 so that the
1e-5 bar applies), checked on sampled (sequence, KV head) units that the CPU oracle recomputes from scratch:
channel means bit-equal, codes byte-equal, top-k sets tie-legal, attention within 1e-5 relative.
"""
import numpy as np
import pytest
import torch

import sik_workloads as W
from helpers import dev, topk_sets_agree

pytestmark = pytest.mark.gpu

import paper_2603_14224_amd as sik  # noqa: E402

TDT = {"fp16": torch.float16, "bf16": torch.bfloat16}


def run_full(oracle, name, steps, units, extra_cap=32):
    cfg = W.CONFIGS[name]
    B, Hkv, Hq, D, L, k = cfg.batch, cfg.n_kv_heads, cfg.n_q_heads, cfg.head_dim, cfg.context, cfg.top_k
    R = Hq // Hkv
    cap = L + (extra_cap if cfg.append else 0)
    K, V = W.make_cache(cfg, capacity=cap)
    lay = sik.make_layout(B, Hkv, Hq, D, cap, TDT[cfg.dtype], torch.float32)
    ws = sik.alloc_workspace(lay, k)
    dK, dV = dev(K, cfg.dtype), dev(V, cfg.dtype)
    dsl = torch.full((B,), L, dtype=torch.int32, device="cuda")
    dmu = torch.empty(B, Hkv, D, device="cuda")
    dcb = torch.empty(B, Hkv, D // 4, 16, 4, device="cuda")
    dcnt = torch.empty(B, Hkv, D // 4, 16, dtype=torch.int32, device="cuda")
    dcodes = torch.zeros(B, Hkv, cap, D // 8, dtype=torch.uint8, device="cuda")
    sik.sik_quantize_keys(lay, dK, dsl, 0, 0, sik.SIK_Q_FIT, dmu, dcb, dcnt, dcodes, ws)
    torch.cuda.synchronize()

    # oracle state of the sampled units, built from the same host bits
    ref = {}
    for (b, h) in units:
        Ku, Vu = K[b:b + 1, h:h + 1].copy(), V[b:b + 1, h:h + 1].copy()
        sl = np.array([L], np.int32)
        mu, codes, cb, cnt = oracle.fit(Ku, cfg.dtype, sl)
        assert np.array_equal(dmu[b, h].cpu().numpy(), mu[0, 0]), "channel means differ"
        assert np.array_equal(dcodes[b, h, :L].cpu().numpy(), codes[0, 0, :L]), "codes differ"
        assert np.array_equal(dcnt[b, h].cpu().numpy(), cnt[0, 0])
        Kp = np.abs(W.from_bits(Ku[0, 0, :L], cfg.dtype).astype(np.float64) - mu[0, 0]).max(axis=0)
        assert np.all(np.abs(dcb[b, h].cpu().numpy() - cb[0, 0]) <= 1e-5 * Kp.reshape(32, 1, 4))
        # the decode steps run on the GPU's own codebook so that both sides score with identical tables
        ref[(b, h)] = dict(K=Ku, V=Vu, sl=sl, mu=mu, codes=codes, cb=dcb[b:b + 1, h:h + 1].cpu().numpy())

    out = torch.empty(B, Hq, D, device="cuda")
    idx = torch.empty(B, Hq, k, dtype=torch.int32, device="cuda")
    n_diff = 0
    for step in range(steps):
        q, kn, vn = W.make_step_inputs(cfg, step)
        ap = cfg.append
        sik.sik_decode_step(lay, dev(q, cfg.dtype), dev(kn, cfg.dtype) if ap else None,
                            dev(vn, cfg.dtype) if ap else None, dK, dV, dsl, dmu, dcb, dcodes, k, 0.0, out, idx, ws)
        torch.cuda.synchronize()
        g_idx, g_out = idx.cpu().numpy(), out.cpu().numpy().astype(np.float64)
        for (b, h), u in ref.items():
            qs = q[b:b + 1, h * R:(h + 1) * R]
            if ap:
                r_out, r_idx = oracle.decode_step(qs, kn[b:b + 1, h:h + 1], vn[b:b + 1, h:h + 1], u["K"], u["V"],
                                                  cfg.dtype, u["sl"], u["mu"], u["cb"], u["codes"], k)
                t = int(u["sl"][0]) - 1
                assert np.array_equal(dcodes[b, h, t].cpu().numpy(), u["codes"][0, 0, t])
            else:
                r_out, r_idx = oracle.decode_step(qs, None, None, u["K"], u["V"], cfg.dtype, u["sl"], u["mu"],
                                                  u["cb"], u["codes"], k)
            s_ref = oracle.score(qs, cfg.dtype, u["cb"], u["codes"], u["sl"])
            gi = g_idx[b, h * R:(h + 1) * R]
            for r in range(R):
                n_diff += topk_sets_agree(gi[r], r_idx[0, r], s_ref[0, r], int(u["sl"][0]), k)
            r_att = oracle.sparse_attn(qs, u["K"], u["V"], cfg.dtype, gi[None])
            for r in range(R):
                d = np.abs(g_out[b, h * R + r] - r_att[0, r]).max()
                assert d <= 1e-5 * np.abs(r_att[0, r]).max(), (name, step, b, h, r, d)
        assert int(dsl[0]) == L + (step + 1 if ap else 0)
    print(f"{name}: {steps} step(s), {len(units)} unit(s), tie-legal index differences: {n_diff}")


def test_full_c2(oracle):
    run_full(oracle, "C2", steps=2, units=[(0, 0), (0, 5)])


def test_full_c3_with_append(oracle):
    run_full(oracle, "C3", steps=2, units=[(0, 3)])


def test_full_c4_large_batch(oracle):
    run_full(oracle, "C4", steps=1, units=[(0, 0), (17, 4), (31, 7)])


def test_full_c5_prefill_compress_then_16_steps(oracle):
    run_full(oracle, "C5", steps=16, units=[(2, 6)])


def run_full_q2(oracle, name, steps, units, extra_cap=32):
    """As run_full, on the 2-bit cache: the library quantises the whole workload (keys, then records), the
    oracle redoes the sampled units from the same host bits; alpha bit-equal, records byte-equal, top-k sets
    tie-legal, attention over the records within 1e-5 relative."""
    cfg = W.CONFIGS[name]
    B, Hkv, Hq, D, L, k = cfg.batch, cfg.n_kv_heads, cfg.n_q_heads, cfg.head_dim, cfg.context, cfg.top_k
    R = Hq // Hkv
    cap = L + (extra_cap if cfg.append else 0)
    K, V = W.make_cache(cfg, capacity=cap)
    lay = sik.make_layout(B, Hkv, Hq, D, cap, TDT[cfg.dtype], torch.float32)
    ws = sik.alloc_workspace(lay, k)
    dK, dV = dev(K, cfg.dtype), dev(V, cfg.dtype)
    dsl = torch.full((B,), L, dtype=torch.int32, device="cuda")
    dmu = torch.empty(B, Hkv, D, device="cuda")
    dal = torch.empty(B, Hkv, D, device="cuda")
    dcb = torch.empty(B, Hkv, D // 4, 16, 4, device="cuda")
    dcnt = torch.empty(B, Hkv, D // 4, 16, dtype=torch.int32, device="cuda")
    dcodes = torch.zeros(B, Hkv, cap, D // 8, dtype=torch.uint8, device="cuda")
    kvq = sik.alloc_kvq(lay)
    sik.sik_quantize_keys(lay, dK, dsl, 0, 0, sik.SIK_Q_FIT, dmu, dcb, dcnt, dcodes, ws)
    sik.sik_quantize_kv(lay, dK, dV, dsl, 0, 0, sik.SIK_Q_FIT, dmu, dal, kvq)
    torch.cuda.synchronize()
    del dK, dV

    ref = {}
    for (b, h) in units:
        Ku, Vu = K[b:b + 1, h:h + 1].copy(), V[b:b + 1, h:h + 1].copy()
        sl = np.array([L], np.int32)
        mu, codes, cb, cnt = oracle.fit(Ku, cfg.dtype, sl)
        al, qkv = oracle.fit_q2(Ku, Vu, cfg.dtype, sl, mu)
        assert np.array_equal(dmu[b, h].cpu().numpy(), mu[0, 0])
        assert np.array_equal(dal[b, h].cpu().numpy(), al[0, 0]), "alpha differs"
        assert np.array_equal(kvq[b, h, :L].cpu().numpy(), oracle.pack_records(codes, qkv)[0, 0, :L]), "records differ"
        ref[(b, h)] = dict(sl=sl, mu=mu, al=al, codes=codes, qkv=qkv, cb=dcb[b:b + 1, h:h + 1].cpu().numpy())

    out = torch.empty(B, Hq, D, device="cuda")
    idx = torch.empty(B, Hq, k, dtype=torch.int32, device="cuda")
    n_diff = 0
    for step in range(steps):
        q, kn, vn = W.make_step_inputs(cfg, step)
        ap = cfg.append
        sik.sik_decode_step_q2(lay, dev(q, cfg.dtype), dev(kn, cfg.dtype) if ap else None,
                               dev(vn, cfg.dtype) if ap else None, kvq, dsl, dmu, dal, dcb, dcodes, k, 0.0, out, idx, ws)
        torch.cuda.synchronize()
        g_idx, g_out = idx.cpu().numpy(), out.cpu().numpy().astype(np.float64)
        for (b, h), u in ref.items():
            qs = q[b:b + 1, h * R:(h + 1) * R]
            _, r_idx = oracle.decode_step_q2(qs, kn[b:b + 1, h:h + 1] if ap else None,
                                             vn[b:b + 1, h:h + 1] if ap else None, cfg.dtype, u["sl"], u["mu"],
                                             u["al"], u["cb"], u["codes"], u["qkv"], k)
            if ap:
                t = int(u["sl"][0]) - 1
                assert np.array_equal(kvq[b, h, t].cpu().numpy(), oracle.pack_records(u["codes"], u["qkv"])[0, 0, t])
            s_ref = oracle.score(qs, cfg.dtype, u["cb"], u["codes"], u["sl"])
            gi = g_idx[b, h * R:(h + 1) * R]
            for r in range(R):
                n_diff += topk_sets_agree(gi[r], r_idx[0, r], s_ref[0, r], int(u["sl"][0]), k)
            r_att = oracle.sparse_attn_q2(qs, cfg.dtype, u["codes"], u["qkv"], u["al"], gi[None])
            for r in range(R):
                d = np.abs(g_out[b, h * R + r] - r_att[0, r]).max()
                assert d <= 1e-5 * np.abs(r_att[0, r]).max(), (name, step, b, h, r, d)
        assert int(dsl[0]) == L + (step + 1 if ap else 0)
    print(f"{name} (2-bit cache): {steps} step(s), {len(units)} unit(s), tie-legal index differences: {n_diff}")


def test_full_c2_two_bit_cache(oracle):
    run_full_q2(oracle, "C2", steps=2, units=[(0, 3)])


def test_full_c4_two_bit_cache(oracle):
    run_full_q2(oracle, "C4", steps=1, units=[(5, 2), (31, 7)])


def test_full_c5_two_bit_cache_with_append(oracle):
    run_full_q2(oracle, "C5", steps=3, units=[(1, 4)])

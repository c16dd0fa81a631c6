"""Full-size parity: the benchmark configurations at their real shapes, in the launch configuration bench.py
times (sik_quantize_keys FIT, then sik_decode_step), with the CPU oracle as the only source of reference values
and EVERY (sequence, head) unit checked.

  1. prefill side: the library fits the whole cache; the oracle fits it from the same host bits; channel means
     bit-equal, codes byte-equal, counts equal, codebook within 1e-5 max|K'_d|, for every (b, KV head);
  2. the ORACLE's codebook is uploaded (means and codes are bit-identical anyway), so that both sides score with
     the same tables, as in the reduced-shape tests;
  3. decode steps on the whole batch: appended rows and codes byte-equal, lengths equal, top-k sets tie-legal for
     every (b, query head), attention (fp32 output, 1e-5 relative) against the oracle's attention over the
     library's own tie-legal sets; one more step with the 16-bit output bench.py times, under the 16-bit bar,
     with the plain max|d| printed.
"""
import numpy as np
import pytest
import torch

import sik_workloads as W
from helpers import bits_of_tensor, check_attention, dev, records_agree, topk_sets_agree

pytestmark = pytest.mark.gpu

import paper_2603_14224_amd as sik  # noqa: E402

TDT = {"fp16": torch.float16, "bf16": torch.bfloat16}


def fit_both_sides(oracle, cfg, cap, K, lay, ws):
    """Library FIT and oracle FIT of the whole cache; every unit compared.  Returns the oracle's state and the
    device tensors, with the oracle's codebook uploaded."""
    B, Hkv, D, L = cfg.batch, cfg.n_kv_heads, cfg.head_dim, cfg.context
    dK = dev(K, cfg.dtype)
    dsl = torch.full((B,), L, dtype=torch.int32, device="cuda")
    dmu = torch.empty(B, Hkv, D, device="cuda")
    dcb = torch.empty(B, Hkv, D // 4, 16, 4, device="cuda")
    dcnt = torch.empty(B, Hkv, D // 4, 16, dtype=torch.int32, device="cuda")
    dcodes = torch.zeros(B, Hkv, cap, D // 8, dtype=torch.uint8, device="cuda")
    sik.sik_quantize_keys(lay, dK, dsl, 0, 0, sik.SIK_Q_FIT, dmu, dcb, dcnt, dcodes, ws)
    torch.cuda.synchronize()
    sl = np.full(B, L, np.int32)
    mu, codes, cb, cnt = oracle.fit(K, cfg.dtype, sl)
    assert np.array_equal(dmu.cpu().numpy(), mu), "channel means differ"
    g_codes = dcodes.cpu().numpy()
    assert np.array_equal(g_codes[:, :, :L], codes[:, :, :L]), "codes differ"
    assert not g_codes[:, :, L:].any()
    assert np.array_equal(dcnt.cpu().numpy(), cnt), "cluster sizes differ"
    g_cb = dcb.cpu().numpy()
    for b in range(B):   # per sequence, to bound the fp64 temporaries
        Kp = np.abs(W.from_bits(K[b, :, :L], cfg.dtype).astype(np.float64) - mu[b, :, None, :]).max(axis=1)
        assert np.all(np.abs(g_cb[b] - cb[b]) <= 1e-5 * Kp.reshape(Hkv, 32, 1, 4)), ("codebook", b)
    dcb.copy_(torch.from_numpy(cb))
    return dict(sl=sl, mu=mu, codes=codes, cb=cb, gpu_cb=g_cb, gpu_cnt=dcnt), dK, dsl, dmu, dcb, dcodes


def check_sets(g_idx, r_idx, s_ref, sl, k):
    n = 0
    for b in range(g_idx.shape[0]):
        for hq in range(g_idx.shape[1]):
            n += topk_sets_agree(g_idx[b, hq], r_idx[b, hq], s_ref[b, hq], int(sl[b]), k)
    return n


def run_full(oracle, name, steps, extra_cap=32):
    cfg = W.CONFIGS[name]
    B, Hkv, Hq, D, L, k = cfg.batch, cfg.n_kv_heads, cfg.n_q_heads, cfg.head_dim, cfg.context, cfg.top_k
    ap = cfg.append
    cap = L + (extra_cap if ap else 0)
    K, V = W.make_cache(cfg, capacity=cap)
    lay = sik.make_layout(B, Hkv, Hq, D, cap, TDT[cfg.dtype], torch.float32)
    lay16 = sik.make_layout(B, Hkv, Hq, D, cap, TDT[cfg.dtype], None)
    ws = sik.alloc_workspace(lay, k)
    o, dK, dsl, dmu, dcb, dcodes = fit_both_sides(oracle, cfg, cap, K, lay, ws)
    dV = dev(V, cfg.dtype)
    sl, mu, codes, cb = o["sl"], o["mu"], o["codes"], o["cb"]
    idx = torch.empty(B, Hq, k, dtype=torch.int32, device="cuda")

    # the 16-bit output that bench.py times (no append, so that the cache is unchanged for the steps below)
    q, _, _ = W.make_step_inputs(cfg, 1000)
    out16 = torch.empty(B, Hq, D, dtype=TDT[cfg.dtype], device="cuda")
    sik.sik_decode_step(lay16, dev(q, cfg.dtype), None, None, dK, dV, dsl, dmu, dcb, dcodes, k, 0.0, out16, idx, ws)
    torch.cuda.synchronize()
    _, r_idx = oracle.decode_step(q, None, None, K, V, cfg.dtype, sl, mu, cb, codes, k)
    g_idx = idx.cpu().numpy()
    n_diff = check_sets(g_idx, r_idx, oracle.score(q, cfg.dtype, cb, codes, sl), sl, k)
    check_attention(out16.float().cpu().numpy().astype(np.float64), oracle.sparse_attn(q, K, V, cfg.dtype, g_idx),
                    False, cfg.dtype, label=f"{name} full shape")
    # every launch structure picks the same set, bit for bit (two launches, one launch, one launch with the 16-bit
    # first pass: all rank by the same binary32 sums)
    want = torch.sort(idx, dim=-1).values.clone()
    for launches in (2, 1, 3):
        idx_l = torch.full_like(idx, -7)
        sik.sik_decode_step_ex(lay16, q=dev(q, cfg.dtype), K=dK, V=dV, seq_len=dsl, mu=dmu, codebook=dcb, codes=dcodes,
                               k=k, out=out16, idx_out=idx_l, workspace=ws, launches=launches)
        torch.cuda.synchronize()
        assert sik.sik_workspace_status(ws) == 0
        assert torch.equal(torch.sort(idx_l, dim=-1).values, want), (name, launches)

    out = torch.empty(B, Hq, D, device="cuda")
    for step in range(steps):
        q, kn, vn = W.make_step_inputs(cfg, step)
        sik.sik_decode_step(lay, dev(q, cfg.dtype), dev(kn, cfg.dtype) if ap else None,
                            dev(vn, cfg.dtype) if ap else None, dK, dV, dsl, dmu, dcb, dcodes, k, 0.0, out, idx, ws)
        torch.cuda.synchronize()
        _, r_idx = oracle.decode_step(q, kn if ap else None, vn if ap else None, K, V, cfg.dtype, sl, mu, cb, codes, k)
        assert np.array_equal(dsl.cpu().numpy(), sl)
        if ap:
            t = int(sl[0]) - 1
            assert np.array_equal(bits_of_tensor(dK[:, :, t]), K[:, :, t])
            assert np.array_equal(bits_of_tensor(dV[:, :, t]), V[:, :, t])
            assert np.array_equal(dcodes[:, :, t].cpu().numpy(), codes[:, :, t])
        g_idx = idx.cpu().numpy()
        n_diff += check_sets(g_idx, r_idx, oracle.score(q, cfg.dtype, cb, codes, sl), sl, k)
        check_attention(out.cpu().numpy().astype(np.float64), oracle.sparse_attn(q, K, V, cfg.dtype, g_idx), True)
    print(f"{name}: {steps} + 1 step(s), all {B * Hkv} KV-head units and {B * Hq} query heads checked, "
          f"tie-legal index differences: {n_diff}")


def test_full_c2(oracle):
    run_full(oracle, "C2", steps=2)


def test_full_c3_with_append(oracle):
    run_full(oracle, "C3", steps=2)


def test_full_c4_large_batch(oracle):
    run_full(oracle, "C4", steps=1)


def test_full_c5_prefill_compress_then_16_steps(oracle):
    run_full(oracle, "C5", steps=16)


def run_full_q2(oracle, name, steps, extra_cap=32):
    """As run_full, on the 2-bit cache: the library quantises the whole workload (keys, then records), the
    oracle does the same from the same host bits; alpha bit-equal, every record compared under the near-tie
    rule of helpers.records_agree (exceptions counted and printed), top-k sets tie-legal, attention over the
    library's own records (decoded by the oracle in fp64) within 1e-5 relative."""
    cfg = W.CONFIGS[name]
    B, Hkv, Hq, D, L, k = cfg.batch, cfg.n_kv_heads, cfg.n_q_heads, cfg.head_dim, cfg.context, cfg.top_k
    ap = cfg.append
    cap = L + (extra_cap if ap else 0)
    K, V = W.make_cache(cfg, capacity=cap)
    lay = sik.make_layout(B, Hkv, Hq, D, cap, TDT[cfg.dtype], torch.float32)
    ws = sik.alloc_workspace(lay, k)
    o, dK, dsl, dmu, dcb, dcodes = fit_both_sides(oracle, cfg, cap, K, lay, ws)
    sl, mu, codes, cb = o["sl"], o["mu"], o["codes"], o["cb"]
    dV = dev(V, cfg.dtype)
    dal = torch.empty(B, Hkv, D, device="cuda")
    kvq = sik.alloc_kvq(lay)
    sik.sik_quantize_kv(lay, dK, dV, dsl, 0, 0, sik.SIK_Q_FIT, dmu, dal, kvq)
    # the same in one call (two passes over K, one over V): identical bits in every output
    mu2, cb2, cnt2 = torch.empty_like(dmu), torch.empty_like(dcb), torch.empty_like(o["gpu_cnt"])
    codes2, al2, kvq2 = torch.zeros_like(dcodes), torch.empty_like(dal), sik.alloc_kvq(lay)
    sik.sik_prefill_compress(lay, dK, dV, dsl, mu2, cb2, cnt2, codes2, al2, kvq2, ws)
    torch.cuda.synchronize()
    assert torch.equal(mu2, dmu) and torch.equal(codes2, dcodes) and torch.equal(cnt2, o["gpu_cnt"])
    assert np.array_equal(cb2.cpu().numpy(), o["gpu_cb"]) and torch.equal(al2, dal) and torch.equal(kvq2, kvq)
    del dK, dV, mu2, cb2, cnt2, codes2, al2, kvq2
    al, qkv = oracle.fit_q2(K, V, cfg.dtype, sl, mu)
    assert np.array_equal(dal.cpu().numpy(), al), "alpha differs"
    got = kvq.cpu().numpy()
    exc = np.zeros(4, np.int64)
    for b in range(B):
        exc += records_agree(oracle, got, K, V, cfg.dtype, mu, al, codes, qkv, b, 0, L)
        assert not got[b, :, L:].any()
    # from here on the oracle reads the library's own records (legal under the rule just checked)
    _, qkv = oracle.unpack_records(got)
    del got

    out = torch.empty(B, Hq, D, device="cuda")
    idx = torch.empty(B, Hq, k, dtype=torch.int32, device="cuda")
    n_diff = 0
    for step in range(steps):
        q, kn, vn = W.make_step_inputs(cfg, step)
        sik.sik_decode_step_q2(lay, dev(q, cfg.dtype), dev(kn, cfg.dtype) if ap else None,
                               dev(vn, cfg.dtype) if ap else None, kvq, dsl, dmu, dal, dcb, dcodes, k, 0.0, out, idx, ws)
        torch.cuda.synchronize()
        _, r_idx = oracle.decode_step_q2(q, kn if ap else None, vn if ap else None, cfg.dtype, sl, mu, al, cb, codes,
                                         qkv, k)
        assert np.array_equal(dsl.cpu().numpy(), sl)
        if ap:
            t = int(sl[0]) - 1
            row = kvq[:, :, t:t + 1].cpu().numpy()
            for b in range(B):
                exc += records_agree(oracle, row, kn[:, :, None, :], vn[:, :, None, :], cfg.dtype, mu, al, codes, qkv,
                                     b, t, t + 1, base=t)
            _, one = oracle.unpack_records(row)
            for f in ("kq", "vq", "kpar", "vpar"):
                getattr(qkv, f)[:, :, t] = getattr(one, f)[:, :, 0]
        g_idx = idx.cpu().numpy()
        n_diff += check_sets(g_idx, r_idx, oracle.score(q, cfg.dtype, cb, codes, sl), sl, k)
        check_attention(out.cpu().numpy().astype(np.float64),
                        oracle.sparse_attn_q2(q, cfg.dtype, codes, qkv, al, g_idx), True)
    print(f"{name} (2-bit cache): {steps} step(s), all {B * Hkv} units, tie-legal index differences: {n_diff}; "
          f"records inside the near-tie band: {exc[0]} of {exc[2]} parameters, {exc[1]} of {exc[3]} codes")


def test_full_c2_two_bit_cache(oracle):
    run_full_q2(oracle, "C2", steps=2)


def test_full_c4_two_bit_cache(oracle):
    run_full_q2(oracle, "C4", steps=1)


def test_full_c5_two_bit_cache_with_append(oracle):
    run_full_q2(oracle, "C5", steps=3)

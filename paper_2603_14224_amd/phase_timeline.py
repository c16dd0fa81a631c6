"""Per-phase timeline of one decode step (debug aid).

Builds the library with -DSIK_TIMELINE into paper_2603_14224_amd/libsik_timeline.so (the marks cost a few
stores per workgroup; the product library has none of them), runs decode steps of a benchmark workload on random
data of the same shapes, and prints when the first / middle / last workgroup of each kernel passed each mark, in
microseconds of the GPU's 100 MHz wall clock since the first scoring workgroup started.  The last column is the
last-arriving workgroup of query head 0.

    python -m paper_2603_14224_amd.phase_timeline C2 [--build]
"""
import ctypes
import os
import sys
import warnings

import numpy as np
import torch

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libsik_timeline.so")
SLOTS = 48
NAMES = {0: "score: entry", 1: "score: loads issued, LDS cleared", 2: "score: tables (+ bin bounds) built",
         3: "score: tokens scored", 4: "score: histograms published",
         24: "fused: entry", 25: "fused: threshold bin found", 26: "fused: scores classified",
         27: "fused: own tokens gathered", 28: "fused: partial + candidates published",
         29: "fused: last arriver starts", 32: "fused: exchange loads issued", 33: "fused: candidates in LDS",
         34: "fused: candidates ranked", 31: "fused: candidates attended", 30: "fused: output written"}


def main():
    name = sys.argv[1] if len(sys.argv) > 1 and not sys.argv[1].startswith("-") else "C2"
    if "--build" in sys.argv or not os.path.exists(LIB):
        from paper_2603_14224_amd import build as b
        b.build(defines=("SIK_TIMELINE",), lib=LIB, objdir_name="_build_timeline")
    from paper_2603_14224_amd import binding
    binding.LIB_PATH = LIB
    import paper_2603_14224_amd as sik
    sys.path.insert(0, ROOT)
    import sik_workloads as W

    cfg = W.CONFIGS[name]
    B, Hkv, Hq, D, L, k = cfg.batch, cfg.n_kv_heads, cfg.n_q_heads, cfg.head_dim, cfg.context, cfg.top_k
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float16
    lay = sik.make_layout(B, Hkv, Hq, D, L, tdt, tdt)
    ws = sik.alloc_workspace(lay, k)
    g = torch.Generator(device="cuda")
    g.manual_seed(0)
    K = torch.randn(B, Hkv, L, D, device="cuda", generator=g).to(tdt)
    V = torch.randn(B, Hkv, L, D, device="cuda", generator=g).to(tdt)
    sl = torch.full((B,), L, dtype=torch.int32, device="cuda")
    mu = torch.empty(B, Hkv, D, device="cuda")
    cb = torch.empty(B, Hkv, D // 4, 16, 4, device="cuda")
    cnt = torch.empty(B, Hkv, D // 4, 16, dtype=torch.int32, device="cuda")
    codes = torch.zeros(B, Hkv, L, D // 8, dtype=torch.uint8, device="cuda")
    sik.sik_quantize_keys(lay, K, sl, 0, 0, sik.SIK_Q_FIT, mu, cb, cnt, codes, ws)
    # a different query every step: each selects its own rows, so a step does not find its rows in the caches
    # because the previous step gathered the same ones
    qs = [torch.randn(B, Hq, D, device="cuda", generator=g).to(tdt) for _ in range(8)]
    out = torch.empty(B, Hq, D, dtype=tdt, device="cuda")
    tl = torch.zeros(4 * SLOTS, dtype=torch.int64, device="cuda")
    lib = sik.lib()
    for fn in ("sik_dbg_tl_score", "sik_dbg_tl_topk", "sik_dbg_tl_attn", "sik_dbg_tl_fused"):
        assert getattr(lib, fn)(ctypes.c_void_p(tl.data_ptr())) == 0
    acc, reps = {}, 20
    for r in range(reps + 3):
        tl.zero_()
        torch.cuda.synchronize()
        sik.sik_decode_step(lay, qs[r % len(qs)], None, None, K, V, sl, mu, cb, codes, k, 0.0, out, None, ws)
        torch.cuda.synchronize()
        t = tl.cpu().numpy().astype(np.int64).reshape(SLOTS, 4)
        if r < 3:
            continue
        t0 = t[0][:3][t[0][:3] > 0].min()
        for s_ in NAMES:
            if t[s_].max() > 0:
                acc.setdefault(s_, []).append([(x - t0) / 100.0 if x > 0 else np.nan for x in t[s_]])
    warnings.simplefilter("ignore")
    print(f"{cfg.name}: mean of {reps} steps, us since the first scoring workgroup started")
    print(f"  {'mark':40s} {'first WG':>9s} {'middle WG':>9s} {'last WG':>9s} {'head 0 last arriver':>20s}")
    rows = sorted(acc.items(), key=lambda kv: np.nanmin(np.array(kv[1])))
    for s_, v in rows:
        a = np.nanmean(np.array(v), axis=0)
        cells = " ".join(f"{x:9.2f}" if not np.isnan(x) else f"{'':9s}" for x in a[:3])
        last = f"{a[3]:20.2f}" if not np.isnan(a[3]) else ""
        print(f"  {NAMES[s_]:40s} {cells} {last}")


if __name__ == "__main__":
    main()

#!/usr/bin/env python3
"""Benchmark of the Self-Indexing KV cache decode step on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input: [quantise-append]
-> lookup table -> LUT-GEMV scores over the 1-bit code plane -> per-head top-k -> sparse attention
over the selected 16-bit K/V rows, for one attention layer.  The default workload is the
Llama-3-8B-shaped 32K-context layer decode (batch 1, 8 KV heads, 32 query heads, head_dim 128,
top-k 1024, bf16).  Inputs are resident in HBM before the timed region; steps rotate over several
distinct layer states so that the working set exceeds the 256 MB Infinity Cache.

Prints ONE JSON line.  One GPU only.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

HBM_PEAK_GBPS = 8000.0
# HBM bytes per launch of the dominant kernel.  Hardware counters cannot be read from inside this process: these are
# the FETCH_SIZE + WRITE_SIZE figures of the committed rocprofv3 --pmc runs of this same command (file named beside
# each; counter units x the factor a 256 MiB plain copy calibrates there).  Workloads or variants without such a
# run report null.
MEASURED_TRAFFIC = {
    ("C2", "select_attend_kernel"): (29488988, "profiles/decode_step_two_launches_C2_C3.md"),
    ("C3", "select_attend_kernel"): (58730732, "profiles/decode_step_two_launches_C2_C3.md"),
    ("C4", "step_kernel"): (335015269, "profiles/decode_step_one_launch_C4_C5.md"),
    ("C5", "step_kernel"): (277505678, "profiles/decode_step_one_launch_C4_C5.md"),
}
# execution times returned by sik_decode_step_profiled, in launch order: small launches run scoring, then fused
# selection + attention; large ones run as one launch, reported in the last slot and named step_kernel here
KERNELS = ("prep_kernel", "score_kernel", "select_kernel", "select_attend_kernel")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400, help="decode steps per timed block")
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--reps", type=int, default=11,
                    help="timed repetitions of the block of --steps steps; the median block gives `value`")
    ap.add_argument("--config", default="C2", choices=["C1", "C2", "C3", "C4", "C5", "T4"])
    ap.add_argument("--also", default=None,
                    help="comma-separated further workloads measured the same way and nested under \"also\" "
                         "(default: C3, the 128K context of the metric, and C4, the large batch that takes the "
                         "one-launch step, when --config is C2 and no variant is on; \"none\" switches it off)")
    ap.add_argument("--layers", type=int, default=0, help="distinct layer states to rotate over (0 = auto)")
    ap.add_argument("--no-graph", action="store_true", help="time plain stream launches only, no HIP-graph replay")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    ap.add_argument("--kv", default="rows", choices=["rows", "q2"],
                    help="rows: 16-bit K/V rows (the headline metric); q2: the 2-bit token-wise cache, one 128-byte "
                         "record per token, dequantised inside the attention kernel")
    ap.add_argument("--forced", type=int, default=0,
                    help="forced-inclusion set of this many tokens per KV head (the paper's 64 sink tokens; with "
                         "--kv q2 kept as 16-bit side rows); the budget top_k then counts them")
    ap.add_argument("--shared", action="store_true",
                    help="group-shared selection: one index set per KV head from the summed scores of its query heads")
    ap.add_argument("--launches", type=int, default=0, choices=[0, 1, 2, 3],
                    help="0: the library's choice; 1: the one-launch step whenever its plan allows; 2: scoring and "
                         "selection + attention as two launches (comparison runs; the headline uses 0)")
    ap.add_argument("--fit", action="store_true",
                    help="measure the prefill-side quantiser instead of the decode step (one layer of the workload)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="first run one plain elementwise copy of 256 MiB (read 256 MiB, write 256 MiB): under "
                         "rocprofv3 --pmc its FETCH_SIZE / WRITE_SIZE give the counters' scale factor")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build measures ONE GPU (batch and KV heads shard without any exchange); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)

    import torch

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.copy_calibration:
        src = torch.ones(64 * 2 ** 20, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.add(src, 1.0, out=dst)  # one launch: 256 MiB read + 256 MiB written
        torch.cuda.synchronize()
        del src, dst
    if args.fit:
        return bench_fit(args)
    variant = args.kv != "rows" or args.forced or args.shared
    also = args.also if args.also is not None else ("C3,C4" if args.config == "C2" and not variant else "none")
    result = bench_decode(args, args.config, cpu=not args.no_cpu_baseline and not args.forced and not args.shared)
    extra = [bench_decode(args, name, cpu=False) for name in also.split(",") if name not in ("", "none", args.config)]
    if extra:
        keep = ("value", "unit", "steps", "warmup", "reps", "ms_per_step", "config", "effective_hbm_GBps",
                "effective_hbm_frac_of_8TBps", "algorithmic_bytes_per_step", "us_per_step_stream_launch",
                "us_per_step_hipgraph", "us_per_block_percentiles", "kernel_us", "roofline")
        result["also"] = [{k_: r[k_] for k_ in keep} for r in extra]
    print(json.dumps(result))


def bench_decode(args, name, cpu):
    """One workload: resident state, warm-up, --reps timed blocks of exactly --steps steps (stream launches and
    HIP-graph replay), per-kernel execution times, roofline.  Returns the result dictionary."""
    import numpy as np
    import torch

    import paper_2603_14224_amd as sik
    import sik_workloads as W
    from helpers import dev

    cfg = W.CONFIGS[name]
    B, Hkv, Hq, D, L, k = cfg.batch, cfg.n_kv_heads, cfg.n_q_heads, cfg.head_dim, cfg.context, cfg.top_k
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float16
    q2 = args.kv == "q2"
    K_steps, reps = args.steps, max(1, args.reps)
    per_layer = (B * Hkv * L * 128 if q2 else 2 * B * Hkv * L * D * 2) + B * Hkv * L * (D // 8)
    n_layers = args.layers or max(2, min(16, -(-2 * 256 * 2 ** 20 // per_layer)))
    # capacity: room for the rows one block (or the warm-up) appends to a layer; lengths are reset between blocks
    n_new = -(-max(K_steps, args.warmup) // n_layers) + 1 if cfg.append else 1
    cap = (L + (n_new + 8 if cfg.append else 0) + 7) // 8 * 8
    lay = sik.make_layout(B, Hkv, Hq, D, cap, tdt, tdt)
    ws = sik.alloc_workspace(lay, k)

    # ---- resident state: n_layers independent draws of the recipe, quantised by the library itself
    layers = []
    t0 = time.time()
    for li in range(n_layers):
        Kb, Vb = W.make_cache(cfg, capacity=cap, layer=li)
        st = dict(K=dev(Kb, cfg.dtype), V=dev(Vb, cfg.dtype),
                  sl=torch.full((B,), L, dtype=torch.int32, device="cuda"),
                  mu=torch.empty(B, Hkv, D, device="cuda"),
                  cb=torch.empty(B, Hkv, D // 4, 16, 4, device="cuda"),
                  cnt=torch.empty(B, Hkv, D // 4, 16, dtype=torch.int32, device="cuda"),
                  codes=torch.zeros(B, Hkv, cap, D // 8, dtype=torch.uint8, device="cuda"))
        sik.sik_quantize_keys(lay, st["K"], st["sl"], 0, 0, sik.SIK_Q_FIT, st["mu"], st["cb"], st["cnt"],
                              st["codes"], ws)
        if q2:  # the records replace the 16-bit rows, which are dropped
            st["alpha"] = torch.empty(B, Hkv, D, device="cuda")
            st["kvq"] = sik.alloc_kvq(lay)
            sik.sik_quantize_kv(lay, st["K"], st["V"], st["sl"], 0, 0, sik.SIK_Q_FIT, st["mu"], st["alpha"],
                                st["kvq"])
            torch.cuda.synchronize()
            st["K"] = st["V"] = None
        if args.forced:  # the first tokens of the context, as attention sinks usually are
            st["fidx"] = torch.arange(args.forced, dtype=torch.int32, device="cuda").repeat(B, Hkv, 1).contiguous()
            if q2:
                st["fK"] = dev(Kb[:, :, :args.forced], cfg.dtype).contiguous()
                st["fV"] = dev(Vb[:, :, :args.forced], cfg.dtype).contiguous()
        if li == 0 and cpu:
            host0 = (Kb, Vb)
        layers.append(st)
    del Kb, Vb
    torch.cuda.synchronize()
    # step inputs: 8 distinct queries reused in turn (each selects its own rows, so a replayed block does not find
    # the rows it gathers still cached from the same query on the same layer); appended key/value rows are
    # distinct for every step a layer sees inside a block (repeating a key would plant exact score ties that real
    # decoding does not have)
    n_q = 8
    qs = [dev(W.make_step_inputs(cfg, s)[0], cfg.dtype) for s in range(n_q)]
    kn_all, vn_all = [], []
    for s in range(n_new):
        _, kn, vn = W.make_step_inputs(cfg, 1000 + s)
        kn_all.append(kn)
        vn_all.append(vn)
    kns = dev(np.stack(kn_all), cfg.dtype)   # [n_new, B, Hkv, D]
    vns = dev(np.stack(vn_all), cfg.dtype)
    out = torch.empty(B, Hq, D, dtype=tdt, device="cuda")
    gen_s = time.time() - t0

    def step(i, profiled=False, idx_out=None):
        """Step i of a block: layer i mod n_layers, query i mod 8, the (i div n_layers)-th new row of that layer."""
        st = layers[i % n_layers]
        j = i % n_q
        a = (i // n_layers) % n_new
        kn, vn = (kns[a], vns[a]) if cfg.append else (None, None)
        if args.forced or args.shared or args.launches:
            return sik.sik_decode_step_ex(lay, q=qs[j], k_new=kn, v_new=vn, K=st["K"], V=st["V"], kvq=st.get("kvq"),
                                          alpha=st.get("alpha"), seq_len=st["sl"], mu=st["mu"], codebook=st["cb"],
                                          codes=st["codes"], k=k, out=out, idx_out=idx_out, workspace=ws,
                                          forced_idx=st.get("fidx"), forced_K=st.get("fK"), forced_V=st.get("fV"),
                                          group_shared=args.shared, profiled=profiled, launches=args.launches)
        if q2:
            return sik.sik_decode_step_q2(lay, qs[j], kn, vn, st["kvq"], st["sl"], st["mu"], st["alpha"], st["cb"],
                                          st["codes"], k, 0.0, out, idx_out, ws, profiled=profiled)
        fn = sik.sik_decode_step_profiled if profiled else sik.sik_decode_step
        return fn(lay, qs[j], kn, vn, st["K"], st["V"], st["sl"], st["mu"], st["cb"], st["codes"], k, 0.0, out,
                  idx_out, ws)

    def reset_lengths():
        for st in layers:
            st["sl"].fill_(L)
        torch.cuda.synchronize()

    # ---- warm-up (untimed)
    for i in range(args.warmup):
        step(i)
    reset_lengths()

    # ---- the timed region: a block = exactly --steps steps between two synchronisations, --reps blocks, each
    # starting from the same state (lengths reset outside the timed region); `value` is the median block
    def timed_blocks(run_block):
        secs = []
        for _ in range(reps):
            reset_lengths()
            t = time.perf_counter()
            run_block()
            torch.cuda.synchronize()
            secs.append((time.perf_counter() - t) / K_steps)
        return np.sort(np.array(secs))

    def stream_block():
        for i in range(K_steps):
            step(i)

    s_stream = timed_blocks(stream_block)
    sec_stream = float(np.median(s_stream))
    s_best, sec_step, launch = s_stream, sec_stream, "stream"
    sec_graph = None
    if not args.no_graph:
        reset_lengths()
        side = torch.cuda.Stream()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            stream_block()
            reset_lengths()
            with torch.cuda.graph(g, stream=side):   # one graph = the --steps steps of a block, nothing else
                stream_block()
        torch.cuda.synchronize()
        reset_lengths()
        g.replay()
        s_graph = timed_blocks(g.replay)
        sec_graph = float(np.median(s_graph))
        if sec_graph < sec_stream:
            s_best, sec_step, launch = s_graph, sec_graph, "hipgraph"
    reset_lengths()
    pct = {f"p{p}": round(float(np.percentile(s_best, p)) * 1e6, 3) for p in (10, 50, 90)}
    pct.update(min=round(float(s_best[0]) * 1e6, 3), blocks=reps, steps_per_block=K_steps, launch=launch)

    # ---- rows the gather really touches: query heads of one GQA group may select the same token
    idx = torch.empty(B, Hkv if args.shared else Hq, k, dtype=torch.int32, device="cuda")
    step(0, idx_out=idx)
    torch.cuda.synchronize()
    srt = idx.view(B * Hkv, -1).sort(dim=1).values
    fresh = torch.ones_like(srt, dtype=torch.bool)
    fresh[:, 1:] = srt[:, 1:] != srt[:, :-1]
    rows_unique = int((fresh & (srt >= 0)).sum())
    rows_nominal = int((idx >= 0).sum())
    del idx, srt, fresh
    reset_lengths()

    # ---- execution time of each kernel: the begin / end timestamps of its dispatch (what a profiler's kernel
    # trace reports), over the steps of one block; the last figure is the span of the step on the GPU
    raw = np.zeros(5)
    n_prof = min(K_steps, 200)
    for i in range(n_prof):
        raw += np.array(step(i, profiled=True))
    raw /= n_prof
    kus = raw[:4]
    reset_lengths()
    # a step that ran as one launch reports its only kernel in the last slot
    names = list(KERNELS)
    if kus[1] == 0 and kus[3] > 0:
        names[3] = "step_kernel"

    ab = W.algorithmic_bytes(cfg)
    if q2:  # a selected (query head, token) costs one 128-byte record instead of 2 x 256 bytes of rows
        ab = dict(ab, gathered=ab["gathered"] // 4)
        ab["total"] = ab["codes"] + ab["gathered"]
    if args.shared:  # the R query heads of a KV head attend over one set of rows
        ab = dict(ab, gathered=ab["gathered"] // (Hq // Hkv))
        ab["total"] = ab["codes"] + ab["gathered"]
    alg_by_kernel = {"prep_kernel": (B * Hkv * (2 * D * 2 + D // 8)) if cfg.append else 0,
                     "score_kernel": ab["codes"], "select_kernel": 0,
                     "select_attend_kernel": ab["gathered"], "step_kernel": ab["codes"] + ab["gathered"]}
    dom = max((1, 3), key=lambda i: kus[i])  # the kernels that move the algorithmic bytes
    dom_name = names[dom]
    dom_bytes = alg_by_kernel[dom_name]
    achieved = dom_bytes / (kus[dom] * 1e-6) / 1e9
    variant = q2 or args.forced or args.shared
    traffic = None if variant or args.launches else MEASURED_TRAFFIC.get((name, dom_name))

    step_us = sec_step * 1e6
    result = {
        "metric": "us per sparse decode step (and effective HBM GB/s)",
        "value": round(step_us, 3),
        "unit": "us/step",
        "n_gpus": 1,
        "steps": K_steps,
        "warmup": args.warmup,
        "reps": reps,
        "ms_per_step": round(sec_step * 1e3, 6),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": cfg.dtype,
        "arithmetic": f"{cfg.dtype} storage of K, V, q and the output; fp32 lookup tables, score sums and softmax",
        "data": "synthetic",
        "config": {"workload": cfg.name, "batch": B, "n_kv_heads": Hkv, "n_q_heads": Hq, "head_dim": D,
                   "context": L, "top_k": k, "kv_dtype": cfg.dtype, "kv_format": args.kv,
                   "forced_tokens": args.forced, "group_shared": args.shared, "append": cfg.append,
                   "layers_rotated": n_layers, "launch": launch,
                   "kernels_per_step": int((kus > 0).sum())},
        "effective_hbm_GBps": round(ab["total"] / sec_step / 1e9, 1),
        "effective_hbm_frac_of_8TBps": round(ab["total"] / sec_step / 1e9 / HBM_PEAK_GBPS, 4),
        "algorithmic_bytes_per_step": ab["total"],
        "us_per_step_stream_launch": round(sec_stream * 1e6, 3),
        "us_per_step_hipgraph": None if sec_graph is None else round(sec_graph * 1e6, 3),
        "us_per_block_percentiles": pct,
        "gathered_rows": {"nominal": rows_nominal, "unique_per_kv_head": rows_unique},
        "kernel_us": dict({names[i]: round(float(kus[i]), 3) for i in range(4) if kus[i] > 0},
                          sum=round(float(kus.sum()), 3), steps_profiled=n_prof, how="begin/end timestamps of each dispatch (HIP events handed to "
                                                      "the launch), mean over the steps of one block"),
        "roofline": {"bound": "hbm", "kernel": dom_name, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "traffic": None if traffic is None else traffic[0],
                     "traffic_source": None if traffic is None else traffic[1],
                     "algorithmic_bytes_per_launch": dom_bytes},
        "setup_seconds": round(gen_s, 1),
    }
    if cpu:
        result["cpu_baseline"] = cpu_baseline(cfg, host0, args.cpu_seconds, q2)
    del layers, ws
    torch.cuda.empty_cache()
    return result


def bench_fit(args):
    """Prefill-side compression of one layer ("one-pass sign-based clustering": means, codes, codebook; with --kv q2
    also alpha and the 2-bit records): value = sik_quantize_keys FIT (two passes over K), or with --kv q2
    sik_prefill_compress (two passes over K, one over V); the separate calls (four passes over K, one over V) and
    one plain read of K and V (a reduction over both tensors: the least any prefill-side pass costs) are timed
    beside it.  Rotates over enough layer copies of K (and V) to stay out of the Infinity Cache."""
    import numpy as np
    import torch

    import paper_2603_14224_amd as sik
    import sik_workloads as W
    from helpers import dev

    cfg = W.CONFIGS[args.config]
    q2 = args.kv == "q2"
    cap = cfg.context
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float16
    lay = sik.make_layout(cfg.batch, cfg.n_kv_heads, cfg.n_q_heads, cfg.head_dim, cap, tdt, tdt)
    ws = sik.alloc_workspace(lay, cfg.top_k)
    B, Hkv, D, L = cfg.batch, cfg.n_kv_heads, cfg.head_dim, cfg.context
    kv_bytes = B * Hkv * L * D * 2
    n_layers = args.layers or max(2, min(8, -(-2 * 256 * 2 ** 20 // kv_bytes)))
    Ks, Vs = [], []
    for li in range(n_layers):
        Kb, Vb = W.make_cache(cfg, capacity=cap, layer=li)
        Ks.append(dev(Kb, cfg.dtype))
        Vs.append(dev(Vb, cfg.dtype) if q2 else None)
    sl = torch.full((B,), L, dtype=torch.int32, device="cuda")
    mu = torch.empty(B, Hkv, D, device="cuda")
    cb = torch.empty(B, Hkv, D // 4, 16, 4, device="cuda")
    cnt = torch.empty(B, Hkv, D // 4, 16, dtype=torch.int32, device="cuda")
    codes = torch.zeros(B, Hkv, cap, D // 8, dtype=torch.uint8, device="cuda")
    alpha = torch.empty(B, Hkv, D, device="cuda") if q2 else None
    kvq = sik.alloc_kvq(lay) if q2 else None

    def separate(i):
        sik.sik_quantize_keys(lay, Ks[i % n_layers], sl, 0, 0, sik.SIK_Q_FIT, mu, cb, cnt, codes, ws)
        if q2:
            sik.sik_quantize_kv(lay, Ks[i % n_layers], Vs[i % n_layers], sl, 0, 0, sik.SIK_Q_FIT, mu, alpha, kvq)

    def fused(i):
        sik.sik_prefill_compress(lay, Ks[i % n_layers], Vs[i % n_layers], sl, mu, cb, cnt, codes, alpha, kvq, ws)

    def plain_read(i):
        Ks[i % n_layers].view(torch.int32).max()
        if q2:
            Vs[i % n_layers].view(torch.int32).max()

    steps, warmup, reps = min(args.steps, 50), min(args.warmup, 5), max(1, min(args.reps, 5))

    def timed(fn):
        for i in range(warmup):
            fn(i)
        secs = []
        for _ in range(reps):
            torch.cuda.synchronize()
            t = time.perf_counter()
            for i in range(steps):
                fn(warmup + i)
            torch.cuda.synchronize()
            secs.append((time.perf_counter() - t) / steps)
        return float(np.median(secs))

    sec_sep = timed(separate)
    sec_read = timed(plain_read)
    sec = timed(fused) if q2 else sec_sep
    # algorithmic traffic: K twice (means, then codes + clusters [+ records]), V once, codes and records written
    nbytes = kv_bytes * (3 if q2 else 2) + B * Hkv * L * (D // 8) + (B * Hkv * L * 128 if q2 else 0)
    read_bytes = kv_bytes * (2 if q2 else 1)
    print(json.dumps({
        "metric": "us per prefill-side compression of one layer", "value": round(sec * 1e6, 2),
        "unit": "us/layer", "n_gpus": 1, "steps": steps, "warmup": warmup, "reps": reps,
        "ms_per_step": round(sec * 1e3, 5),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": cfg.name + " / prefill-compress", "batch": B, "n_kv_heads": Hkv, "head_dim": D,
                   "context": L, "kv_dtype": cfg.dtype, "kv_format": args.kv, "layers_rotated": n_layers,
                   "entry_point": "sik_prefill_compress" if q2 else "sik_quantize_keys"},
        "separate_calls_us": round(sec_sep * 1e6, 2),
        "plain_read_of_K" + ("_and_V" if q2 else "") + "_us": round(sec_read * 1e6, 2),
        "plain_read_GBps": round(read_bytes / sec_read / 1e9, 1),
        "ratio_to_plain_read": round(sec / sec_read, 2),
        "roofline": {"bound": "hbm", "kernel": "colsum + encode" + (" (with alpha and records)" if q2 else ""),
                     "achieved": round(nbytes / sec / 1e9, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(nbytes / sec / 1e9 / HBM_PEAK_GBPS, 4), "traffic": None,
                     "algorithmic_bytes_per_launch": nbytes}}))


def cpu_baseline(cfg, host0, budget_s, q2=False):
    """The CPU oracle, as it stands, on the same workload's layer 0: whole decode steps on the host
    cores of this machine (OpenMP over batch x head), as many as fit the time budget."""
    import numpy as np

    import sik_workloads as W
    from oracle import sik_oracle as oracle

    cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    cores = min(cores, int(os.environ.get("OMP_NUM_THREADS", cores)))
    used = oracle.set_threads(cores)
    K, V = host0
    B, cap = K.shape[0], K.shape[2]
    sl = np.full(B, cfg.context, np.int32)
    t = time.perf_counter()
    mu, codes, cb, cnt = oracle.fit(K, cfg.dtype, sl)
    stages = {"quantise_fit": time.perf_counter() - t}
    if q2:
        al, qkv = oracle.fit_q2(K, V, cfg.dtype, sl, mu)

    def one(q, kn, vn):
        if q2:
            oracle.decode_step_q2(q, kn, vn, cfg.dtype, sl, mu, al, cb, codes, qkv, cfg.top_k)
        else:
            oracle.decode_step(q, kn, vn, K, V, cfg.dtype, sl, mu, cb, codes, cfg.top_k)

    # the stages of one step, timed apart (16-bit cache, no append)
    q0 = W.make_step_inputs(cfg, 10 ** 6)[0]
    t = time.perf_counter()
    s0 = oracle.score(q0, cfg.dtype, cb, codes, sl)
    stages["score"] = time.perf_counter() - t
    t = time.perf_counter()
    i0 = oracle.topk(s0, sl, cfg.top_k)
    stages["topk"] = time.perf_counter() - t
    t = time.perf_counter()
    oracle.sparse_attn(q0, K, V, cfg.dtype, i0)
    stages["attention"] = time.perf_counter() - t
    del s0, i0

    n, t_total = 0, 0.0
    while True:
        q, kn, vn = W.make_step_inputs(cfg, n)
        t = time.perf_counter()
        if cfg.append and sl.max() < cap:
            one(q, kn, vn)
        else:
            one(q, None, None)
        t_total += time.perf_counter() - t
        n += 1
        if t_total >= budget_s or n >= 128:  # (128 steps of the 32K workload: about 18 core-seconds)
            break
    oracle.set_threads(1)
    res = {"value": round(t_total / n * 1e6, 1), "unit": "us/step", "cores": used, "kind": "oracle",
           "sample": f"{n} whole decode step(s) of layer 0 of the same workload (fp64 oracle, OpenMP over batch x head)",
           "stages_us": {k_: round(v * 1e6, 1) for k_, v in stages.items()}}
    if t_total / n * used <= budget_s:  # one more step on a single thread, when that fits the budget too
        q, _, _ = W.make_step_inputs(cfg, n)
        t = time.perf_counter()
        one(q, None, None)
        res["single_thread_us_per_step"] = round((time.perf_counter() - t) * 1e6, 1)
    return res


if __name__ == "__main__":
    main()

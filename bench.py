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
# HBM bytes per launch of the dominant kernel, from the FETCH_SIZE and WRITE_SIZE counter runs whose summaries are
# profiles/decode_step_C2_32k.md and profiles/decode_step_C3_C4_C5.md (counter units x the factor a 256 MiB plain
# copy calibrates: 2 KiB and 1 KiB).  Counters cannot be read from inside this process, so workloads without such a
# committed run report null.
MEASURED_TRAFFIC_BYTES = {("C2", "select_attend_kernel"): int(14269.1 * 2048 + 252.9 * 1024),
                          ("C3", "select_attend_kernel"): int(28470.9 * 2048 + 538.2 * 1024),
                          ("C4", "select_attend_kernel"): int(168768.0 * 2048 + 2679.4 * 1024),
                          ("C5", "select_attend_kernel"): int(141435.2 * 2048 + 2586.5 * 1024)}
# event intervals of sik_decode_step_profiled, in launch order; the third one is empty when selection and
# attention run fused in one launch (every benchmark workload)
KERNELS = ("prep_kernel", "score_kernel", "select_kernel_unfused_only", "select_attend_kernel")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--config", default="C2", choices=["C1", "C2", "C3", "C4", "C5", "T4"])
    ap.add_argument("--layers", type=int, default=0, help="distinct layer states to rotate over (0 = auto)")
    ap.add_argument("--no-graph", action="store_true", help="time plain stream launches instead of HIP-graph replay")
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
    ap.add_argument("--fit", action="store_true",
                    help="measure the prefill-side quantiser instead of the decode step: sik_quantize_keys FIT "
                         "(channel means, sign codes, codebook) and, with --kv q2, sik_quantize_kv FIT (alpha, records) "
                         "of one layer of the workload")
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

    import numpy as np
    import torch

    import paper_2603_14224_amd as sik
    import sik_workloads as W
    from helpers import dev

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.copy_calibration:
        src = torch.ones(64 * 2 ** 20, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.add(src, 1.0, out=dst)  # one launch: 256 MiB read + 256 MiB written
        torch.cuda.synchronize()
        del src, dst
    cfg = W.CONFIGS[args.config]
    B, Hkv, Hq, D, L, k = cfg.batch, cfg.n_kv_heads, cfg.n_q_heads, cfg.head_dim, cfg.context, cfg.top_k
    tdt = torch.bfloat16 if cfg.dtype == "bf16" else torch.float16
    q2 = args.kv == "q2"
    per_layer = (B * Hkv * L * 128 if q2 else 2 * B * Hkv * L * D * 2) + B * Hkv * L * (D // 8)
    n_layers = args.layers or max(2, min(16, -(-2 * 256 * 2 ** 20 // per_layer)))
    total_steps = args.warmup + args.steps
    # capacity: room for the appended rows of every step that lands on a layer
    cap = L + (-(-total_steps * 3 // n_layers) + 8 if cfg.append else 0)
    cap = (cap + 7) // 8 * 8
    lay = sik.make_layout(B, Hkv, Hq, D, cap, tdt, tdt)
    ws = sik.alloc_workspace(lay, k)
    if args.fit:
        return bench_fit(args, cfg, lay, ws, cap, q2)

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
        if li == 0:
            host0 = (Kb, Vb)
        layers.append(st)
    torch.cuda.synchronize()
    # step inputs: 8 distinct queries reused in turn; appended key/value rows are distinct for every
    # step a layer sees (repeating a key would plant exact score ties that real decoding does not have)
    n_q = 8
    qs = [dev(W.make_step_inputs(cfg, s)[0], cfg.dtype) for s in range(n_q)]
    n_new = (-(-total_steps // n_layers) + 2) if cfg.append else 1
    kn_all, vn_all = [], []
    for s in range(n_new):
        _, kn, vn = W.make_step_inputs(cfg, 1000 + s)
        kn_all.append(kn); vn_all.append(vn)
    kns = dev(np.stack(kn_all), cfg.dtype)   # [n_new, B, Hkv, D]
    vns = dev(np.stack(vn_all), cfg.dtype)
    out = torch.empty(B, Hq, D, dtype=tdt, device="cuda")
    gen_s = time.time() - t0

    def step(i, profiled=False, base=0):
        st = layers[i % n_layers]
        j = i % n_q
        a = ((i - base) // n_layers) % n_new  # how many rows this layer has been given since its reset
        kn, vn = (kns[a], vns[a]) if cfg.append else (None, None)
        if args.forced or args.shared:
            return sik.sik_decode_step_ex(lay, q=qs[j], k_new=kn, v_new=vn, K=st["K"], V=st["V"], kvq=st.get("kvq"),
                                          alpha=st.get("alpha"), seq_len=st["sl"], mu=st["mu"], codebook=st["cb"],
                                          codes=st["codes"], k=k, out=out, workspace=ws, forced_idx=st.get("fidx"),
                                          forced_K=st.get("fK"), forced_V=st.get("fV"), group_shared=args.shared,
                                          profiled=profiled)
        if q2:
            return sik.sik_decode_step_q2(lay, qs[j], kn, vn, st["kvq"], st["sl"], st["mu"], st["alpha"], st["cb"],
                                          st["codes"], k, 0.0, out, None, ws, profiled=profiled)
        fn = sik.sik_decode_step_profiled if profiled else sik.sik_decode_step
        return fn(lay, qs[j], kn, vn, st["K"], st["V"], st["sl"], st["mu"], st["cb"], st["codes"], k, 0.0, out, None,
                  ws)

    def reset_lengths():
        for st in layers:
            st["sl"].fill_(L)

    # ---- warm-up (untimed), then the timed region: exactly --steps steps between two synchronisations
    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()

    def timed_stream():
        torch.cuda.synchronize()
        t = time.perf_counter()
        for i in range(args.steps):
            step(args.warmup + i)
        torch.cuda.synchronize()
        return (time.perf_counter() - t) / args.steps

    launch = "stream"
    sec_stream = timed_stream()
    sec_step = sec_stream
    sec_graph = None
    if not args.no_graph:
        # one graph = `rounds` decode steps on every layer in turn.  With append, the graph first resets
        # the lengths (one small fill per layer, inside the timed region) so that every replay appends
        # the same `rounds` distinct rows at the same positions instead of piling up copies.
        # A graph covers every one of the n_q queries (each selects its own rows), so that replays do not
        # find the rows they gather still in the Infinity Cache from the previous replay.
        rounds = min(n_q, n_new - 1) if cfg.append else math.lcm(n_layers, n_q) // n_layers
        per_graph = n_layers * rounds
        reps = max(1, args.steps // per_graph)

        def graph_body():
            if cfg.append:
                reset_lengths()
            for i in range(per_graph):
                step(i)

        reset_lengths()
        side = torch.cuda.Stream()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            graph_body()
            torch.cuda.synchronize()
            reset_lengths()
            torch.cuda.synchronize()
            with torch.cuda.graph(g, stream=side):
                graph_body()
        torch.cuda.synchronize()
        reset_lengths()
        for _ in range(max(1, args.warmup // per_graph)):
            g.replay()
        torch.cuda.synchronize()
        t = time.perf_counter()
        for _ in range(reps):
            g.replay()
        torch.cuda.synchronize()
        sec_graph = (time.perf_counter() - t) / (reps * per_graph)
        if sec_graph < sec_stream:
            sec_step, launch = sec_graph, "hipgraph"
    reset_lengths()

    # ---- spread of the step time: events on the launch stream around groups of `grp` consecutive steps (a
    # single step is shorter than the cost of an event pair); percentiles of the group means
    grp = 2 * n_layers
    n_grp = max(1, min(40, total_steps // grp))
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n_grp)]
    for gi, (e0, e1) in enumerate(ev):
        e0.record()
        for i in range(grp):
            step(gi * grp + i)
        e1.record()
    torch.cuda.synchronize()
    grp_us = np.sort(np.array([e0.elapsed_time(e1) for e0, e1 in ev]) * 1e3 / grp)
    pct = {f"p{p}": round(float(np.percentile(grp_us, p)), 3) for p in (10, 50, 90)}
    reset_lengths()

    # ---- rows the gather really touches: query heads of one GQA group may select the same token
    idx = torch.empty(B, Hq, k, dtype=torch.int32, device="cuda")
    st0 = layers[0]
    if args.shared:
        idx = torch.empty(B, Hkv, k, dtype=torch.int32, device="cuda")
    if args.forced or args.shared:
        sik.sik_decode_step_ex(lay, q=qs[0], k_new=kns[0] if cfg.append else None,
                               v_new=vns[0] if cfg.append else None, K=st0["K"], V=st0["V"], kvq=st0.get("kvq"),
                               alpha=st0.get("alpha"), seq_len=st0["sl"], mu=st0["mu"], codebook=st0["cb"],
                               codes=st0["codes"], k=k, out=out, idx_out=idx, workspace=ws,
                               forced_idx=st0.get("fidx"), forced_K=st0.get("fK"), forced_V=st0.get("fV"),
                               group_shared=args.shared)
    elif q2:
        sik.sik_decode_step_q2(lay, qs[0], kns[0] if cfg.append else None, vns[0] if cfg.append else None,
                               st0["kvq"], st0["sl"], st0["mu"], st0["alpha"], st0["cb"], st0["codes"], k, 0.0, out,
                               idx, ws)
    else:
        sik.sik_decode_step(lay, qs[0], kns[0] if cfg.append else None, vns[0] if cfg.append else None, st0["K"],
                            st0["V"], st0["sl"], st0["mu"], st0["cb"], st0["codes"], k, 0.0, out, idx, ws)
    torch.cuda.synchronize()
    srt = idx.view(B * Hkv, -1).sort(dim=1).values
    fresh = torch.ones_like(srt, dtype=torch.bool)
    fresh[:, 1:] = srt[:, 1:] != srt[:, :-1]
    rows_unique = int((fresh & (srt >= 0)).sum())
    rows_nominal = int((idx >= 0).sum())
    del idx, srt, fresh
    reset_lengths()

    # ---- per-kernel durations, HIP events on the launch stream, same steps as the timed region
    # (each interval includes the cost of the event pair; an empty interval measured in the same call
    # is subtracted)
    raw = np.zeros(5)
    n_prof = min(args.steps, 200)
    for i in range(n_prof):
        raw += np.array(step(args.warmup + i, profiled=True))
    raw /= n_prof
    kus = np.maximum(raw[:4] - raw[4], 0.05)
    reset_lengths()

    ab = W.algorithmic_bytes(cfg)
    if q2:  # a selected (query head, token) costs one 128-byte record instead of 2 x 256 bytes of rows
        ab = dict(ab, gathered=ab["gathered"] // 4)
        ab["total"] = ab["codes"] + ab["gathered"]
    if args.shared:  # the R query heads of a KV head attend over one set of rows
        ab = dict(ab, gathered=ab["gathered"] // (Hq // Hkv))
        ab["total"] = ab["codes"] + ab["gathered"]
    alg_by_kernel = {"prep_kernel": (B * Hkv * (2 * D * 2 + D // 8)) if cfg.append else 0,
                     "score_kernel": ab["codes"], "select_kernel_unfused_only": 0,
                     "select_attend_kernel": ab["gathered"]}
    dom = max((1, 3), key=lambda i: kus[i])  # the two kernels that move the algorithmic bytes
    dom_name = KERNELS[dom]
    dom_bytes = alg_by_kernel[dom_name]
    achieved = dom_bytes / (kus[dom] * 1e-6) / 1e9

    step_us = sec_step * 1e6
    result = {
        "metric": "us per sparse decode step (and effective HBM GB/s)",
        "value": round(step_us, 3),
        "unit": "us/step",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(sec_step * 1e3, 6),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": cfg.name, "batch": B, "n_kv_heads": Hkv, "n_q_heads": Hq, "head_dim": D,
                   "context": L, "top_k": k, "kv_dtype": cfg.dtype, "kv_format": args.kv, "forced_tokens": args.forced, "group_shared": args.shared, "append": cfg.append,
                   "layers_rotated": n_layers, "launch": launch},
        "effective_hbm_GBps": round(ab["total"] / sec_step / 1e9, 1),
        "effective_hbm_frac_of_8TBps": round(ab["total"] / sec_step / 1e9 / HBM_PEAK_GBPS, 4),
        "algorithmic_bytes_per_step": ab["total"],
        "us_per_step_stream_launch": round(sec_stream * 1e6, 3),
        "us_per_step_hipgraph": None if sec_graph is None else round(sec_graph * 1e6, 3),
        "us_per_step_percentiles": dict(pct, groups=n_grp, steps_per_group=grp, launch="stream"),
        "gathered_rows": {"nominal": rows_nominal, "unique_per_kv_head": rows_unique},
        "kernel_us_hip_events": {KERNELS[i]: round(float(kus[i]), 3) for i in range(4)},
        "hip_event_pair_overhead_us": round(float(raw[4]), 3),
        "roofline": {"bound": "hbm", "kernel": dom_name, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "traffic": None if q2 else MEASURED_TRAFFIC_BYTES.get((args.config, dom_name)),
                     "algorithmic_bytes_per_launch": dom_bytes},
        "setup_seconds": round(gen_s, 1),
    }

    if not args.no_cpu_baseline and not args.forced and not args.shared:
        result["cpu_baseline"] = cpu_baseline(cfg, host0, args.cpu_seconds, q2)
    print(json.dumps(result))


def bench_fit(args, cfg, lay, ws, cap, q2):
    """Prefill-compress of one layer ("one-pass sign-based clustering": means, codes, codebook; plus the 2-bit
    records with --kv q2): two (q2: four) passes over K, one over V, all HBM-bound; rotates over enough layer
    copies of K (and V) to stay out of the Infinity Cache."""
    import torch

    import paper_2603_14224_amd as sik
    import sik_workloads as W
    from helpers import dev

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

    def fit(i):
        sik.sik_quantize_keys(lay, Ks[i % n_layers], sl, 0, 0, sik.SIK_Q_FIT, mu, cb, cnt, codes, ws)
        if q2:
            sik.sik_quantize_kv(lay, Ks[i % n_layers], Vs[i % n_layers], sl, 0, 0, sik.SIK_Q_FIT, mu, alpha, kvq)

    steps, warmup = min(args.steps, 50), min(args.warmup, 5)
    for i in range(warmup):
        fit(i)
    torch.cuda.synchronize()
    t = time.perf_counter()
    for i in range(steps):
        fit(warmup + i)
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t) / steps
    # K is read twice (means, then codes + clusters), with q2 twice more (alpha, records) and V once; codes and
    # records are written
    nbytes = kv_bytes * (5 if q2 else 2) + B * Hkv * L * (D // 8) + (B * Hkv * L * 128 if q2 else 0)
    print(json.dumps({
        "metric": "us per prefill-compress of one layer (quantiser FIT)", "value": round(sec * 1e6, 2),
        "unit": "us/layer", "n_gpus": 1, "steps": steps, "warmup": warmup, "ms_per_step": round(sec * 1e3, 5),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": cfg.name + " / prefill-compress", "batch": B, "n_kv_heads": Hkv, "head_dim": D,
                   "context": L, "kv_dtype": cfg.dtype, "kv_format": args.kv, "layers_rotated": n_layers},
        "roofline": {"bound": "hbm", "kernel": "colsum + encode" + (" + alpha + quantize_kv" if q2 else ""),
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
        if t_total >= budget_s or n >= 64:
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

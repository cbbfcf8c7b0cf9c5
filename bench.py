#!/usr/bin/env python3
"""Benchmark of the SpecPrefill token-importance hot path on one MI355X.

One "step" = sp_score + sp_pool_select + sp_gather over one synthetic prompt batch whose
queries and K cache are already resident in HBM.  The default workload is the 8B-draft /
32K-token scoring configuration (32 layers, 32 query / 8 KV heads, head dim 128, 8 look-ahead
queries, 2 GiB bf16 K cache).  Prints ONE JSON line.

  python bench.py --gpus 1 --steps 20 --warmup 5
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0   # MI355X published HBM3E peak


def measured_traffic(workload, general):
    """HBM bytes per sp_score launch as read from the FETCH_SIZE / WRITE_SIZE counter runs whose
    summaries sit under profiles/ (counters cannot be collected from inside this process)."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if general or not os.path.exists(path):
        return None
    with open(path) as f:
        table = json.load(f)
    entry = table.get(f"workload{workload}:stream_score_kernel") or table.get(f"workload{workload}:sp_score")
    return None if entry is None else entry["traffic_bytes_per_launch"]


def cpu_baseline(w, inp, layer_reduce, sample_layers):
    """Times the fp64 oracle, unchanged, on the same inputs (full prompt, all heads and queries)
    plus selection and gather on its scores.  sample_layers = 0: a two-layer pilot decides how
    many layers fit about 15 s (cost is linear in layers); when the whole depth fits, whole
    passes are repeated until about 10 s have been spent and their mean is reported."""
    import numpy as np
    from oracle import specprefill_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = os.cpu_count() or 1
    scale = 1.0 / math.sqrt(w.d)

    def score_pass(n_layers):
        t0 = time.perf_counter()
        scores, _ = orc.token_importance(inp["q"][:n_layers], inp["k"][:n_layers], inp["cu_seqlens"], scale,
                                         layer_reduce)
        return scores, time.perf_counter() - t0

    note = ""
    if sample_layers <= 0:
        pilot = min(2, w.L)
        _, t_pilot = score_pass(pilot)
        sample_layers = max(pilot, min(w.L, int(15.0 / max(t_pilot / pilot, 1e-6))))
        note = f" (after a {pilot}-layer pilot of {t_pilot:.2f} s)"
    sample_layers = min(sample_layers, w.L)
    passes, spent = 0, 0.0
    while True:
        scores, dt = score_pass(sample_layers)
        passes += 1
        spent += dt
        if sample_layers < w.L or spent >= 10.0 or passes >= 20:
            break
    t_score = spent / passes
    t1 = time.perf_counter()
    kept, cu_keep, _, _ = orc.pool_select(scores.astype(np.float32), inp["cu_seqlens"], w.chunk, w.pool_window,
                                          w.keep_rate)
    orc.gather(kept, cu_keep, inp["cu_seqlens"], inp["token_ids"])
    t_sel = time.perf_counter() - t1
    est_full = t_score * (w.L / sample_layers) + t_sel
    what = (f"all {w.L} layers, mean of {passes} whole passes of {t_score:.2f} s" if sample_layers == w.L else
            f"{sample_layers} of {w.L} layers in {t_score:.2f} s, scaled linearly in layers")
    return {
        "value": w.T / est_full, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
        "sample": f"{what}{note}; same inputs (full {w.T}-token prompt, all heads and queries); "
                  f"plus selection+gather {t_sel:.3f} s",
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", type=int, default=3, help="1..5, numbered as the benchmark configs")
    ap.add_argument("--layer-reduce", choices=["max", "mean"], default="max")
    ap.add_argument("--general", action="store_true", help="force the general two-pass scoring kernels")
    ap.add_argument("--cpu-sample-layers", type=int, default=0,
                    help="layers the oracle is timed on (0: as many as fit about 15 s, all of them if possible)")
    ap.add_argument("--skip-cpu", action="store_true")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MIB",
                    help="also launch a plain device copy of MIB MiB three times outside the timed region, so a "
                         "counter run of this command shows what FETCH_SIZE/WRITE_SIZE read for known traffic")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (no collectives are part of it); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2502_02789_amd import binding as sp, device as dev, synth

    sp.load_library()                       # fails loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    w = synth.workload(args.workload)
    mode = sp.SP_LAYER_MAX if args.layer_reduce == "max" else sp.SP_LAYER_MEAN

    t_gen = time.perf_counter()
    inp = synth.make_qk(w, threads=16)
    inp["token_ids"] = synth.make_token_ids(w)
    q = dev.bf16_from_bits(inp["q"])
    ks = [dev.bf16_from_bits(k) for k in inp["k"]]
    cu = torch.from_numpy(inp["cu_seqlens"]).cuda()
    ids = torch.from_numpy(inp["token_ids"]).cuda()
    embed = None
    if w.embed_dim:
        embed = dev.bf16_from_bits(synth.make_embedding(w.vocab, w.embed_dim, w.seed, threads=16))
    t_gen = time.perf_counter() - t_gen

    scorer = dev.Scorer(q, ks, cu, H_kv=w.H_kv, scale=1.0 / math.sqrt(w.d), layer_reduce=mode)
    cap = sp.sp_keep_upper_bound(list(w.seqlens), w.chunk, w.keep_rate)
    sel = dev.Selector(scorer.scores, cu, chunk=w.chunk, pool_window=w.pool_window, keep_rate=w.keep_rate,
                       capacity=cap)
    gat = dev.Gatherer(sel, token_ids=ids, embed=embed)
    stream = torch.cuda.current_stream()

    def step(ev=None):
        if ev is not None:
            ev[0].record(stream)
        scorer.run(stream, general=args.general)
        if ev is not None:
            ev[1].record(stream)
        sel.run(stream)
        gat.run(stream)
        if ev is not None:
            ev[2].record(stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.calibrate_copy:
        src = torch.empty(args.calibrate_copy << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(events[i])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed * 1e3 / args.steps
    score_ms = sorted(e[0].elapsed_time(e[1]) for e in events)
    tail_ms = sorted(e[1].elapsed_time(e[2]) for e in events)
    score_avg_ms = sum(score_ms) / len(score_ms)
    tail_avg_ms = sum(tail_ms) / len(tail_ms)

    k_bytes = w.k_bytes()
    algo_bytes = k_bytes + 4 * w.T                  # K cache read once + fp32 score per token written
    achieved = algo_bytes / (score_avg_ms * 1e-3) / 1e9
    n_keep = int(sel.cu_keep[-1])

    out = {
        "metric": "prompt tokens scored+selected/sec (sp_score + sp_pool_select + sp_gather)",
        "value": w.T / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 inputs, fp32 accumulate (selection in fp64)", "data": "synthetic",
        "config": {
            "workload": f"{w.name}: B={w.B} T={w.T} L={w.L} H={w.H} H_kv={w.H_kv} d={w.d} N={w.N} "
                        f"chunk={w.chunk} keep_rate={w.keep_rate} pool_window={w.pool_window}",
            "layer_reduce": args.layer_reduce, "k_cache_bytes": k_bytes, "kept_tokens": n_keep,
            "score_kernels": "general" if args.general else "auto",
        },
        "roofline": {
            "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBPS, "traffic": measured_traffic(args.workload, args.general),
            "kernel": "sp_score (all its launches)", "avg_ms": score_avg_ms, "median_ms": score_ms[len(score_ms) // 2],
            "algorithmic_bytes": algo_bytes,
        },
        "select_gather_ms": tail_avg_ms,
        "k_cache_gbps": k_bytes / (score_avg_ms * 1e-3) / 1e9,
        "input_generation_s": t_gen,
    }
    if not args.skip_cpu:
        out["cpu_baseline"] = cpu_baseline(w, inp, 0 if args.layer_reduce == "max" else 1,
                                           args.cpu_sample_layers)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()

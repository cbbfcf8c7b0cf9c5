#!/usr/bin/env python3
"""Benchmark of the SpecPrefill token-importance hot path on one MI355X.

One "step" = sp_score + sp_pool_select + sp_gather over one synthetic prompt batch whose
queries and K cache are already resident in HBM.  The default workload is the 8B-draft /
32K-token scoring configuration (32 layers, 32 query / 8 KV heads, head dim 128, 8 look-ahead
queries, 2 GiB bf16 K cache).  Prints ONE JSON line.  After the timed loop the run checks what
it timed: sp_score_check, the scores against the fp64 oracle (the cpu_baseline leg computes them
anyway) and the keep set against the oracle's; a miss makes the process exit non-zero.

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
SCORE_RTOL = 2e-3        # score tolerance against the fp64 oracle (the same as the parity tests)


def measured_traffic(workload, general, layer_reduce):
    """HBM bytes per sp_score launch as read from the FETCH_SIZE / WRITE_SIZE counter runs whose
    summaries sit under profiles/ (counters cannot be collected from inside this process)."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if general or layer_reduce != "max" or not os.path.exists(path):
        return None
    with open(path) as f:
        table = json.load(f)
    entry = table.get(f"workload{workload}:sp_score")
    return None if entry is None else entry["traffic_bytes_per_launch"]


def cpu_baseline(w, inp, layer_reduce, sample_layers):
    """Times the fp64 oracle, unchanged, on the same inputs (full prompt, all heads and queries)
    plus selection and gather on its scores.  sample_layers = 0: a two-layer pilot decides how
    many layers fit about 15 s (cost is linear in layers); when the whole depth fits, whole
    passes are repeated until about 10 s have been spent and their mean is reported.
    Returns (json object, oracle scores or None if only a layer subset was run)."""
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
    out = {
        "value": w.T / est_full, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
        "sample": f"{what}{note}; same inputs (full {w.T}-token prompt, all heads and queries); "
                  f"plus selection+gather {t_sel:.3f} s",
    }
    return out, (scores if sample_layers == w.L else None)


def check_against(w, inp, gpu_scores, gpu_kept, gpu_cu_keep, ref_scores, ref_name):
    """Scores element by element (tolerance of the parity tests), then the keep set: selection by the
    oracle on the reference scores against what the GPU kept; chunks may differ only if their
    reference chunk score lies within the score tolerance of the k-th."""
    import numpy as np
    from oracle import specprefill_oracle as orc
    ref = np.asarray(ref_scores, dtype=np.float64)
    got = np.asarray(gpu_scores, dtype=np.float64)
    finite = bool(np.isfinite(got).all())
    err = np.abs(got - ref) / np.maximum(np.abs(ref), 1e-300)
    scores_ok = finite and bool((np.abs(got - ref) <= SCORE_RTOL * np.abs(ref) + 1e-30).all())
    kept_o, cu_keep_o, cs, cu_chunks = orc.pool_select(ref.astype(np.float32), inp["cu_seqlens"], w.chunk,
                                                       w.pool_window, w.keep_rate)
    cu = inp["cu_seqlens"]
    equal, swapped, keep_ok = True, 0, True
    for b in range(w.B):
        g = gpu_kept[int(gpu_cu_keep[b]):int(gpu_cu_keep[b + 1])].astype(np.int64)
        o = kept_o[int(cu_keep_o[b]):int(cu_keep_o[b + 1])]
        if len(g) == len(o) and (g == o).all():
            continue
        equal = False
        seg = cs[cu_chunks[b]:cu_chunks[b + 1]]
        k = orc.keep_count(len(seg), w.keep_rate)
        kth = np.sort(seg)[::-1][k - 1]
        gc = set(((g - int(cu[b])) // w.chunk).tolist())
        oc = set(((o - int(cu[b])) // w.chunk).tolist())
        if len(gc) != len(oc):
            keep_ok = False
        for j in gc ^ oc:
            swapped += 1
            if abs(seg[j] - kth) > SCORE_RTOL * abs(kth):
                keep_ok = False
    return {
        "checked_against": ref_name, "score_max_rel_err": float(err.max()) if finite else None,
        "scores_within_tolerance": scores_ok, "keep_set_equal": equal, "swapped_chunks": swapped,
        "ok": bool(scores_ok and keep_ok),
    }


class Problem:
    """One workload resident on the GPU with the three calls' argument structs."""

    def __init__(self, number, layer_reduce, threads=16):
        import torch
        from paper_2502_02789_amd import binding as sp, device as dev, synth
        self.w = w = synth.workload(number)
        self.mode_name = layer_reduce
        mode = sp.SP_LAYER_MAX if layer_reduce == "max" else sp.SP_LAYER_MEAN
        t0 = time.perf_counter()
        self.inp = inp = synth.make_qk(w, threads=threads)
        inp["token_ids"] = synth.make_token_ids(w)
        q = dev.bf16_from_bits(inp["q"])
        ks = [dev.bf16_from_bits(k) for k in inp["k"]]
        cu = torch.from_numpy(inp["cu_seqlens"]).cuda()
        ids = torch.from_numpy(inp["token_ids"]).cuda()
        embed = None
        if w.embed_dim:
            embed = dev.bf16_from_bits(synth.make_embedding(w.vocab, w.embed_dim, w.seed, threads=threads))
        self.t_gen = time.perf_counter() - t0
        # the benchmark box runs nothing else on its GPU: the single-pass kernels may be used; the
        # workspace is this object's alone, as a serving loop's would be, so from the second call on
        # sp_score is told that it still holds what the call before left (SP_SCORE_WORKSPACE_KEPT)
        # a batch comes with the length of its longest prompt, as a serving engine knows it (max_seqlen)
        self.scorer = dev.Scorer(q, ks, cu, H_kv=w.H_kv, scale=1.0 / math.sqrt(w.d), layer_reduce=mode,
                                 exclusive_device=True, keep_workspace=True,
                                 max_seqlen=max(w.seqlens) if w.B > 1 else 0)
        cap = sp.sp_keep_upper_bound(list(w.seqlens), w.chunk, w.keep_rate)
        self.sel = dev.Selector(self.scorer.scores, cu, chunk=w.chunk, pool_window=w.pool_window,
                                keep_rate=w.keep_rate, capacity=cap)
        self.gat = dev.Gatherer(self.sel, token_ids=ids, embed=embed)
        self.stream = torch.cuda.current_stream()

    def step(self, ev=None, general=False):
        s = self.stream
        if ev is not None:
            ev[0].record(s)
        self.scorer.run(s, general=general)
        if ev is not None:
            ev[1].record(s)
        self.sel.run(s)
        if ev is not None:
            ev[2].record(s)
        self.gat.run(s)
        if ev is not None:
            ev[3].record(s)

    def timed(self, steps, warmup, general=False):
        """-> (wall ms per step, sorted sp_score ms, sorted select ms, sorted gather ms)"""
        import torch
        for _ in range(warmup):
            self.step(general=general)
        torch.cuda.synchronize()
        events = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(steps)]
        t0 = time.perf_counter()
        for i in range(steps):
            self.step(events[i], general=general)
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3 / steps
        return (wall_ms, sorted(e[0].elapsed_time(e[1]) for e in events),
                sorted(e[1].elapsed_time(e[2]) for e in events), sorted(e[2].elapsed_time(e[3]) for e in events))

    def gather_bytes(self):
        """Algorithmic bytes of sp_gather: per kept token its row read and written, ids and positions."""
        n_keep = int(self.sel.cu_keep[-1])
        row = 2 * self.w.embed_dim * 2 if self.w.embed_dim else 0
        return n_keep * (row + 4 * 4)


def side_measurement(number, layer_reduce, steps, warmup, raw_cache_too=False, fp8_too=False):
    """GPU-only timing of another workload / layer reduction (no oracle leg), cross-checked
    against the library's plain two-pass kernels on the same inputs.  raw_cache_too: the same
    buffers once more taken as an UN-rotated cache that sp_score rotates itself (rope_theta > 0),
    cross-checked the same way.  fp8_too: the same keys as an 8-bit cache."""
    import numpy as np
    import torch
    from paper_2502_02789_amd import binding as sp
    pr = Problem(number, layer_reduce)
    w = pr.w
    _, score_ms, sel_ms, gat_ms = pr.timed(steps, warmup)
    pr.scorer.check()
    fast = pr.scorer.scores.cpu().numpy().astype(np.float64)
    pr.scorer.run(pr.stream, general=True)
    torch.cuda.synchronize()
    plain = pr.scorer.scores.cpu().numpy().astype(np.float64)
    rel = float((np.abs(fast - plain) / np.maximum(np.abs(plain), 1e-300)).max())
    avg = sum(score_ms) / len(score_ms)
    algo = w.k_bytes() + 4 * w.T
    g_avg = sum(gat_ms) / len(gat_ms)
    out = {
        "workload": f"{w.name}: B={w.B} T={w.T} L={w.L} H={w.H} H_kv={w.H_kv} d={w.d} N={w.N}",
        "layer_reduce": layer_reduce, "sp_score_us": avg * 1e3, "sp_score_gbps": algo / (avg * 1e-3) / 1e9,
        "frac_of_hbm_peak": algo / (avg * 1e-3) / 1e9 / HBM_PEAK_GBPS,
        "sp_pool_select_us": sum(sel_ms) / len(sel_ms) * 1e3, "sp_gather_us": g_avg * 1e3,
        "sp_gather_gbps": pr.gather_bytes() / (g_avg * 1e-3) / 1e9,
        "max_rel_diff_vs_plain_kernels": rel, "ok": bool(rel <= 2 * SCORE_RTOL),
    }
    if w.B > 1:
        # the same batch without the promise of a longest prompt: the kernels that keep logits between two passes
        from paper_2502_02789_amd import device as dev
        mode = sp.SP_LAYER_MAX if layer_reduce == "max" else sp.SP_LAYER_MEAN
        two = dev.Scorer(pr.scorer.q, pr.scorer.k_layers, pr.scorer.cu, H_kv=w.H_kv, scale=1.0 / math.sqrt(w.d),
                         layer_reduce=mode, exclusive_device=True)
        ms = []
        for i in range(warmup + steps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(pr.stream)
            two.run(pr.stream)
            b.record(pr.stream)
            if i >= warmup:
                ms.append((a, b))
        torch.cuda.synchronize()
        out["max_seqlen"] = max(w.seqlens)
        out["sp_score_us_without_max_seqlen"] = sum(a.elapsed_time(b) for a, b in ms) / len(ms) * 1e3
        rel2 = float((np.abs(two.scores.cpu().numpy().astype(np.float64) - plain) / np.maximum(np.abs(plain), 1e-300)).max())
        out["ok"] = bool(out["ok"] and rel2 <= 2 * SCORE_RTOL)
        del two
        torch.cuda.empty_cache()
    if fp8_too:
        # the same keys once more as an 8-bit cache (OCP E4M3 codes, one scale per layer and KV head; quantised
        # here with torch, which is input preparation), cross-checked against the plain kernels on the same codes
        from paper_2502_02789_amd import device as dev
        mode = sp.SP_LAYER_MAX if layer_reduce == "max" else sp.SP_LAYER_MEAN
        codes, scales = [], []
        for k in pr.scorer.k_layers:
            amax = k.abs().amax(dim=(0, 2)).float()
            sc = torch.where(amax > 0, amax / 448.0, torch.ones_like(amax))
            codes.append((k.float() / sc[None, :, None]).to(torch.float8_e4m3fn).view(torch.uint8))
            scales.append(sc)
        k_scale = torch.stack(scales).contiguous()
        f8 = dev.Scorer(pr.scorer.q, codes, pr.scorer.cu, H_kv=w.H_kv, scale=1.0 / math.sqrt(w.d), layer_reduce=mode,
                        exclusive_device=True, max_seqlen=max(w.seqlens) if w.B > 1 else 0, k_scale=k_scale)
        ms = []
        for i in range(warmup + steps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(pr.stream)
            f8.run(pr.stream)
            b.record(pr.stream)
            if i >= warmup:
                ms.append((a, b))
        torch.cuda.synchronize()
        t8 = sum(a.elapsed_time(b) for a, b in ms) / len(ms)
        fast8 = f8.scores.cpu().numpy().astype(np.float64)
        f8.run(pr.stream, general=True)
        torch.cuda.synchronize()
        plain8 = f8.scores.cpu().numpy().astype(np.float64)
        rel8 = float((np.abs(fast8 - plain8) / np.maximum(np.abs(plain8), 1e-300)).max())
        algo8 = w.k_bytes() // 2 + 4 * w.T
        out["fp8_cache_sp_score_us"] = t8 * 1e3
        out["fp8_cache_gbps"] = algo8 / (t8 * 1e-3) / 1e9
        out["fp8_cache_frac_of_hbm_peak"] = algo8 / (t8 * 1e-3) / 1e9 / HBM_PEAK_GBPS
        out["fp8_cache_max_rel_diff_vs_plain_kernels"] = rel8
        out["ok"] = bool(out["ok"] and rel8 <= 2 * SCORE_RTOL)
        del f8, codes
        torch.cuda.empty_cache()
    if raw_cache_too:
        from paper_2502_02789_amd import device as dev
        old = pr.scorer
        q_pos = torch.tensor([[m + n for n in range(w.N)] for m in w.seqlens], dtype=torch.int32, device="cuda")
        mode = sp.SP_LAYER_MAX if layer_reduce == "max" else sp.SP_LAYER_MEAN
        pr.scorer = None
        del old.workspace
        raw = dev.Scorer(old.q, old.k_layers, old.cu, H_kv=w.H_kv, scale=1.0 / math.sqrt(w.d), layer_reduce=mode,
                         rope_theta=5e5, q_pos=q_pos, exclusive_device=True)
        ms = []
        for i in range(warmup + steps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record(pr.stream)
            raw.run(pr.stream)
            b.record(pr.stream)
            if i >= warmup:
                ms.append((a, b))
        torch.cuda.synchronize()
        ms = [a.elapsed_time(b) for a, b in ms]
        fast = raw.scores.cpu().numpy().astype(np.float64)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record(pr.stream)
        raw.run(pr.stream, general=True)
        b.record(pr.stream)
        torch.cuda.synchronize()
        out["raw_cache_plain_kernels_us"] = a.elapsed_time(b) * 1e3
        plain = raw.scores.cpu().numpy().astype(np.float64)
        rel = float((np.abs(fast - plain) / np.maximum(np.abs(plain), 1e-300)).max())
        out["raw_cache_rotated_by_sp_score_us"] = sum(ms) / len(ms) * 1e3
        out["raw_cache_max_rel_diff_vs_plain_kernels"] = rel
        out["ok"] = bool(out["ok"] and rel <= 2 * SCORE_RTOL)
        del raw
    del pr
    torch.cuda.empty_cache()
    return out


def short_prompt_measurement(steps, warmup):
    """Workload 1 (one 1024-token prompt, no look-ahead): the separate calls against the single
    fused launch (sp_score_pool_select), GPU time per step from HIP events."""
    import numpy as np
    import torch
    from paper_2502_02789_amd import device as dev
    pr = Problem(1, "max")
    stream = pr.stream

    def timed(fn):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        for a, b in ev:
            a.record(stream)
            fn()
            b.record(stream)
        torch.cuda.synchronize()
        ms = sorted(a.elapsed_time(b) for a, b in ev)
        return ms[len(ms) // 2] * 1e3

    def separate():
        pr.scorer.run(stream)
        pr.sel.run(stream)

    t_sep = timed(separate)
    kept_sep = pr.sel.kept_idx.clone()
    scores_sep = pr.scorer.scores.clone()
    t_fused = timed(lambda: dev.score_pool_select(pr.scorer, pr.sel, stream))
    same_keep = bool((kept_sep == pr.sel.kept_idx).all())
    rel = float(((scores_sep - pr.scorer.scores).abs() / scores_sep.abs()).max())
    w = pr.w
    return {
        "workload": f"{w.name}: B={w.B} T={w.T} L={w.L} H={w.H} H_kv={w.H_kv} d={w.d} N={w.N}",
        "sp_score_plus_sp_pool_select_us": t_sep, "sp_score_pool_select_us": t_fused,
        "same_keep_set": same_keep, "max_rel_diff_of_scores": rel, "ok": bool(same_keep and rel <= 2 * SCORE_RTOL),
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=100,
                    help="untimed steps first; the first few dozen calls after start-up run up to 20 %% slower (clocks and caches settling)")
    ap.add_argument("--workload", type=int, default=3, help="1..5, numbered as the benchmark configs")
    ap.add_argument("--layer-reduce", choices=["max", "mean"], default="max")
    ap.add_argument("--general", action="store_true", help="force the general two-pass scoring kernels")
    ap.add_argument("--cpu-sample-layers", type=int, default=0,
                    help="layers the oracle is timed on (0: as many as fit about 15 s, all of them if possible)")
    ap.add_argument("--skip-cpu", action="store_true")
    ap.add_argument("--only-also", type=int, default=0, metavar="N",
                    help="print only the side measurement of workload N (with its 8-bit and raw-cache variants) and exit")
    ap.add_argument("--no-also", action="store_true",
                    help="skip the GPU-only side measurements of the other workloads and of the layer-mean mode")
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
    from paper_2502_02789_amd import binding as sp

    sp.load_library()                       # fails loudly if the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    if args.only_also:
        print(json.dumps(side_measurement(args.only_also, args.layer_reduce, steps=args.steps, warmup=args.warmup,
                                          raw_cache_too=(args.only_also == 4), fp8_too=True)), flush=True)
        return
    pr = Problem(args.workload, args.layer_reduce)
    w = pr.w
    if args.calibrate_copy:
        pr.step(general=args.general)
        torch.cuda.synchronize()
        src = torch.empty(args.calibrate_copy << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    ms_per_step, score_ms, sel_ms, gat_ms = pr.timed(args.steps, args.warmup, general=args.general)
    score_avg_ms = sum(score_ms) / len(score_ms)
    gat_avg_ms = sum(gat_ms) / len(gat_ms)
    sel_avg_ms = sum(sel_ms) / len(sel_ms)

    # what was timed is what gets checked: the outputs of the last timed step
    timeout_status = "ok"
    try:
        pr.scorer.check()
    except sp.SpError as e:
        timeout_status = str(e)
    gpu_scores = pr.scorer.scores.cpu().numpy()
    gpu_kept = pr.sel.kept_idx.cpu().numpy()
    gpu_cu_keep = pr.sel.cu_keep.cpu().numpy()
    # the same steps on a workspace that is taken as new by every call (the flag never set)
    pr.scorer._keep = False
    fresh_score_ms = pr.timed(max(10, args.steps // 2), 5, general=args.general)[1]
    pr.scorer._keep = True
    fresh_matches = bool((pr.scorer.scores.cpu().numpy() == gpu_scores).all() or args.general)

    k_bytes = w.k_bytes()
    algo_bytes = k_bytes + 4 * w.T                  # K cache read once + fp32 score per token written
    achieved = algo_bytes / (score_avg_ms * 1e-3) / 1e9
    n_keep = int(gpu_cu_keep[-1])

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
            "flags": "SP_SCORE_EXCLUSIVE_DEVICE | SP_SCORE_WORKSPACE_KEPT (from the second call on)",
        },
        "roofline": {
            "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBPS,
            "traffic": measured_traffic(args.workload, args.general, args.layer_reduce),
            "kernel": "sp_score (all its launches)", "avg_ms": score_avg_ms, "median_ms": score_ms[len(score_ms) // 2],
            "algorithmic_bytes": algo_bytes,
            "avg_ms_without_workspace_kept": sum(fresh_score_ms) / len(fresh_score_ms),
            "same_scores_without_workspace_kept": fresh_matches,
        },
        "select_gather_ms": sel_avg_ms + gat_avg_ms,
        "sp_pool_select_us": sel_avg_ms * 1e3, "sp_gather_us": gat_avg_ms * 1e3,
        "sp_gather_gbps": pr.gather_bytes() / (gat_avg_ms * 1e-3) / 1e9,
        "k_cache_gbps": k_bytes / (score_avg_ms * 1e-3) / 1e9,
        "input_generation_s": pr.t_gen,
    }
    # what plain reading of the same K cache achieves here and now (read-only probe kernels)
    from paper_2502_02789_amd import probe
    out["roofline"].update(probe.stream_ceiling(pr.scorer.k_layers))
    out["roofline"]["frac_of_stream_ceiling"] = achieved / out["roofline"]["stream_ceiling_gbps"]

    ok = timeout_status == "ok" and fresh_matches
    oracle_scores = None
    if not args.skip_cpu:
        out["cpu_baseline"], oracle_scores = cpu_baseline(w, pr.inp, 0 if args.layer_reduce == "max" else 1,
                                                           args.cpu_sample_layers)
    if oracle_scores is not None:
        parity = check_against(w, pr.inp, gpu_scores, gpu_kept, gpu_cu_keep, oracle_scores, "fp64 oracle, same inputs")
    else:
        # the oracle did not run the whole depth: the library's plain two-pass kernels (pinned to the
        # oracle by the parity tests) stand in, on the same device buffers
        pr.scorer.run(pr.stream, general=True)
        torch.cuda.synchronize()
        parity = check_against(w, pr.inp, gpu_scores, gpu_kept, gpu_cu_keep, pr.scorer.scores.cpu().numpy(),
                               "plain two-pass kernels of the library, same inputs")
    parity["sp_score_check"] = timeout_status
    out["parity"] = parity
    ok = ok and parity["ok"]

    if not args.no_also and args.workload == 3 and not args.general:
        del pr
        torch.cuda.empty_cache()
        also = []
        other = "mean" if args.layer_reduce == "max" else "max"
        # (workload, layer reduction, also as an 8-bit cache); the last entry is the headline workload again, for
        # its 8-bit figures
        for number, mode, fp8 in ((3, other, False), (2, "max", False), (5, "max", True), (4, "max", True), (4, other, False),
                                  (3, args.layer_reduce, True)):
            m = side_measurement(number, mode, steps=20, warmup=40 if number != 4 else 10,
                                 raw_cache_too=(number == 4 and fp8), fp8_too=fp8)
            if number == args.workload and mode == args.layer_reduce:
                # the headline workload again, for its 8-bit figures only (its bf16 figures are the line's own)
                m = {k: v for k, v in m.items() if k in ("workload", "layer_reduce", "ok") or k.startswith("fp8_")}
            also.append(m)
            ok = ok and also[-1]["ok"]
        also.append(short_prompt_measurement(steps=50, warmup=20))
        ok = ok and also[-1]["ok"]
        out["also"] = also
    print(json.dumps(out), flush=True)
    if not ok:
        print("bench.py: the timed run FAILED its own check (see \"parity\" / \"also\")", file=sys.stderr)
        sys.exit(1)


if __name__ == "__main__":
    main()

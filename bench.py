#!/usr/bin/env python3
"""Benchmark of the compress-as-you-prefill hot path on one MI355X.

A "step" is one whole prefill of the workload: every block of the prefix
through every layer, each as kvp_prefill_chunk (attention + scoring) followed
by kvp_compact (select + merge + move), with Q, K, V of all layers already
resident in HBM.  The metric is prefill tokens/s at the fixed KV budget.

Prints ONE JSON line.  `roofline` is for the attention kernel (the dominant
one): algorithmic flops 4 d Hq (n c + n (n + 1) / 2) per launch over its HIP
event time on the launching stream.  `rooflines` has an entry for every kernel
of the path (scoring against its own MFMA flops; select, merge, move and the
decode step against HBM, with the bytes taken from what this run's compactions
actually did).  `attainable` holds what this GPU reaches on a register-resident
bf16 MFMA loop and on a plain device copy, measured in the same run, and every
roofline entry also gives its fraction of those.  `cpu_baseline` is the NumPy
oracle timed on this machine's host cores on a bounded sample of the same workload.
"""
import argparse
import json
import os
import statistics
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA, vendor figure
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E, vendor figure
# HBM bytes per attention launch (fetch + write) at the long_video steady state, from the
# rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs summarised in profiles/ (launch-weighted mean,
# counters scaled by what they read for a plain 256 MiB copy); None for a workload not measured
ATTENTION_TRAFFIC_BYTES = {"long_video": 52326293}


def attention_flops(wl, t0_n_pairs):
    """Algorithmic flops of the attention launches of one layer over the given blocks."""
    total = 0
    c = 0
    per = []
    for _, n in t0_n_pairs:
        f = 4 * wl.head_dim * wl.n_q_heads * (n * c + n * (n + 1) // 2)
        per.append(f)
        total += f
        c = min(wl.budget, c + n)
    return total, per


def generate(wl, device, threads):
    import torch
    from kvp_workload import layer_inputs, bits_to_torch

    def one(layer):
        return layer_inputs(wl, layer)

    out = []
    with ThreadPoolExecutor(max_workers=threads) as ex:
        for qb, kb, vb in ex.map(one, range(wl.n_layers)):
            out.append(tuple(bits_to_torch(x, device) for x in (qb, kb, vb)))
    torch.cuda.synchronize()
    return out


def run_steps(driver, cache, wl, data, ranges, steps, outs, obs=None, keydiff=False, events=None):
    """`steps` whole prefills: every block through every layer, in the order `driver` gives
    (compactions in line, or on a second stream beside the following layers' attention).
    `obs`: per-layer proxy queries that score the candidates instead of the block's own;
    `keydiff`: the keys alone score them.  `events`: a list that receives one (start, end) pair
    of HIP events per step, recorded on the main stream (the end after the side stream has been
    joined), for the per-step median."""
    import torch
    for _ in range(steps):
        if events is not None:
            start = torch.cuda.Event(enable_timing=True)
            start.record()
        for layer in range(wl.n_layers):
            cache.set_state(layer, 0, 0)
        for t0, n in ranges:
            driver.block(t0, lambda l: tuple(x[t0:t0 + n] for x in data[l]), lambda l: outs[l][:n],
                         (lambda l: obs[l]) if obs is not None else None, keydiff)
        if events is not None:
            driver.finish()
            end = torch.cuda.Event(enable_timing=True)
            end.record()
            events.append((start, end))
    driver.finish()


def attainable_peaks(device):
    """What this GPU reaches on (a) dense 32x32x16 bf16 MFMAs on register operands, eight waves on
    every CU, no memory traffic, and (b) a plain 256 MiB device copy (bytes read + bytes written).
    Medians of five launches each, timed with HIP events on the launching stream."""
    import torch
    import paper_2604_16734_amd as K
    stream = torch.cuda.current_stream(device).cuda_stream
    cus = torch.cuda.get_device_properties(device).multi_processor_count
    sink = torch.empty(cus * 512, dtype=torch.float32, device=device)

    def timed(fn, reps=5):
        fn()
        torch.cuda.synchronize()
        out = []
        for _ in range(reps):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            fn()
            b.record()
            b.synchronize()
            out.append(a.elapsed_time(b) * 1e-3)
        return statistics.median(out)

    flops = [0.0]

    def mfma():
        rc, flops[0] = K.kvp_probe_mfma(sink.data_ptr(), sink.numel() * 4, cus, 12000, stream)
        if rc:
            raise K.KvpError(rc, "kvp_probe_mfma")
    t_mfma = timed(mfma)
    nbytes = 256 << 20
    src = torch.empty(nbytes, dtype=torch.uint8, device=device).fill_(3)
    dst = torch.empty_like(src)
    best = 0.0
    for wgs in (cus * 4, cus * 8, cus * 16, cus * 32):
        def copy():
            rc = K.kvp_probe_copy(dst.data_ptr(), src.data_ptr(), nbytes, wgs, stream)
            if rc:
                raise K.KvpError(rc, "kvp_probe_copy")
        best = max(best, 2 * nbytes / timed(copy))
    assert bool((dst == 3).all())
    del src, dst
    return {"mfma_bf16_tflops": round(flops[0] / t_mfma / 1e12, 1), "hbm_copy_GBps": round(best / 1e9, 1),
            "compute_units": cus,
            "how": "kvp_probe_mfma: %d workgroups x 8 waves x 192000 MFMAs 32x32x16 bf16 on registers; "
                   "kvp_probe_copy: 256 MiB, read + written bytes, best of four grid sizes; medians of 5" % cus}


def bench_workload(wl, steps, warmup, device, threads, profile=True, streams=1, n_obs=0, scratch_sets=16, variants=True,
                   eq1_alone=True, score_sweep=1):
    import torch
    import paper_2604_16734_amd as K
    from kvp_workload import chunk_ranges

    data = generate(wl, device, threads)
    ranges = chunk_ranges(wl.n_tokens, wl.chunk)
    two = streams == 2 and wl.n_layers >= 4
    scratch_sets = max(2 if two else 1, min(scratch_sets, wl.n_layers))
    cache = K.Cache(wl.n_layers, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.budget, wl.chunk,
                    wl.segments, merge=True, scratch_sets=scratch_sets, device=device)
    cache.set_score_sweep(score_sweep)
    driver = K.Prefill(cache, wl.n_layers, overlap=two)
    outs = [torch.empty((wl.chunk, wl.n_q_heads, wl.head_dim), dtype=torch.bfloat16, device=device)
            for _ in range(wl.n_layers)]
    run_steps(driver, cache, wl, data, ranges, warmup, outs)
    torch.cuda.synchronize()
    step_events = []
    t_begin = time.perf_counter()
    run_steps(driver, cache, wl, data, ranges, steps, outs, events=step_events)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_begin
    ms_per_step = 1e3 * elapsed / steps
    ms_median = statistics.median(a.elapsed_time(b) for a, b in step_events)
    proxy = None
    if n_obs and variants:
        # the paper's literal scoring (Sec. 3.2): n_obs proxy queries per layer, the same for every block
        gen = torch.Generator(device=device).manual_seed(1234)
        obs = [torch.randn((n_obs, wl.n_q_heads, wl.head_dim), generator=gen, device=device).to(torch.bfloat16)
               for _ in range(wl.n_layers)]
        run_steps(driver, cache, wl, data, ranges, 1, outs, obs)
        torch.cuda.synchronize()
        t_proxy = time.perf_counter()
        run_steps(driver, cache, wl, data, ranges, steps, outs, obs)
        torch.cuda.synchronize()
        t_proxy = (time.perf_counter() - t_proxy) / steps
        proxy = {"n_obs": n_obs, "tokens_per_s": round(wl.n_tokens / t_proxy, 1), "ms_per_step": round(1e3 * t_proxy, 4)}
    keydiff = None
    if variants:
        run_steps(driver, cache, wl, data, ranges, 1, outs, keydiff=True)
        torch.cuda.synchronize()
        t_kd = time.perf_counter()
        run_steps(driver, cache, wl, data, ranges, steps, outs, keydiff=True)
        torch.cuda.synchronize()
        t_kd = (time.perf_counter() - t_kd) / steps
        keydiff = {"tokens_per_s": round(wl.n_tokens / t_kd, 1), "ms_per_step": round(1e3 * t_kd, 4)}
    layerwise = None
    if variants:
        # the order of calls a model has: one attention call per layer as the block moves up the
        # stack, one kvp_compact_layers per block (runtime.LayerwisePrefill)
        lcache = K.Cache(wl.n_layers, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.budget, wl.chunk,
                         wl.segments, merge=True, scratch_sets=wl.n_layers, device=device)
        ldriver = K.LayerwisePrefill(lcache, wl.n_layers)

        def layerwise_steps(count):
            for _ in range(count):
                for layer in range(wl.n_layers):
                    lcache.set_state(layer, 0, 0)
                for t0, n in ranges:
                    for layer in range(wl.n_layers):
                        q, k, v = (x[t0:t0 + n] for x in data[layer])
                        ldriver.layer(layer, t0, q, k, v, out=outs[layer][:n])
                    ldriver.end_block()
        layerwise_steps(1)
        torch.cuda.synchronize()
        t_lw = time.perf_counter()
        layerwise_steps(steps)
        torch.cuda.synchronize()
        t_lw = (time.perf_counter() - t_lw) / steps
        layerwise = {"tokens_per_s": round(wl.n_tokens / t_lw, 1), "ms_per_step": round(1e3 * t_lw, 4),
                     "scratch_sets": wl.n_layers}
        lcache.close()
    bulk = None
    if variants and wl.budget > wl.chunk and wl.budget + wl.budget <= 8192 and wl.n_tokens > wl.budget:
        # hybrid execution (Sec. 4.3): the first `budget` tokens in one causal pass, then blocks
        bcache = K.Cache(wl.n_layers, wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.budget, wl.budget,
                         wl.segments, merge=True, scratch_sets=scratch_sets, device=device)
        bdriver = K.Prefill(bcache, wl.n_layers, overlap=two)
        branges = [(0, wl.budget)] + [(wl.budget + t0, n) for t0, n in chunk_ranges(wl.n_tokens - wl.budget, wl.chunk)]
        bouts = [torch.empty((wl.budget, wl.n_q_heads, wl.head_dim), dtype=torch.bfloat16, device=device)
                 for _ in range(wl.n_layers)]
        run_steps(bdriver, bcache, wl, data, branges, 1, bouts)
        torch.cuda.synchronize()
        t_bulk = time.perf_counter()
        run_steps(bdriver, bcache, wl, data, branges, steps, bouts)
        torch.cuda.synchronize()
        t_bulk = (time.perf_counter() - t_bulk) / steps
        bulk = {"first_block": wl.budget, "tokens_per_s": round(wl.n_tokens / t_bulk, 1), "ms_per_step": round(1e3 * t_bulk, 4)}
        bcache.close()
        del bouts
    decode = None
    if variants:
        # generation over the compressed caches (Eq. 1 with one query row): the attention of one new
        # token in every layer, its own key and value being the whole tail
        run_steps(driver, cache, wl, data, ranges, 1, outs)
        torch.cuda.synchronize()
        dq = [x[0][0].contiguous() for x in data]
        dk = [x[1][:1].contiguous() for x in data]
        dv = [x[2][:1].contiguous() for x in data]
        dout = torch.empty_like(dq[0])
        ptrs = [(dq[l].data_ptr(), dk[l].data_ptr(), dv[l].data_ptr()) for l in range(wl.n_layers)]
        stream = torch.cuda.current_stream(device).cuda_stream

        def decode_tokens(count):
            for _ in range(count):
                for l, (pq, pk, pv) in enumerate(ptrs):
                    rc = K.kvp_decode_step(cache.handle, l, pq, pk, pv, 1, dout.data_ptr(), stream)
                    if rc:
                        raise K.KvpError(rc, "kvp_decode_step")
        decode_tokens(2)
        torch.cuda.synchronize()
        n_dec = 20
        t_dec = time.perf_counter()
        decode_tokens(n_dec)
        torch.cuda.synchronize()
        t_dec = (time.perf_counter() - t_dec) / n_dec
        cache.profile_enable(True)
        decode_tokens(2)
        torch.cuda.synchronize()
        dec_launches, dec_ms, _ = cache.profile_read()["decode"]
        cache.profile_enable(False)
        kept = min(wl.budget, wl.n_tokens)
        dec_bytes = 2 * wl.n_kv_heads * (kept + 1) * wl.head_dim * 2      # K and V rows of one layer, read once
        decode = {"us_per_token_all_layers": round(1e6 * t_dec, 2), "us_per_layer_on_device": round(1e3 * dec_ms / dec_launches, 3),
                  "bytes_per_layer": dec_bytes, "GBps_on_device": round(dec_bytes / (1e-3 * dec_ms / dec_launches) / 1e9, 1),
                  "keys": kept + 1}
    res = {
        "decode_step": decode,
        "bulk_first_pass": bulk,
        "layerwise_order": layerwise,
        "keydiff_scoring": keydiff,
        "proxy_scoring": proxy,
        "tokens_per_s": wl.n_tokens / (elapsed / steps),
        "ms_per_step": ms_per_step,
        "ms_per_step_median_hip_events": ms_median,
        "persistent_kv_bytes": cache.persistent_bytes,
        "scratch_bytes": cache.nbytes - cache.persistent_bytes,
        "chunk_kv_bytes": 2 * wl.chunk * wl.n_kv_heads * wl.head_dim * 2,
        "full_cache_kv_bytes": 2 * wl.n_layers * wl.n_kv_heads * wl.head_dim * 2 * wl.n_tokens,
    }
    if profile:
        prof_steps = 1
        totals_before = cache.totals()
        cache.profile_enable(True)
        torch.cuda.synchronize()
        t_begin = time.perf_counter()
        # per-kernel times are taken with everything in line on one stream: beside another
        # kernel a launch takes longer than it needs
        run_steps(K.Prefill(cache, wl.n_layers, overlap=False), cache, wl, data, ranges, prof_steps, outs)
        torch.cuda.synchronize()
        res["profiled_ms_per_step"] = 1e3 * (time.perf_counter() - t_begin) / prof_steps
        stats = cache.profile_read()
        cache.profile_enable(False)
        flops_layer, _ = attention_flops(wl, ranges)
        flops_step = flops_layer * wl.n_layers
        kern = {}
        for name, (launches, ms, layers) in stats.items():
            if launches:
                kern[name] = {"launches_per_step": launches // prof_steps, "layers_per_launch": layers / launches,
                              "ms_per_step": ms / prof_steps, "avg_us": 1e3 * ms / launches}
        res["kernels"] = kern
        att_ms = stats["attention"][1] / prof_steps
        col_ms = stats["colsum"][1] / prof_steps      # 0 when the scores come out of the attention launch itself
        res["attention_tflops"] = flops_step / (att_ms * 1e-3) / 1e12
        res["attention_plus_scoring_tflops"] = flops_step / ((att_ms + col_ms) * 1e-3) / 1e12
        res["attention_flops_per_launch"] = flops_step / stats["attention"][0] * prof_steps
        # ---- what the compactions of that pass actually did, and the bytes that takes
        done = {k: v - totals_before[k] for k, v in cache.totals().items()}
        # ---- the same pass with the scores taken by the separate kernel: the attention launch then
        # holds Eq. 1 alone (what earlier versions of this line reported as the attention roofline)
        res["eq1_alone"] = None
        if eq1_alone:
            cache.set_score_sweep(0)
            cache.profile_enable(True)
            run_steps(K.Prefill(cache, wl.n_layers, overlap=False), cache, wl, data, ranges, prof_steps, outs)
            torch.cuda.synchronize()
            alone = cache.profile_read()
            cache.profile_enable(False)
            cache.set_score_sweep(score_sweep)
            a_n, a_ms, _ = alone["attention"]
            c_n, c_ms, _ = alone["colsum"]
            res["eq1_alone"] = {
                "avg_launch_us": round(1e3 * a_ms / a_n, 2),
                "achieved": round(flops_step * prof_steps / (a_ms * 1e-3) / 1e12, 2),
                "separate_scoring_avg_launch_us": round(1e3 * c_ms / c_n, 2) if c_n else None,
                "with_separate_scoring_tflops": round(flops_step * prof_steps / ((a_ms + c_ms) * 1e-3) / 1e12, 2),
            }
        row = wl.head_dim * 2                       # bytes of one K or V row
        appended, select_bytes, colsum_flops, evicting_launches = 0, 0, 0, 0
        c = 0
        for _, n in ranges:
            if c + n <= wl.budget:
                appended += n * wl.n_kv_heads
            else:
                # score and token index of every candidate in, keep flag and merge target out
                select_bytes += (c + n) * wl.n_kv_heads * (4 + 4 + 1 + 4)
                colsum_flops += 2 * wl.head_dim * wl.n_q_heads * (n * c + n * (n + 1) // 2)
                evicting_launches += 1
            c = min(wl.budget, c + n)
        appended *= wl.n_layers * prof_steps
        select_bytes = select_bytes * wl.n_layers * prof_steps + done["moved_rows"] * 16 + done["merge_destinations"] * 32
        colsum_flops *= wl.n_layers * prof_steps
        # a moved row: K and V read and written, token index and weight written, its plan entry read
        move_bytes = (appended + done["moved_rows"]) * (4 * row + 8) + done["moved_rows"] * 16
        # a merge: destination and sources read (K, V and weight), destination written, its plan entry read
        merge_bytes = ((done["merge_destinations"] + done["merge_sources"]) * (2 * row + 4)
                       + done["merge_destinations"] * (2 * row + 4 + 32))
        res["compaction_totals_per_step"] = {k: v // prof_steps for k, v in done.items()}
        res["compaction_totals_per_step"]["appended_rows"] = appended // prof_steps
        res["hbm_bytes_per_step"] = {"select": select_bytes // prof_steps, "merge": merge_bytes // prof_steps,
                                     "move": move_bytes // prof_steps}
        res["colsum_flops_per_step"] = colsum_flops // prof_steps
    cache.close()
    del data
    torch.cuda.empty_cache()
    return res


def cpu_baseline(wl, min_s=10.0, budget_s=25.0):
    """The oracle as it stands on this machine's host cores: whole layers of the workload until
    min_s of oracle time has passed (a layer is cut short at budget_s); layer-tokens per
    second divided by the layer count gives whole-job tokens/s."""
    import numpy as np
    from kvp_workload import layer_inputs, bf16_bits_to_f32, chunk_ranges
    from oracle import kvp_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = len(os.sched_getaffinity(0))
    ranges = chunk_ranges(wl.n_tokens, wl.chunk)
    done_tokens, done_blocks, layers_started = 0, 0, 0
    elapsed = 0.0                                   # oracle time only: input generation is not the method
    for layer in range(wl.n_layers):
        qb, kb, vb = layer_inputs(wl, layer)
        q, k, v = (bf16_bits_to_f32(x).astype(np.float64) for x in (qb, kb, vb))
        layers_started += 1
        t_begin = time.perf_counter()
        oc = O.LayerCache(wl.n_kv_heads, wl.head_dim, wl.budget, wl.segments, True)
        for t0, n in ranges:
            oc.step(t0, q[t0:t0 + n], k[t0:t0 + n], v[t0:t0 + n])
            done_tokens += n
            done_blocks += 1
            if elapsed + time.perf_counter() - t_begin > budget_s:
                break
        elapsed += time.perf_counter() - t_begin
        if elapsed > min_s:
            break
    return {
        "value": done_tokens / (elapsed * wl.n_layers),
        "unit": "tokens/s",
        "cores": cores,
        "kind": "oracle",
        "sample": "%d of %d layers, %d blocks of the %d per layer (%d layer-tokens) in %.1f s, "
                  "float64 NumPy; scaled by the layer count" % (
                      layers_started, wl.n_layers, done_blocks, len(ranges), done_tokens, elapsed),
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="long_video")
    ap.add_argument("--others", type=int, default=1, help="also time the other four shapes (few steps)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle leg")
    ap.add_argument("--streams", type=int, default=1, choices=(1, 2),
                    help="1: everything in line, the compactions of a group of layers after the group's attention "
                         "launches (measured faster); 2: those compactions on a second stream beside the next "
                         "group's attention")
    ap.add_argument("--scratch-sets", type=int, default=16,
                    help="scratch sets of the cache: one select/merge/move launch covers a group of layers, "
                         "sets / 2 of them with two streams (two events between the streams per group), "
                         "min(sets, 16) with one")
    ap.add_argument("--n-obs", type=int, default=64,
                    help="also time the prefill scored with this many proxy queries (0: skip)")
    ap.add_argument("--variants", type=int, default=1,
                    help="also time proxy-query and key-only scoring, the bulk first pass and the decode step")
    ap.add_argument("--peaks", type=int, default=1,
                    help="also measure what this GPU attains on a register-resident bf16 MFMA loop and a device copy")
    ap.add_argument("--score-sweep", type=int, default=1, choices=(0, 1),
                    help="1: the scores of Eq. 4 out of the attention launch's second sweep (the library's default); "
                         "0: by the separate column-sum kernel (for profiles of the attention launch with Eq. 1 alone)")
    ap.add_argument("--eq1-alone", type=int, default=1,
                    help="also time one pass with the scores taken by the separate kernel (the attention launch "
                         "then holds Eq. 1 alone); 0 keeps that pass out of a counter run")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run a plain 256 MiB device copy (reference for HBM traffic counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus %d is not supported (no collectives, "
              "nothing to shard: budget, scores and eviction are per layer and KV head)" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2604_16734_amd as K
    from kvp_workload import WORKLOADS, get_workload
    K.lib()                                   # fail loudly if the HIP library is not built
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    device = "cuda:0"
    threads = min(16, len(os.sched_getaffinity(0)))
    wl = get_workload(args.workload)
    if args.copy_probe:
        a = torch.empty(256 << 20, dtype=torch.uint8, device=device).fill_(1)
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        del a, b
    main_res = bench_workload(wl, args.steps, args.warmup, device, threads, streams=args.streams, n_obs=args.n_obs,
                              scratch_sets=args.scratch_sets, variants=bool(args.variants), eq1_alone=bool(args.eq1_alone),
                              score_sweep=args.score_sweep)

    others = {}
    if args.others:
        for w in WORKLOADS:
            if w.name != wl.name:
                r = bench_workload(w, max(3, args.steps // 2), 2, device, threads, profile=True, streams=args.streams,
                                   scratch_sets=args.scratch_sets, variants=False, eq1_alone=False)
                others[w.name] = {
                    "tokens_per_s": round(r["tokens_per_s"], 1), "ms_per_step": round(r["ms_per_step"], 4),
                    "attention_tflops": round(r["attention_tflops"], 2),
                    "attention_plus_scoring_tflops": round(r["attention_plus_scoring_tflops"], 2),
                    "persistent_kv_bytes": r["persistent_kv_bytes"],
                }

    peaks = attainable_peaks(device) if args.peaks else None
    att = main_res["kernels"]["attention"]
    achieved = main_res["attention_tflops"]
    kern = main_res["kernels"]

    def entry(kernel, bound, achieved_v, unit, per_launch_key, per_launch, note=None):
        peak = PEAK_BF16_TFLOPS if bound == "mfma" else PEAK_HBM_GBS
        e = {"kernel": kernel, "bound": bound, "achieved": round(achieved_v, 2), "peak": peak, "unit": unit,
             "frac": round(achieved_v / peak, 4), "avg_launch_us": round(kern[kernel]["avg_us"], 2),
             per_launch_key: per_launch}
        if peaks:
            got = peaks["mfma_bf16_tflops"] if bound == "mfma" else peaks["hbm_copy_GBps"]
            e["frac_of_attainable"] = round(achieved_v / got, 4)
        if note:
            e["note"] = note
        return e

    executed = main_res["attention_flops_per_launch"]
    if "colsum" not in kern:
        executed += main_res["colsum_flops_per_step"] / att["launches_per_step"]
    rooflines = [entry("attention", "mfma", achieved, "TFLOP/s", "flops_per_launch", main_res["attention_flops_per_launch"])]
    if "colsum" in kern:
        f = main_res["colsum_flops_per_step"]
        rooflines.append(entry("colsum", "mfma", f / (kern["colsum"]["ms_per_step"] * 1e-3) / 1e12, "TFLOP/s",
                               "flops_per_launch", f / kern["colsum"]["launches_per_step"],
                               "the second QK^T sweep's own flops 2 d Hq (n c + n (n + 1) / 2); they are not "
                               "counted as algorithmic work of the path (see attention_plus_scoring_frac)"))
    for name in ("select", "merge", "move"):
        if name in kern:
            b = main_res["hbm_bytes_per_step"][name]
            rooflines.append(entry(name, "hbm", b / (kern[name]["ms_per_step"] * 1e-3) / 1e9, "GB/s",
                                   "bytes_per_launch", round(b / kern[name]["launches_per_step"], 1),
                                   "bytes from this run's own counts (compaction_totals_per_step)"))
    dec = main_res["decode_step"]
    if dec:
        e = {"kernel": "decode", "bound": "hbm", "achieved": dec["GBps_on_device"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
             "frac": round(dec["GBps_on_device"] / PEAK_HBM_GBS, 4), "avg_launch_us": dec["us_per_layer_on_device"],
             "bytes_per_launch": dec["bytes_per_layer"]}
        if peaks:
            e["frac_of_attainable"] = round(dec["GBps_on_device"] / peaks["hbm_copy_GBps"], 4)
        rooflines.append(e)
    compact_us = sum(kern[k]["ms_per_step"] for k in ("select", "merge", "move") if k in kern) * 1e3
    compact_bytes = sum(main_res["hbm_bytes_per_step"].values())
    line = {
        "metric": "prefill tokens/s at fixed KV budget (1 GPU)",
        "value": round(main_res["tokens_per_s"], 1),
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(main_res["ms_per_step"], 4),
        "ms_per_step_median_hip_events": round(main_res["ms_per_step_median_hip_events"], 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": wl.name, "n_layers": wl.n_layers, "n_q_heads": wl.n_q_heads,
            "n_kv_heads": wl.n_kv_heads, "head_dim": wl.head_dim, "prefix_tokens": wl.n_tokens,
            "chunk": wl.chunk, "kv_budget_per_head": wl.budget, "merge": 1,
            "step": "whole prefill: all blocks x all layers of prefill_chunk + compact",
        },
        "roofline": {
            "kernel": "attention",
            "bound": "mfma",
            "achieved": round(achieved, 2),
            "peak": PEAK_BF16_TFLOPS,
            "unit": "TFLOP/s",
            "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
            "traffic": ATTENTION_TRAFFIC_BYTES.get(wl.name),
            "traffic_source": "stored figure from the rocprofv3 --pmc runs summarised under profiles/ "
                              "(FETCH_SIZE and WRITE_SIZE scaled by a plain copy); not measured by this run",
            "avg_launch_us": round(att["avg_us"], 2),
            "flops_per_launch": main_res["attention_flops_per_launch"],
            "attention_plus_scoring_tflops": round(main_res["attention_plus_scoring_tflops"], 2),
            "attention_plus_scoring_frac": round(main_res["attention_plus_scoring_tflops"] / PEAK_BF16_TFLOPS, 4),
            "frac_of_attainable": round(achieved / peaks["mfma_bf16_tflops"], 4) if peaks else None,
            # context, not the roofline figure: the launch recomputes QK^T for the scores (Eq. 4 needs
            # every row's final normaliser), so its matrix pipe executes these flops, not flops_per_launch
            "mfma_flops_executed_per_launch": executed,
            "executed_tflops": round(executed / (att["avg_us"] * 1e-6) / 1e12, 2),
            "executed_frac": round(executed / (att["avg_us"] * 1e-6) / 1e12 / PEAK_BF16_TFLOPS, 4),
            "note": "the launch holds Eq. 1 AND the second sweep that leaves the scores of Eq. 4; only Eq. 1's flops "
                    "are counted, so this is the attention-plus-scoring figure. eq1_alone: the same run with the "
                    "scores taken by the separate kernel instead (kvp_set_score_sweep 0), i.e. the attention launch "
                    "with Eq. 1 only, and what the two launches reach together",
            "eq1_alone": dict(main_res["eq1_alone"], unit="TFLOP/s",
                              frac=round(main_res["eq1_alone"]["achieved"] / PEAK_BF16_TFLOPS, 4),
                              with_separate_scoring_frac=round(main_res["eq1_alone"]["with_separate_scoring_tflops"] / PEAK_BF16_TFLOPS, 4))
                         if main_res["eq1_alone"] else None,
        },
        "rooflines": rooflines,
        "select_merge_move": {
            "us_per_evicting_layer_block": round(compact_us / max(1.0, kern["select"]["launches_per_step"] * kern["select"]["layers_per_launch"]), 2) if "select" in kern else None,
            "layers_per_launch": kern["select"]["layers_per_launch"] if "select" in kern else None,
            "GBps": round(compact_bytes / (compact_us * 1e-6) / 1e9, 1) if compact_us else None,
            "frac_of_hbm_peak": round(compact_bytes / (compact_us * 1e-6) / 1e9 / PEAK_HBM_GBS, 4) if compact_us else None,
        },
        "attainable": peaks,
        "compaction_totals_per_step": main_res["compaction_totals_per_step"],
        "kernels": {k: {kk: round(vv, 3) for kk, vv in v.items()} for k, v in main_res["kernels"].items()},
        "profiled_ms_per_step": round(main_res["profiled_ms_per_step"], 4),
        "peak_kv_bytes": {
            "persistent": main_res["persistent_kv_bytes"],
            "scratch": main_res["scratch_bytes"],
            "one_block_kv_in_flight": main_res["chunk_kv_bytes"],
            "full_cache_would_be": main_res["full_cache_kv_bytes"],
        },
        "other_workloads": others,
        "proxy_query_scoring": main_res["proxy_scoring"],
        "keydiff_scoring": main_res["keydiff_scoring"],
        "bulk_first_pass": main_res["bulk_first_pass"],
        "layerwise_order": main_res["layerwise_order"],
        "decode_step": main_res["decode_step"],
    }
    if not args.no_cpu:
        line["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(line))


if __name__ == "__main__":
    main()

#!/usr/bin/env python3
"""Benchmark of the parallel draft step on one MI355X.

    python bench.py --gpus 1 --steps K --warmup W [--workload all|c0|c1|c2|c3|c4]

A "step" is one ps_draft_step: one forward of the one-layer drafter over n_new real rows plus k [MASK]
rows against the KV cache, LM head with fused softmax/top-k included; in the default mode it is ONE launch of
the persistent kernel.  All inputs are seeded, synthetic and resident in HBM before the timed region.

By default every bf16 workload (c1 7B, c2 13B with the accepted-length mix, c3 batch 8, c4 Llama-3-8B shape)
is timed in turn, K steps each after W warm-up steps, and ONE JSON line is printed whose headline figures
(value, ms_per_step, config, roofline, cpu_baseline) are those of the largest workload, c4; the key
"workloads" carries the same figures for each of them, "c0_latency_us" the tiny fp32 correctness workload's
latency, "stream_read" what a plain streaming read of HBM reaches on this machine.  Per workload:
  * draft tokens/s (k+1 tokens per sequence per step) and latency from the host clock around the K steps,
  * per-step latency percentiles and the persistent kernel's average duration from HIP events on the launch
    stream, and with them the HBM roofline: algorithmic bytes (weights once + valid K/V once + new K/V rows
    once) / duration / 8 TB/s,
  * the HBM traffic per launch that rocprofv3's FETCH_SIZE / WRITE_SIZE counters showed for the same command
    (profiles/hbm_traffic.txt, written from the runs that profiles/*_hbm_traffic.md document),
  * the CPU oracle timed on this machine's host cores on the same inputs, as a baseline.

Aids for the profiles (all run committed code only):
    --calibrate-copy          a copy kernel of known size, to scale the profiler's counters
    --summarize DB [DB ...]   per-kernel durations / counter values of rocprofv3 result databases
    --timeline                per-stretch clock stamps of the persistent kernel (a -DPS_TIMELINE build)
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0   # MI355X HBM3E, published peak
BENCH_WORKLOADS = ("c1", "c2", "c3", "c4")
HEADLINE = "c4"         # the largest single-GPU workload
TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic.txt")


def algorithmic_bytes(wl, kv_len, n_new, k):
    """Weights once + valid KV once + new KV rows written once (per step), in bytes."""
    s = wl.shape
    esz = 2 if s.dtype == "bf16" else 4
    m = n_new + k
    weights = {
        "qkv": (s.q_dim + 2 * s.kv_dim) * s.hidden + s.hidden,
        "oproj": s.hidden * s.q_dim,
        "gateup": 2 * s.ffn * s.hidden + s.hidden,
        "down": s.hidden * s.ffn,
        "lmhead": s.vocab * s.hidden + s.hidden,
    }
    per = {n: v * esz for n, v in weights.items()}
    per["mask_emb"] = k * s.hidden * esz
    per["kv_read"] = sum(2 * l * s.kv_dim * esz for l in kv_len)
    per["kv_write"] = len(kv_len) * 2 * m * s.kv_dim * esz
    per["total"] = sum(per.values())
    return per


def load_traffic_table():
    """profiles/hbm_traffic.txt: lines `workload mode fetch_bytes write_bytes` (HBM bytes per launch of the
    dominant kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled with the copy kernel)."""
    table = {}
    if os.path.exists(TRAFFIC_TABLE):
        for line in open(TRAFFIC_TABLE):
            f = line.split("#")[0].split()
            if len(f) == 4:
                table[(f[0], f[1])] = int(f[2]) + int(f[3])
    return table


def workload_label(wl, kv_len, mix, n_new_mean):
    s = wl.shape
    return ("%s: 1 decoder layer H%d %dq/%dkv x%d F%d V%d, batch %d, KV %s, n_new %s, k %d, topk %d"
            % (wl.name, s.hidden, s.n_heads, s.n_kv_heads, s.head_dim, s.ffn, s.vocab, wl.batch,
               list(kv_len) if wl.batch > 1 else kv_len[0],
               "mix %s (mean %.2f)" % (list(wl.n_new_mix), n_new_mean) if mix else wl.n_new, wl.k, wl.topk))


def setup_workload(torch, wl, steps):
    from paper_2410_05589_amd import binding as B
    from paper_2410_05589_amd import inputs
    shape = wl.shape
    kv_len = inputs.draw_kv_len(wl)
    mix = inputs.draw_n_new_mix(wl, steps) if wl.n_new_mix else None
    max_new = max(wl.n_new_mix) if wl.n_new_mix else wl.n_new
    w = inputs.make_weights(shape, wl.seed)
    drafter = B.Drafter(shape, w, max_batch=wl.batch, max_new=max_new,
                        max_positions=max(kv_len) + max_new + wl.k, max_topk=wl.topk, k_max=wl.k)
    # one input set per distinct n_new (the accepted-length mix of c2); the cache is reset by keeping kv_len
    # fixed, so every step rewrites the same n_new + k rows
    variants = {}
    for n_new in sorted(set(mix)) if mix else [wl.n_new]:
        inp = inputs.make_step_inputs(wl, kv_len=kv_len, n_new=n_new, k=wl.k)
        dev = {n: B.to_device(inp[n], shape.dtype) for n in ("x", "k_cache", "v_cache")}
        outs = drafter.alloc_outputs(wl.batch, n_new, wl.k, wl.topk)
        a = drafter.make_args(dev["x"], dev["k_cache"], dev["v_cache"], inp["kv_offsets"], inp["kv_len"],
                              n_new, wl.k, wl.topk, outs)
        variants[n_new] = (a, inp, outs)
    seq = mix if mix else [wl.n_new] * steps
    return w, drafter, variants, seq, kv_len, mix, max_new


def measure_workload(torch, wl, args, traffic_table, with_oracle, kernel_timing):
    """Times `args.steps` steps of one workload after `args.warmup` warm-up steps; returns its report."""
    from paper_2410_05589_amd import binding as B
    shape = wl.shape
    w, drafter, variants, seq, kv_len, mix, max_new = setup_workload(torch, wl, args.steps + args.warmup)
    stream = torch.cuda.current_stream()
    for i in range(args.warmup):
        drafter.step(variants[seq[i]][0])
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record(stream)
    for i in range(args.steps):
        drafter.step(variants[seq[args.warmup + i]][0])
    ev1.record(stream)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    ev_ms = ev0.elapsed_time(ev1) / args.steps
    tokens_per_step = wl.batch * (wl.k + 1)
    value = tokens_per_step / (ms_per_step * 1e-3)
    timed = seq[args.warmup:]
    n_new_mean = float(np.mean(timed))
    bytes_mean = float(np.mean([algorithmic_bytes(wl, kv_len, n, wl.k)["total"] for n in timed]))
    per = algorithmic_bytes(wl, kv_len, seq[-1], wl.k)

    # ---- per-kernel durations, live, with HIP events on the launch stream (second region of steps)
    kernel_us = roofline = per_step_us = None
    if kernel_timing:
        ksteps = min(args.steps, 200)
        evs = [[torch.cuda.Event(enable_timing=True) for _ in range(B.PS_PROFILE_EVENTS)] for _ in range(ksteps)]
        for row in evs:
            for e in row:
                e.record(stream)          # creates the underlying hipEvent_t
        torch.cuda.synchronize()
        for i in range(ksteps):
            st = B.ps_draft_set_profile_events(drafter.ctx, [e.cuda_event for e in evs[i]])
            assert st == B.PS_OK
            drafter.step(variants[seq[args.warmup + i]][0])
        B.ps_draft_set_profile_events(drafter.ctx, None)
        torch.cuda.synchronize()
        acc = np.zeros(B.PS_PROFILE_EVENTS - 1)
        per_step = []
        for row in evs:
            for j in range(B.PS_PROFILE_EVENTS - 1):
                acc[j] += row[j].elapsed_time(row[j + 1])
            # fused: events 0 and 1 bracket the one kernel of the step; multi: first to last event = all its kernels
            per_step.append(row[0].elapsed_time(row[1 if args.mode == "fused" else -1]) * 1e3)
        per_step_us = {q: round(float(np.percentile(per_step, p)), 2) for q, p in (("p10", 10), ("median", 50), ("p90", 90))}
        kernel_us = {n: float(acc[j] / ksteps * 1e3) for j, n in enumerate(B.PROFILE_KERNELS)}
        dname = "bf16_t" if shape.dtype == "bf16" else "float"
        mt = (wl.batch * (max_new + wl.k) + 15) // 16
        if args.mode == "fused":
            dom_us = float(acc[0] / ksteps * 1e3)   # events 0 and 1 bracket the single launch
            kernel_us = {"fused_kernel": dom_us}
            dom_bytes = float(np.mean([algorithmic_bytes(wl, kv_len, n, wl.k)["total"] for n in timed[:ksteps]]))
            kname = "fused_kernel<%s, %d, %d>" % (dname, shape.head_dim, mt)
        else:
            dom_us = kernel_us["lmhead"]
            dom_bytes = per["lmhead"]
            kname = "gemm_kernel<%s, %d, 4>  (LM head)" % (dname, (wl.batch * (wl.k + 1) + 15) // 16)
        achieved = dom_bytes / (dom_us * 1e-6) / 1e9
        roofline = {"bound": "hbm", "kernel": kname, "achieved": round(achieved, 1), "peak": PEAK_HBM_GBS,
                    "unit": "GB/s", "frac": round(achieved / PEAK_HBM_GBS, 4),
                    "traffic": traffic_table.get((wl.name, args.mode)),
                    "algorithmic_bytes_per_launch": int(dom_bytes), "avg_launch_us": round(dom_us, 2)}

    # ---- the same step captured once in a HIP graph and replayed (only when every step has the same n_new)
    graph_us = None
    if kernel_timing and not mix:
        a0 = variants[wl.n_new][0]
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                drafter.step(a0, stream=side)
        torch.cuda.synchronize()
        for _ in range(min(args.warmup, 20)):
            graph.replay()
        torch.cuda.synchronize()
        g0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        graph_us = (time.perf_counter() - g0) * 1e6 / args.steps
    status = drafter.last_status()

    step_gbs = bytes_mean / (ms_per_step * 1e-3) / 1e9
    rep = {
        "value": round(value, 1), "unit": "tokens/s", "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "dtype": shape.dtype,
        "config": {"workload": workload_label(wl, kv_len, mix, n_new_mean), "tokens_per_step": tokens_per_step},
        "latency_us": round(ms_per_step * 1e3, 2),
        "latency_us_hip_events": round(ev_ms * 1e3, 2),
        "latency_us_per_step_events": per_step_us,
        "latency_us_graph_replay": round(graph_us, 2) if graph_us else None,
        "step_roofline": {"algorithmic_bytes": int(bytes_mean), "achieved_GBps": round(step_gbs, 1),
                          "peak_GBps": PEAK_HBM_GBS, "frac": round(step_gbs / PEAK_HBM_GBS, 4),
                          "roofline_latency_us": round(bytes_mean / PEAK_HBM_GBS / 1e3, 2)},
        "kernel_us": {n: round(v, 2) for n, v in kernel_us.items()} if kernel_us else None,
        "roofline": roofline,
        "status_after_run": B.ps_draft_strerror(status),
    }
    if with_oracle:
        from oracle import ps_oracle
        try:
            from threadpoolctl import threadpool_info
            threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
        except Exception:
            threads = 1
        a, inp, outs = variants[seq[-1]]
        n_new = seq[-1]
        times = []
        for _ in range(args.oracle_steps):
            c0 = time.perf_counter()
            ref = ps_oracle.draft_step(shape, w, inp["x"], inp["k_cache"], inp["v_cache"], inp["kv_offsets"], inp["kv_len"],
                                       n_new, wl.k, wl.topk)
            times.append(time.perf_counter() - c0)
        best = float(np.mean(times))
        torch.cuda.synchronize()
        gpu_top1 = outs["top_ids"].cpu().numpy()[..., 0]   # sanity: the timed GPU step agrees with the oracle on the top-1 tokens
        agree = float((gpu_top1 == ref["top_ids"][..., 0]).mean())
        rep["cpu_baseline"] = {"value": round(tokens_per_step / best, 2), "unit": "tokens/s", "cores": int(threads),
                               "kind": "oracle", "sample": "%d full steps of the same workload (numpy float64, "
                               "mean %.2f s per step, host cores available %d)" % (args.oracle_steps, best,
                                                                                    len(os.sched_getaffinity(0))),
                               "top1_agreement_with_gpu": agree}
    drafter.close()
    return rep


def stream_read_report(torch, mib=1536, iters=20):
    """A plain streaming read of `mib` MiB of HBM (larger than the 256 MB Infinity Cache) with the weight
    streams' access pattern and nothing else (ps_measure_stream_read): the read rate this machine gives."""
    from paper_2410_05589_amd import debug as DBG
    n = mib << 20
    buf = torch.ones(n, dtype=torch.uint8, device="cuda:0")
    stream = torch.cuda.current_stream()
    for _ in range(3):
        assert DBG.ps_measure_stream_read(buf.data_ptr(), n, stream.cuda_stream) == 0
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(iters):
        DBG.ps_measure_stream_read(buf.data_ptr(), n, stream.cuda_stream)
    e1.record(stream)
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / iters
    gbs = n / (us * 1e-6) / 1e9
    return {"GBps": round(gbs, 1), "frac_of_peak": round(gbs / PEAK_HBM_GBS, 4), "bytes": n, "us": round(us, 2),
            "kernel": "stream_read_kernel (16-byte non-temporal loads, 8 in flight per lane, one workgroup of 512 per CU)"}


def calibrate_copy(torch, mib, iters):
    """Runs the copy kernel of known size (exactly `mib` MiB read and written per launch): under rocprofv3
    --pmc FETCH_SIZE (then WRITE_SIZE), true KiB / counter is the factor for the other kernels' counters."""
    from paper_2410_05589_amd import debug as DBG
    n = mib << 20
    src = torch.ones(n, dtype=torch.uint8, device="cuda:0")
    dst = torch.zeros(n, dtype=torch.uint8, device="cuda:0")
    stream = torch.cuda.current_stream().cuda_stream
    torch.cuda.synchronize()
    for _ in range(iters):
        assert DBG.ps_measure_copy(dst.data_ptr(), src.data_ptr(), n, stream) == 0
    torch.cuda.synchronize()
    print("copy_kernel: %d MiB read and %d MiB written per launch, %d launches" % (mib, mib, iters))


def summarize(paths):
    """Per-kernel durations (kernel trace) and per-kernel counter averages (--pmc) of rocprofv3 databases."""
    import re
    import sqlite3
    for path in paths:
        c = sqlite3.connect(path)
        tables = [r[0] for r in c.execute("select name from sqlite_master where type in ('table', 'view')")]
        print("== %s" % path)
        if "kernels" in tables:
            rows = c.execute("select name, count(*), avg(end-start), min(end-start), max(end-start), sum(end-start) "
                             "from kernels group by name order by sum(end-start) desc").fetchall()
            tot = sum(r[5] for r in rows) or 1
            print("%-70s %6s %10s %10s %10s %6s" % ("kernel", "calls", "avg_us", "min_us", "max_us", "pct"))
            for r in rows:
                n = re.sub(r"\(.*", "", re.sub(r"\(anonymous namespace\)::", "", r[0]))
                print("%-70s %6d %10.2f %10.2f %10.2f %6.1f" % (n[:70], r[1], r[2] / 1e3, r[3] / 1e3, r[4] / 1e3, 100 * r[5] / tot))
        if "counters_collection" in tables:
            rows = c.execute("select kernel_name, counter_name, count(*), avg(value), min(value), max(value) from "
                             "counters_collection group by kernel_name, counter_name order by avg(value) desc").fetchall()
            print("%-60s %-14s %6s %14s %14s %14s" % ("kernel", "counter", "calls", "avg", "min", "max"))
            for r in rows[:16]:
                n = re.sub(r"\(.*", "", re.sub(r"\(anonymous namespace\)::", "", r[0]))
                print("%-60s %-14s %6d %14.1f %14.1f %14.1f" % (n[:60], r[1], r[2], r[3], r[4], r[5]))


# (attention stamps: those of the bf16 kernels; 46 is taken by the float32 kernels only)
STAMP_NAMES = {1: "start", 32: "attn start", 44: "attn unit top", 45: "attn query rows placed", 46: "attn maxima exchanged",
               47: "attn key groups done", 48: "attn unit done", 34: "attn units done", 36: "attn end", 40: "merge start",
               41: "merge statistics here", 43: "merge wavefront lists done", 49: "merge barrier passed", 42: "merge candidates", 56: "merge row written", 62: "end"}
for _ph, _nm in enumerate(["qkv", "oproj", "gateup", "down", "lm"]):
    for _k, _sfx in enumerate(["enter", "panel staged", "streamed", "tile sums added", "epilogue done", "end"]):
        STAMP_NAMES[2 + _ph * 6 + _k] = _nm + " " + _sfx
STAMP_ORDER = [1] + list(range(2, 8)) + [32, 44, 45, 46, 47, 48, 34, 36] + list(range(8, 32)) + [40, 41, 43, 49, 42, 56, 62]


def timeline(torch, wl, steps=30):
    """Clock stamps of the persistent kernel (a library built with PS_BUILD_DEFS=-DPS_TIMELINE): for every
    stamp the earliest, median and latest workgroup, in microseconds since the first workgroup started."""
    from paper_2410_05589_amd import debug as DBG
    w, drafter, variants, seq, kv_len, mix, max_new = setup_workload(torch, wl, steps)
    tl = torch.zeros(64 * 1024, dtype=torch.int64, device="cuda:0")
    assert DBG.ps_draft_debug_timeline(drafter.ctx, tl.data_ptr()) == 0
    for i in range(steps):     # the last of a back-to-back series is the one that is looked at
        drafter.step(variants[seq[i]][0])
    torch.cuda.synchronize()
    t = tl.cpu().numpy().reshape(64, 1024)[:, :256].astype(np.float64)
    if t[63].max() == 0:
        print("no stamps: the library was not built with -DPS_TIMELINE", file=sys.stderr)
        sys.exit(2)
    wall0, wall1 = t[0] * 0.01, t[63] * 0.01     # 100 MHz counter -> us
    f = np.median((t[62] - t[1]) / (wall1 - wall0))   # shader clock ticks per us
    base = wall0.min()
    print("workload %s, n_new %d: kernel spans %.2f .. %.2f us per workgroup; %.1f clock ticks per us"
          % (wl.name, seq[steps - 1], (wall1 - wall0).min(), (wall1 - wall0).max(), f))
    print("%-26s %8s %8s %8s | %9s" % ("stamp", "min", "median", "max", "d(median)"))
    prev = None
    for e in STAMP_ORDER:
        x = ((wall0 - base) + (t[e] - t[1]) / f)[t[e] > 0]
        if x.size == 0:
            continue
        med = float(np.median(x))
        print("%-26s %8.2f %8.2f %8.2f | %9.2f" % (STAMP_NAMES.get(e, str(e)), x.min(), med, x.max(), med - prev if prev is not None else 0.0))
        prev = med
    drafter.close()


def input_stage_report(torch, name="c1", steps=200, warmup=20):
    """The draft step with its input stage fused in (Section 4.3), on workload `name`: token ids instead of hidden
    states (the real rows are gathered from the shared embedding table), and token ids + target features through
    the fully connected layer (a small-M GEMM kernel in front of the persistent kernel).  Latency per step from HIP
    events; algorithmic bytes = the step's + what the input stage has to read (the projection's weights once, the
    gathered embedding rows, the features)."""
    from paper_2410_05589_amd import binding as B
    from paper_2410_05589_amd import inputs
    from paper_2410_05589_amd.configs import WORKLOADS
    wl = WORKLOADS[name]
    shape = wl.shape
    esz = 2 if shape.dtype == "bf16" else 4
    w = inputs.make_weights(shape, wl.seed)
    w.update(inputs.make_input_stage_weights(shape, wl.seed))
    kv_len = inputs.draw_kv_len(wl)
    inp = inputs.make_step_inputs(wl, kv_len=kv_len)
    tin = inputs.make_input_stage_inputs(wl)
    d = B.Drafter(shape, w, max_batch=wl.batch, max_new=wl.n_new, max_positions=max(kv_len) + wl.m, max_topk=wl.topk, k_max=wl.k)
    dev = {n: B.to_device(inp[n], shape.dtype) for n in ("x", "k_cache", "v_cache")}
    tok = torch.from_numpy(tin["token_ids"]).to("cuda:0")
    feat = B.to_device(tin["features"], shape.dtype)
    outs = d.alloc_outputs(wl.batch, wl.n_new, wl.k, wl.topk)
    base = algorithmic_bytes(wl, kv_len, wl.n_new, wl.k)["total"]
    rows = wl.batch * wl.n_new
    modes = {"hidden_states": (dict(x=dev["x"]), base),
             "token_ids": (dict(x=None, token_ids=tok), base),     # (the gathered rows replace the x rows: same bytes)
             "token_ids_and_features": (dict(x=None, token_ids=tok, features=feat),
                                        base + (2 * shape.hidden * shape.hidden + shape.hidden + rows * shape.hidden) * esz)}
    rep = {"workload": name}
    stream = torch.cuda.current_stream()
    for mode, (kw, nbytes) in modes.items():
        a = d.make_args(kw.pop("x"), dev["k_cache"], dev["v_cache"], inp["kv_offsets"], inp["kv_len"], wl.n_new, wl.k, wl.topk, outs, **kw)
        for _ in range(warmup):
            d.step(a)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(steps):
            d.step(a)
        e1.record(stream)
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / steps
        gbs = nbytes / (us * 1e-6) / 1e9
        rep[mode] = {"latency_us": round(us, 2), "algorithmic_bytes": int(nbytes),
                     "roofline": {"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                  "frac": round(gbs / PEAK_HBM_GBS, 4), "traffic": None}}
    assert d.last_status() == 0
    d.close()
    return rep


def sampling_report(torch, name="c1", steps=200, warmup=20):
    """The draft step with the sampling epilogue on (temperature 1, one Gumbel-max draw per output row inside
    the persistent kernel) against the same step without it, on workload `name`; the draw adds no bytes."""
    from paper_2410_05589_amd import binding as B
    from paper_2410_05589_amd import inputs
    from paper_2410_05589_amd.configs import WORKLOADS
    wl = WORKLOADS[name]
    shape = wl.shape
    w = inputs.make_weights(shape, wl.seed)
    kv_len = inputs.draw_kv_len(wl)
    inp = inputs.make_step_inputs(wl, kv_len=kv_len)
    d = B.Drafter(shape, w, max_batch=wl.batch, max_new=wl.n_new, max_positions=max(kv_len) + wl.m, max_topk=wl.topk, k_max=wl.k)
    dev = {n: B.to_device(inp[n], shape.dtype) for n in ("x", "k_cache", "v_cache")}
    nbytes = algorithmic_bytes(wl, kv_len, wl.n_new, wl.k)["total"]
    rep = {"workload": name}
    stream = torch.cuda.current_stream()
    for mode, sample in (("top_k_only", False), ("with_draw", True)):
        outs = d.alloc_outputs(wl.batch, wl.n_new, wl.k, wl.topk, sample=sample)
        a = d.make_args(dev["x"], dev["k_cache"], dev["v_cache"], inp["kv_offsets"], inp["kv_len"], wl.n_new, wl.k, wl.topk, outs,
                        temperature=1.0, sample_seed=2024)
        for _ in range(warmup):
            d.step(a)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(steps):
            d.step(a)
        e1.record(stream)
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / steps
        gbs = nbytes / (us * 1e-6) / 1e9
        rep[mode] = {"latency_us": round(us, 2),
                     "roofline": {"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                  "frac": round(gbs / PEAK_HBM_GBS, 4), "traffic": None}}
    d.close()
    return rep


def group_attention_report(torch, with_oracle, T=2048, k=4, heads=32, d=128, calls=20):
    """The attention of group-wise parallel training (Section 4.1) for one training sequence of T tokens laid out
    as T parallel groups of k + 1 rows, the 7B drafter's 32 heads x 128, bf16.  A dense contraction: its bound is
    the MFMA peak; FLOPs = 4 d per visible (query, key) pair and head (scores and P.V)."""
    from paper_2410_05589_amd import binding as B
    from paper_2410_05589_amd import inputs
    from paper_2410_05589_amd import train as TR
    inp = inputs.make_group_attention_inputs(1, 1, T, k, heads, heads, d, "bf16")
    a = TR.make_args(1, T, k, heads, heads, d, "bf16", 10000.0)
    q, kk, v = (B.to_device(inp[n], "bf16") for n in ("q", "k", "v"))
    out = torch.empty((1, T * (k + 1), heads, d), dtype=torch.float32, device="cuda:0")
    ws = torch.empty(TR.ps_group_attention_workspace_bytes(a) + 256, dtype=torch.uint8, device="cuda:0")
    a.q, a.k_, a.v, a.out = q.data_ptr(), kk.data_ptr(), v.data_ptr(), out.data_ptr()
    a.workspace, a.workspace_bytes = (ws.data_ptr() + 255) & ~255, ws.numel() - 256
    stream = torch.cuda.current_stream()
    for _ in range(3):
        assert TR.ps_group_attention(a, stream.cuda_stream) == 0
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(calls):
        TR.ps_group_attention(a, stream.cuda_stream)
    e1.record(stream)
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) * 1e3 / calls
    pairs = (k + 1) * T * (T + 1) // 2 + T * k * (k + 1) // 2
    flops = 4.0 * d * pairs * heads
    tf = flops / (us * 1e-6) / 1e12
    rep = {"workload": "T %d tokens x (1 + %d [MASK]) = %d rows, %d heads x %d, bf16, 1 sequence" % (T, k, T * (k + 1), heads, d),
           "latency_us": round(us, 1), "visible_pairs_per_head": pairs, "dtype": "bf16",
           "roofline": {"bound": "mfma", "achieved": round(tf, 2), "peak": 2500.0, "unit": "TFLOP/s", "frac": round(tf / 2500.0, 4),
                        "traffic": None, "flops_per_launch": flops,
                        "note": "scores and P.V on the matrix cores, every operand split into bf16 high + low parts (2 MFMAs per product); a query tile fills 5..15 of an MFMA tile's 16 rows"}}
    if with_oracle:
        from oracle import group_attention as ga
        Ts = 96                                    # the oracle on the first 96 tokens (480 rows) of 4 heads
        c0 = time.perf_counter()
        want = ga.group_attention(inp["q"][0][:Ts * (k + 1), :4], inp["k"][0][:Ts * (k + 1), :4], inp["v"][0][:Ts * (k + 1), :4],
                                  Ts, k, 10000.0, "bf16")
        cpu_s = time.perf_counter() - c0
        got = out.cpu().numpy()[0, :Ts * (k + 1), :4]
        spairs = ((k + 1) * Ts * (Ts + 1) // 2 + Ts * k * (k + 1) // 2) * 4
        rep["cpu_baseline"] = {"value": round(4.0 * d * spairs / cpu_s / 1e9, 3), "unit": "GFLOP/s", "cores": 1, "kind": "oracle",
                               "sample": "the first %d tokens of 4 heads (numpy float64, %.2f s)" % (Ts, cpu_s)}
        rep["max_abs_error_vs_oracle_on_sample"] = float(np.abs(got - want).max())
    return rep


def verify_walk_report(torch, with_oracle, vocab=32000, k=5, calls=200):
    """Tree construction + acceptance walk (the step after the draft step in Algorithm 1) on a tree of the
    workload's drafter: 61 nodes (fan-out 4, 2, 2, 1, 1 over the k+1 = 6 draft rows) for k = 5, 46 nodes
    (fan-out 3, 2, 1, ...) for k = 8; the workload's vocabulary; one sequence; a target that agrees with the
    drafter's next row to 70 %.  Latency per call from HIP
    events over `calls` back-to-back calls; bytes = what the walk has to read when P stays on chip (first
    rejection at a node: the target's row and the draft row; further ones: the draft row; the final draw: the
    target's row if P is still that row), counted on the oracle's walk of the same inputs."""
    from paper_2410_05589_amd import inputs
    from paper_2410_05589_amd import verify as VF
    dev = torch.device("cuda:0")
    fan = ([4, 2, 2, 1, 1] + [1] * 8)[:k] if k <= 5 else ([3, 2] + [1] * 8)[:k]
    rows, topk, batch = k + 1, 8, 1
    parent, rank = inputs.draft_tree(fan)
    inp = inputs.verify_inputs(1, batch, parent, rank, rows, topk, vocab, agreement=0.7)
    n = len(parent)
    tree = VF.make_tree(parent, rank)
    top_ids = torch.from_numpy(inp["top_ids"]).to(dev)
    tokens = torch.zeros((batch, n), dtype=torch.int32, device=dev)
    q, p, r = (torch.from_numpy(inp[x]).to(dev) for x in ("q", "p", "r"))
    n_acc = torch.zeros((batch,), dtype=torch.int32, device=dev)
    path = torch.zeros((batch, rows), dtype=torch.int32, device=dev)
    out_tokens = torch.zeros((batch, rows + 1), dtype=torch.int32, device=dev)
    a = VF.ps_verify_args()
    a.batch, a.rows, a.vocab = batch, rows, vocab
    a.tokens, a.q, a.p, a.r = tokens.data_ptr(), q.data_ptr(), p.data_ptr(), r.data_ptr()
    a.n_accepted, a.path, a.out_tokens = n_acc.data_ptr(), path.data_ptr(), out_tokens.data_ptr()
    stream = torch.cuda.current_stream().cuda_stream

    def build():
        st = VF.ps_tree_tokens(tree, batch, rows, topk, top_ids.data_ptr(), tokens.data_ptr(), stream)
        assert st == 0, st

    def walk():
        st = VF.ps_verify_walk(tree, a, stream)
        assert st == 0, st

    def timed(fns):
        for _ in range(20):
            for f in fns:
                f()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(calls):
            for f in fns:
                f()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / calls

    both_us = timed([build, walk])
    walk_us = timed([walk])
    a.tokens, a.top_ids, a.topk = None, top_ids.data_ptr(), topk     # the walk reads its tokens from top_ids itself
    fused_us = timed([walk])
    a.tokens = tokens.data_ptr()
    rep = {"workload": "tree of %d nodes (fan-out %s), %d draft rows, V %d, batch 1, target agrees 70 %%"
                       % (n, ",".join(str(f) for f in fan), rows, vocab),
           "latency_us_tree_and_walk": round(both_us, 2), "latency_us_walk": round(walk_us, 2),
           "latency_us_walk_from_top_ids": round(fused_us, 2), "calls": calls,
           "dtype": "f64", "n_accepted": int(n_acc.cpu().numpy()[0])}
    if with_oracle:
        from oracle import verify_walk as vw
        tok = vw.tree_tokens(inp["top_ids"][0], parent, rank)
        c0 = time.perf_counter()
        ref = vw.acceptance_walk(parent, tok, inp["q"][0], inp["p"][0], inp["r"][0])
        cpu_s = time.perf_counter() - c0
        nbytes = vocab * (8 * ref["rejected_from_row"] + 4 * ref["rejected_from_residual"]
                          + (4 if ref["final_from_row"] else 0))
        gbs = nbytes / (walk_us * 1e-6) / 1e9
        rep.update({"agrees_with_oracle": bool(out_tokens.cpu().numpy()[0, :len(ref["tokens"])].tolist() == ref["tokens"]),
                    "rejections": ref["rejected_from_row"] + ref["rejected_from_residual"],
                    "roofline": {"bound": "hbm", "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
                                 "frac": round(gbs / PEAK_HBM_GBS, 5), "algorithmic_bytes_per_launch": int(nbytes),
                                 "traffic": None,
                                 "note": "a chain of dependent steps on one compute unit (8 for V 128256) per sequence: bound by latency, not by HBM"},
                    "cpu_baseline": {"value": round(cpu_s * 1e6, 1), "unit": "us per walk", "cores": 1, "kind": "oracle",
                                     "sample": "one walk of the same inputs (numpy float64)"}})
    return rep


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=300)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--workload", default="all", help="all (c1..c4 timed, c4 the headline) or one of c0..c4")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--oracle-steps", type=int, default=2)
    ap.add_argument("--no-kernel-timing", action="store_true")
    ap.add_argument("--no-next-rows", action="store_true", help="skip the tree + acceptance walk report")
    ap.add_argument("--mode", choices=["fused", "multi"], default="fused",
                    help="fused: the whole step as one persistent kernel (default); multi: one kernel per phase")
    ap.add_argument("--calibrate-copy", action="store_true")
    ap.add_argument("--copy-mib", type=int, default=1024)
    ap.add_argument("--summarize", nargs="+", metavar="DB")
    ap.add_argument("--timeline", action="store_true")
    args = ap.parse_args()
    if args.summarize:
        summarize(args.summarize)
        return
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus %d is not supported"
              % args.gpus, file=sys.stderr)
        sys.exit(2)

    os.environ["PS_DRAFT_MODE"] = args.mode
    import torch
    from paper_2410_05589_amd.configs import WORKLOADS

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    if args.calibrate_copy:
        calibrate_copy(torch, args.copy_mib, 5)
        return
    if args.timeline:
        timeline(torch, WORKLOADS["c1" if args.workload == "all" else args.workload])
        return

    names = BENCH_WORKLOADS if args.workload == "all" else (args.workload,)
    traffic = load_traffic_table()
    reports = {}
    for name in names:
        reports[name] = measure_workload(torch, WORKLOADS[name], args, traffic, not args.no_cpu_baseline,
                                         not args.no_kernel_timing)
        print("bench.py: %s done: %.2f us per step" % (name, reports[name]["latency_us"]), file=sys.stderr, flush=True)
    head = reports[HEADLINE if args.workload == "all" else args.workload]
    result = {
        "metric": "draft tokens/sec (parallel draft step, k+1 tokens per sequence per step)",
        "value": head["value"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": head["dtype"], "data": "synthetic", "mode": args.mode,
    }
    result.update({k: v for k, v in head.items() if k not in result})
    if args.workload == "all":
        result["workloads"] = reports
        c0 = argparse.Namespace(**vars(args))
        c0.steps, c0.warmup = min(args.steps, 200), min(args.warmup, 20)
        result["c0_latency_us"] = measure_workload(torch, WORKLOADS["c0"], c0, traffic, False, False)["latency_us"]
    result["stream_read"] = stream_read_report(torch)
    if not args.no_next_rows:
        hw = WORKLOADS[HEADLINE if args.workload == "all" else args.workload]
        result["next_rows"] = {"verify_walk": verify_walk_report(torch, not args.no_cpu_baseline, vocab=hw.shape.vocab, k=hw.k),
                               "input_stage": input_stage_report(torch), "sampling": sampling_report(torch),
                               "group_attention": group_attention_report(torch, not args.no_cpu_baseline)}
    print(json.dumps(result))


if __name__ == "__main__":
    main()

#!/usr/bin/env python3
"""Benchmark of the RSR matvec hot path on one MI355X.

A step is one full pass of the online hot path (gather v through the column
permutation, aggregate per group, distribute) for the metric workload: a
ternary 4096 x 14336 matrix (P(0)=0.35, P(+1)=P(-1)=0.325), one bf16 vector,
float32 output.  Preprocessing is done once before the timed region; all
handles, vectors and outputs are resident in HBM when timing starts.

One replay is K launches back to back on one stream (one HIP graph; for short
replays plain launches queued behind a spin kernel are timed as well and the
faster way counts).  A timed region is bracketed by HIP events on that stream
and holds as many consecutive replays as make at least 1000 launches (one
replay when K >= 1000), its time divided by their number: the per-replay time
does not carry the two event records.  At least eleven regions are timed and
the median is reported.  Launch i uses weight set i mod H, with H
distinct preprocessed matrices whose streams together exceed twice the 256 MB
Infinity Cache, and consecutive replays continue the rotation, so every launch
streams its weights from HBM ("cold") whatever K is.  Extra fields: the same
loop on a single weight set ("warm", cache resident), the dense packed-2-bit
comparison kernel, and two reference legs in the same launch geometry (an
empty kernel; a kernel that only reads the same number of bytes).  One JSON
line is printed.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
COLD_WORKING_SET = 600e6      # bytes of distinct weight streams cycled through


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=4000)
    ap.add_argument("--warmup", type=int, default=400)
    ap.add_argument("--k", type=int, default=8)
    ap.add_argument("--kind", default="fused", choices=["fused", "2pass"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip warm and dense legs")
    ap.add_argument("--sets", type=int, default=0, help="weight sets to cycle (0 = from size)")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="also run one plain device copy of 256 MiB (a kernel of known traffic, "
                         "to calibrate rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    ap.add_argument("--no-two-chains", action="store_true",
                    help="skip the leg in which two launch chains overlap (its kernels run "
                         "concurrently, which blurs a per-kernel trace)")
    ap.add_argument("--max-sets", type=int, default=40, help="with --configs: weight sets per workload at most")
    ap.add_argument("--no-auto-k", action="store_true", help="with --configs: skip the lines where the "
                                                             "library chooses k (many extra launches)")
    ap.add_argument("--only", default="", help="with --configs: run only the workloads whose name "
                                               "contains this text")
    ap.add_argument("--configs", action="store_true",
                    help="instead of the metric line: time the other workload families (binary "
                         "1024^2, ternary 4096^2 over k, the 2B and 8B layer sets, the retrieval "
                         "table) warm and cold, RSR and dense, one JSON line with a list")
    return ap.parse_args()


MIN_REPLAYS = 11              # timed replays (the median is reported)
PLAIN_LAUNCH_MAX_STEPS = 512  # up to here the K launches are also timed without a graph


def time_graphs(torch, launch_fn, steps, warmup, period=1, replays=MIN_REPLAYS, lanes=1, chain=1):
    """Times `steps` back-to-back launches, captured in HIP graphs, between two HIP events
    on the launch stream; returns the per-replay times in ms (one replay = exactly `steps`
    launches).

    launch_fn(i, stream) makes launch number i; it may depend on i only through i mod
    `period` (the weight set it uses).  When `steps` is not a multiple of `period`,
    consecutive replays continue the rotation where the previous one stopped: replay r
    covers launches r*steps .. r*steps + steps - 1, one captured graph per distinct window,
    so the distance between two uses of the same weight set is `period` launches whatever
    `steps` is.

    lanes = 2 deals the launches of a graph alternately to two streams (two independent
    chains in the captured graph): consecutive launches may then overlap on the GPU.

    chain > 1: a timed region holds `chain` consecutive replays (chain * steps launches) and
    its time is divided by `chain`: with few steps per replay the two event records around a
    region would otherwise weigh as much as a launch.
    """
    from math import gcd
    stream = torch.cuda.Stream()
    side = torch.cuda.Stream() if lanes == 2 else None
    # (long replays visit every weight set many times: one graph serves)
    ngraphs = period // gcd(steps % period, period) if (steps % period and steps < 8 * period) else 1
    with torch.cuda.stream(stream):
        for i in range(min(max(warmup, 1), 64)):     # eager warm-up (also sets kernel attributes)
            launch_fn(i, stream)
        stream.synchronize()
        graphs = []
        for gi in range(ngraphs):
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                if side is not None:
                    side.wait_stream(stream)
                for i in range(steps):
                    launch_fn(gi * steps + i, side if (side is not None and i % 2) else stream)
                if side is not None:
                    stream.wait_stream(side)
            graphs.append(graph)
        # untimed warm-up launches through the same path: every graph once, at least `warmup` launches
        reps = max(ngraphs, (warmup + steps - 1) // steps)
        for r in range(reps):
            graphs[r % ngraphs].replay()
        stream.synchronize()
        torch.cuda.synchronize()
        # the timed replays are enqueued back to back with an event between each two, and the
        # host waits once at the end: the GPU never idles between replays (idle gaps let its
        # clocks drop), and every interval between two events holds exactly `steps` launches
        nrep = max(replays, -(-ngraphs // chain))
        if steps <= PLAIN_LAUNCH_MAX_STEPS:
            spin_for(torch, stream, 200.0)           # the GPU is busy while the host runs ahead
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(nrep + 1)]
        marks[0].record(stream)
        nxt = reps
        for r in range(nrep):
            for _ in range(chain):
                graphs[nxt % ngraphs].replay()
                nxt += 1
            marks[r + 1].record(stream)
        stream.synchronize()
        torch.cuda.synchronize()
        return [marks[r].elapsed_time(marks[r + 1]) / chain for r in range(nrep)]


_spin_ticks_per_us = None


def spin_for(torch, stream, microseconds):
    """Keeps the GPU busy on `stream` for about the given time (a spin kernel)."""
    global _spin_ticks_per_us
    if _spin_ticks_per_us is None:
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda._sleep(100000)
        a.record(stream)
        torch.cuda._sleep(1000000)
        b.record(stream)
        stream.synchronize()
        _spin_ticks_per_us = 1000000 / max(a.elapsed_time(b) * 1e3, 1.0)
    torch.cuda._sleep(int(max(1.0, microseconds * _spin_ticks_per_us)))


def time_stream(torch, launch_fn, steps, warmup, period=1, replays=MIN_REPLAYS, chain=1):
    """The same measurement with plain launches instead of a graph: `steps` launches are
    enqueued behind a spin kernel long enough to cover the host's enqueue time, so that the
    GPU finds them waiting and runs them back to back between the two events.  Returns the
    per-region times in ms."""
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        n = 0
        t_host = time.time()
        for i in range(max(warmup, 8)):
            launch_fn(i, stream)
            n += 1
        host_us = (time.time() - t_host) * 1e6 / n     # host cost of one enqueue
        stream.synchronize()
        spin_for(torch, stream, 100.0 + 1.5 * host_us * steps * chain * replays)
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(replays + 1)]
        marks[0].record(stream)
        for r in range(replays):
            for i in range(steps * chain):
                launch_fn(r * steps * chain + i, stream)
            marks[r + 1].record(stream)
        stream.synchronize()
        torch.cuda.synchronize()
        return [marks[r].elapsed_time(marks[r + 1]) / chain for r in range(replays)]


def log(msg):
    """Progress line on stderr (the JSON line on stdout stays the only output there)."""
    print("bench.py: " + msg, file=sys.stderr, flush=True)


def median(xs):
    xs = sorted(xs)
    n = len(xs)
    return xs[n // 2] if n % 2 else 0.5 * (xs[n // 2 - 1] + xs[n // 2])


def time_graph(torch, launch_fn, steps, warmup, period=1):
    """Median time in ms of a replay of `steps` launches (see time_graphs); regions of at
    least 1000 launches."""
    return median(time_graphs(torch, launch_fn, steps, warmup, period, chain=max(1, -(-1000 // steps))))


def run_configs(args):
    """The workload families beside the metric one.  A step = the whole layer sequence of a
    family on one stream; cold = weight sets cycled so that > 600 MB of streams pass between
    two uses of the same set (fewer sets when one set is that large already)."""
    import numpy as np
    import torch
    import rsr_inputs as gen
    import paper_2603_27462_amd as rsr
    dev = "cuda:0"
    torch.cuda.set_device(0)
    rsr.load_library()
    B, T2, TF, D = (rsr.RSR_BINARY, rsr.RSR_TERNARY_2PASS, rsr.RSR_TERNARY_FUSED,
                    rsr.RSR_DENSE_TERNARY_P2)
    kind_name = {B: "binary", T2: "2pass", TF: "fused", D: "dense_packed2"}
    steps = min(args.steps, 500)
    results = []

    def one(name, make_layers, k, kind, bf16, batch=1, max_sets=40):
        """make_layers(set_index) -> list of int8 matrices (numpy); an entry that is itself a
        list is a group of sibling layers (same input) served by one stacked handle."""
        vt = rsr.RSR_BF16 if bf16 else rsr.RSR_F32
        if (args.only and args.only not in name) or (args.no_auto_k and k == 0 and kind != D):
            return
        max_sets = min(max_sets, args.max_sets)
        print("  ... %s %s k=%d batch=%d" % (name, kind_name[kind], k, batch), file=sys.stderr, flush=True)

        def prep(M):
            if isinstance(M, list):
                return rsr.rsr_preprocess_stacked([torch.from_numpy(x).to(dev) for x in M], k, kind)
            return rsr.rsr_preprocess(torch.from_numpy(M).to(dev), k, kind)

        try:
            sets = [[prep(M) for M in make_layers(0)]]
        except rsr.RsrError as e:
            results.append({"workload": name, "kind": kind_name[kind], "k": k, "error": str(e)})
            return
        nbytes = sum(rsr.rsr_algorithmic_bytes(h, vt, batch) for h in sets[0])
        nsets = int(min(max_sets, max(2, np.ceil(COLD_WORKING_SET / nbytes))))
        for i in range(1, nsets):
            sets.append([prep(M) for M in make_layers(i)])
        vs, outs = [], []
        for h in sets[0]:
            shape = (batch, h.cols)
            x = torch.randn(shape, device=dev)
            vs.append(x.to(torch.bfloat16) if bf16 else x)
            if hasattr(h, "layer_rows"):
                outs.append([[torch.empty(r, dtype=torch.float32, device=dev) for r in h.layer_rows]
                             for _ in range(nsets)])
            else:
                outs.append(torch.empty((nsets, batch, h.rows), dtype=torch.float32, device=dev))

        def run(h, v, o, j, s):
            if hasattr(h, "layer_rows"):
                rsr.rsr_matvec_stacked(h, v[0], None, o[j], stream=s)
            else:
                rsr.rsr_matvec_ex(h, v, out=o[j], stream=s)

        def cold(i, s):
            j = i % nsets
            for h, v, o in zip(sets[j], vs, outs):
                run(h, v, o, j, s)

        def warm(i, s):
            for h, v, o in zip(sets[0], vs, outs):
                run(h, v, o, 0, s)

        tc = time_graph(torch, cold, steps, 50, period=nsets) * 1e3 / steps
        tw = time_graph(torch, warm, steps, 50) * 1e3 / steps
        results.append({"workload": name, "kind": kind_name[kind], "k": k, "batch": batch,
                        "k_used": [h.k for h in sets[0]],
                        "v_dtype": "bf16" if bf16 else "f32", "launches": len(sets[0]),
                        "weight_sets": nsets, "algorithmic_MB": nbytes / 1e6,
                        "cold_us": tc, "warm_us": tw, "cold_GBs": nbytes / tc / 1e3,
                        "kernel": rsr.rsr_kernel_name(sets[0][0], vt)})
        print("  %-44s %-13s k=%2d batch=%d: cold %8.2f us  warm %8.2f us  %6.1f MB  %5.0f GB/s  k used %s"
              % (name, kind_name[kind], k, batch, tc, tw, nbytes / 1e6, nbytes / tc / 1e3,
                 sorted(set(h.k for h in sets[0]))),
              file=sys.stderr, flush=True)
        for hs in sets:
            for h in hs:
                rsr.rsr_destroy(h)

    s0 = gen.BASE_SEED
    one("binary 1024x1024", lambda i: [gen.binary_matrix(1024, 1024, 0.5, s0 + 100 + i)], 8, B, False)
    for k in (4, 6, 8, 10):
        for kind in (T2, TF):
            one("ternary 4096x4096", lambda i: [gen.ternary_matrix(4096, 4096, 1 / 3, s0 + 200 + i)],
                k, kind, False)
    one("ternary 4096x4096", lambda i: [gen.ternary_matrix(4096, 4096, 1 / 3, s0 + 200 + i)], 0, D, False)

    def layers_2b(i):
        return [gen.ternary_matrix(l.rows, l.cols, gen.LLM_2B_P_ZERO, s0 + 300 + 10 * i + n)
                for n, l in enumerate(gen.LLM_2B_LAYERS)]

    def layers_8b(i):
        return [gen.ternary_matrix(l.rows, l.cols, gen.LLM_8B_P_ZERO, s0 + 700 + 10 * i + n)
                for n, l in enumerate(gen.LLM_8B_LAYERS)]

    def layers_2b_merged(i):
        # layers that share their input (q, k, v; gate, up) in one stacked handle and one launch each
        m = layers_2b(i)
        return [m[0:3], m[3], m[4:6], m[6]]

    for k in (6, 8, 0):      # k = 0: the library picks k per layer by timing
        one("2B layer set (7 layers)", layers_2b, k, TF, True)
    one("2B layer set (7 layers)", layers_2b, 0, D, True)
    one("2B layer set, siblings stacked (4 launches)", layers_2b_merged, 0, TF, True)
    one("2B layer set, siblings stacked (4 launches)", layers_2b_merged, 0, D, True)
    for batch in (1, 4):
        for k in (8, 0):
            one("8B layers (3)", layers_8b, k, TF, True, batch=batch, max_sets=12)
        one("8B layers (3)", layers_8b, 0, D, True, batch=batch, max_sets=12)
    table = lambda i: [gen.column_density_binary(1 << 20, 256, 0.05, 0.5, s0 + 900 + i)]
    for k in (4, 8, 12, 0):
        one("retrieval 1048576x256", table, k, B, False, max_sets=6)
    one("retrieval 1048576x256", table, 0, D, False, max_sets=6)
    # 64 queries: back to back (the timed loop above is exactly that, per query) or one call
    one("retrieval 1048576x256, 64 queries in one call", table, 8, B, False, batch=64, max_sets=2)
    one("retrieval 1048576x256, 64 queries in one call", table, 0, D, False, batch=64, max_sets=2)
    print(json.dumps({"configs": results, "steps": steps, "data": "synthetic", "n_gpus": 1}))


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (blocks would shard across GPUs "
              "without communication, but no such run exists); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import rsr_inputs as gen
    import paper_2603_27462_amd as rsr

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    if args.configs:
        run_configs(args)
        return
    dev = "cuda:0"
    torch.cuda.set_device(0)
    rsr.load_library()

    layer = gen.METRIC_LAYER
    rows, cols = layer.rows, layer.cols
    kind = rsr.RSR_TERNARY_FUSED if args.kind == "fused" else rsr.RSR_TERNARY_2PASS

    # ---- inputs (seeded, synthetic) and one-time preprocessing --------------------
    M0 = gen.metric_matrix()
    bits, vals = gen.normal_bf16(cols, seed=gen.BASE_SEED + 41)
    v = torch.from_numpy(bits.view(np.int16)).to(dev).view(torch.bfloat16)
    t_pre = time.time()
    h0 = rsr.rsr_preprocess(torch.from_numpy(M0).to(dev), args.k, kind)
    torch.cuda.synchronize()
    t_pre = time.time() - t_pre
    alg_bytes = rsr.rsr_algorithmic_bytes(h0, rsr.RSR_BF16, 1)
    nsets = args.sets or int(np.ceil(COLD_WORKING_SET / alg_bytes))
    handles = [h0]
    for i in range(1, nsets):
        Mi = gen.ternary_matrix(rows, cols, gen.LLM_8B_P_ZERO, gen.BASE_SEED + 1000 + i)
        handles.append(rsr.rsr_preprocess(torch.from_numpy(Mi).to(dev), args.k, kind))
        del Mi
    outs = torch.zeros((nsets, rows), dtype=torch.float32, device=dev)

    # correctness of the timed configuration against the float64 definition
    import oracle
    want = oracle.dense_matvec(M0, vals.astype(np.float64))
    got = rsr.rsr_matvec_ex(h0, v).cpu().numpy()
    max_err = float(np.max(np.abs(got - want)))
    tol = 1e-4 * float(np.abs(vals.astype(np.float64)).sum())
    if not max_err <= tol:
        print("bench.py: GPU result outside tolerance (%g > %g)" % (max_err, tol), file=sys.stderr)
        sys.exit(1)

    def cold(i, s):
        j = i % nsets
        rsr.rsr_matvec_ex(handles[j], v, out=outs[j], stream=s)

    def warm(i, s):
        rsr.rsr_matvec_ex(h0, v, out=outs[0], stream=s)

    # two ways of issuing the same K launches; short replays are timed with plain launches (a
    # graph replay carries a fixed begin/end cost of about 12 us that would be spread over K)
    log("%d weight sets preprocessed; timing" % nsets)
    # timed regions hold at least 1000 launches: `chain` replays of `steps` launches each
    chain = max(1, -(-1000 // args.steps))
    times_graph = time_graphs(torch, cold, args.steps, args.warmup, period=nsets, chain=chain)
    times_plain = (time_stream(torch, cold, args.steps, args.warmup, period=nsets, chain=chain)
                   if args.steps <= PLAIN_LAUNCH_MAX_STEPS else None)
    use_plain = times_plain is not None and median(times_plain) < median(times_graph)
    times = times_plain if use_plain else times_graph
    ms = median(times)
    us_per_step = ms * 1e3 / args.steps

    def timed(fn, period=1):
        """Median ms of a replay of `steps` launches of fn, issued the way the headline was."""
        if use_plain:
            return median(time_stream(torch, fn, args.steps, args.warmup, period, chain=chain))
        return median(time_graphs(torch, fn, args.steps, args.warmup, period, chain=chain))

    kname = rsr.rsr_kernel_name(h0, rsr.RSR_BF16)
    result = {
        "metric": "ternary matvec/s + effective HBM GB/s (% of peak), 4096x14336, batch 1",
        "value": args.steps / (ms * 1e-3),
        "unit": "matvec/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "input_dtype": "bf16", "data": "synthetic",
        "config": {"workload": "ternary 4096x14336 (P0=0.35), bf16 v, float32 accumulation, batch 1, "
                               "RSR %s k=%d; %d weight sets (%.0f MB of streams) cycled so that every "
                               "launch reads its weights from HBM" %
                               (args.kind, args.k, nsets, nsets * alg_bytes / 1e6),
                   "rows": rows, "cols": cols, "k": args.k, "kind": args.kind, "batch": 1,
                   "v_dtype": "bf16", "weight_sets": nsets,
                   "bytes_between_two_uses_of_a_set": (nsets - 1) * alg_bytes},
        "protocol": {"timed_with": "plain launches behind a spin kernel" if use_plain else "HIP graph replay",
                     "timed_regions": len(times), "replays_per_region": chain,
                     "launches_per_replay": args.steps, "launches_per_region": chain * args.steps,
                     "statistic": "median", "us_per_step_min": min(times) * 1e3 / args.steps,
                     "us_per_step_max": max(times) * 1e3 / args.steps,
                     "graph_us_per_step": median(times_graph) * 1e3 / args.steps,
                     "plain_launch_us_per_step": (median(times_plain) * 1e3 / args.steps
                                                  if times_plain is not None else None),
                     "note": "one replay = exactly `steps` launches back to back on one stream; a timed region "
                             "= `replays_per_region` consecutive replays between two HIP events on that stream "
                             "(at least 1000 launches, so that the event records do not weigh on short "
                             "replays), its time divided by that count; consecutive replays continue the "
                             "rotation over the weight sets; the statistic is taken over the regions; the "
                             "faster of the two ways of issuing the launches is the value"},
    }
    achieved = alg_bytes / (us_per_step * 1e-6) / 1e9
    dense_equiv_bytes = rows * cols // 4 + cols * 2 + rows * 4
    result["roofline"] = {
        "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": achieved / HBM_PEAK_GBS, "traffic": None,
        "kernel": kname,
        "algorithmic_bytes_per_launch": alg_bytes,
        "avg_launch_us": us_per_step,
        "dense_equivalent_bytes": dense_equiv_bytes,
        "dense_equivalent_GBs": dense_equiv_bytes / (us_per_step * 1e-6) / 1e9,
        "dense_equivalent_frac": dense_equiv_bytes / (us_per_step * 1e-6) / 1e9 / HBM_PEAK_GBS,
    }
    traffic_file = os.path.join(ROOT, "profiles", "traffic_rsr_metric.json")
    if os.path.exists(traffic_file):
        with open(traffic_file) as f:
            t = json.load(f)
        if t.get("k") == args.k and t.get("kind") == args.kind and t.get("kernel") == kname:
            result["roofline"]["traffic"] = t.get("hbm_bytes_per_launch")
            result["roofline"]["traffic_source"] = ("profiles/traffic_rsr_metric.json (rocprofv3 FETCH_SIZE + "
                                                    "WRITE_SIZE of an earlier run of this command, not "
                                                    "measured in this run)")
    result["max_abs_err_vs_f64"] = max_err
    result["tolerance"] = tol
    result["preprocess_s"] = t_pre

    if not args.no_extras:
        # the reference legs, same protocol and launch geometry: a launch that does nothing, and
        # a launch that only reads the same number of bytes once
        log("headline %.3f us/step; reference legs" % us_per_step)
        wg, th, lds = rsr.rsr_launch_shape(h0, rsr.RSR_BF16)
        read_bytes = alg_bytes // 1024 * 1024
        pool = torch.randint(0, 255, (nsets * read_bytes,), dtype=torch.uint8, device=dev)
        ms_e = timed(lambda i, s: rsr.rsr_probe_empty(wg, th, lds, s))
        ms_rc = timed(lambda i, s: rsr.rsr_probe_read(pool[(i % nsets) * read_bytes:], read_bytes, wg, th, s),
                      period=nsets)
        ms_rw = timed(lambda i, s: rsr.rsr_probe_read(pool, read_bytes, wg, th, s))
        del pool
        result["reference_legs"] = {
            "launch_floor_us": ms_e * 1e3 / args.steps,
            "stream_read_us": ms_rc * 1e3 / args.steps,
            "stream_read_warm_us": ms_rw * 1e3 / args.steps,
            "stream_read_frac_hbm_peak": read_bytes / (ms_rc * 1e-3 / args.steps) / 1e9 / HBM_PEAK_GBS,
            "geometry": {"workgroups": wg, "threads": th, "lds_bytes": lds, "bytes": read_bytes},
            "note": "an empty kernel, and a kernel that reads algorithmic_bytes_per_launch once and "
                    "discards them, each in the multiply kernel's launch geometry: what one launch per "
                    "product costs on this protocol before any arithmetic",
        }
        log("warm leg")
        ms_w = timed(warm)
        result["warm"] = {"matvec_per_s": args.steps / (ms_w * 1e-3),
                          "us_per_step": ms_w * 1e3 / args.steps,
                          "note": "single weight set, Infinity-Cache resident: not an HBM figure"}
        # what independent products gain when two launch chains may overlap (not the metric:
        # a batch-1 decode is one dependent chain)
        two = None
        if args.steps >= 8 * nsets and not args.no_two_chains:
            log("two launch chains")
            ms_2 = median(time_graphs(torch, cold, args.steps, args.warmup, nsets, lanes=2))
            two = {"rsr_us_per_step": ms_2 * 1e3 / args.steps}
        # dense packed-2-bit comparison kernel, same protocol
        log("dense comparison kernel")
        dsets = int(np.ceil(COLD_WORKING_SET / dense_equiv_bytes))
        for hh in handles[1:]:
            rsr.rsr_destroy(hh)
        handles[:] = [h0]
        dh = [rsr.rsr_preprocess(torch.from_numpy(M0).to(dev), 0, rsr.RSR_DENSE_TERNARY_P2)]
        for i in range(1, dsets):
            Mi = gen.ternary_matrix(rows, cols, gen.LLM_8B_P_ZERO, gen.BASE_SEED + 1000 + i)
            dh.append(rsr.rsr_preprocess(torch.from_numpy(Mi).to(dev), 0, rsr.RSR_DENSE_TERNARY_P2))
            del Mi
        douts = torch.zeros((dsets, rows), dtype=torch.float32, device=dev)
        gd = rsr.rsr_matvec_ex(dh[0], v).cpu().numpy()
        derr = float(np.max(np.abs(gd - want)))

        def dcold(i, s):
            j = i % dsets
            rsr.rsr_matvec_ex(dh[j], v, out=douts[j], stream=s)

        def dwarm(i, s):
            rsr.rsr_matvec_ex(dh[0], v, out=douts[0], stream=s)

        ms_d = timed(dcold, period=dsets)
        ms_dw = timed(dwarm)
        dbytes = rsr.rsr_algorithmic_bytes(dh[0], rsr.RSR_BF16, 1)
        result["dense_packed2"] = {
            "matvec_per_s": args.steps / (ms_d * 1e-3), "us_per_step": ms_d * 1e3 / args.steps,
            "GBs": dbytes / (ms_d * 1e-3 / args.steps) / 1e9,
            "warm_us_per_step": ms_dw * 1e3 / args.steps,
            "weight_sets": dsets, "max_abs_err_vs_f64": derr,
            "kernel": rsr.rsr_kernel_name(dh[0], rsr.RSR_BF16),
            "algorithmic_bytes_per_launch": dbytes,
            "frac_hbm_peak": dbytes / (ms_d * 1e-3 / args.steps) / 1e9 / HBM_PEAK_GBS,
            # 16x16x32 bf16 MFMA steps: every matrix entry times the 16 B columns, 2 flops
            "mfma_TFLOPs": rows * cols * 16 * 2 / (ms_d * 1e-3 / args.steps) / 1e12,
            "frac_mfma_bf16_peak": rows * cols * 16 * 2 / (ms_d * 1e-3 / args.steps) / 2.5e15,
        }
        result["speedup_vs_dense_packed2"] = ms_d / ms
        if two is not None:
            two["dense_us_per_step"] = median(time_graphs(torch, dcold, args.steps, args.warmup, dsets,
                                                          lanes=2)) * 1e3 / args.steps
            two["note"] = ("the same cold launches dealt alternately to two streams of one graph, so that "
                           "the start-up of one launch overlaps the end of the other: throughput of "
                           "independent products, reported beside the metric and not part of it")
            result["two_launch_chains"] = two

    if not args.no_cpu_baseline:
        # the oracle as it stands (plain C, float64), on the host cores: the dense definition on
        # one thread, then the same routine on row slices from one thread per core (the C call
        # releases the interpreter lock), about 10 s each; and the oracle's own RSR multiply
        from concurrent.futures import ThreadPoolExecutor
        log("oracle on the host cores")
        v64 = vals.astype(np.float64)
        t0 = time.time()
        n1 = 0
        while time.time() - t0 < 8.0:
            oracle.dense_matvec(M0, v64)
            n1 += 1
        dt1 = time.time() - t0
        cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
        cores = max(1, min(cores, int(os.environ.get("OMP_NUM_THREADS", cores))))
        bounds = np.linspace(0, rows, cores + 1).astype(int)
        slices = [np.ascontiguousarray(M0[bounds[i]:bounds[i + 1]]) for i in range(cores)]
        with ThreadPoolExecutor(max_workers=cores) as pool_:
            t0 = time.time()
            nall = 0
            while time.time() - t0 < 8.0:
                list(pool_.map(lambda Ms: oracle.dense_matvec(Ms, v64), slices))
                nall += 1
            dtall = time.time() - t0
        art = oracle.preprocess(M0, args.k, oracle.TERNARY_FUSED if args.kind == "fused"
                                else oracle.TERNARY_2PASS)
        t1 = time.time()
        n2 = 0
        while time.time() - t1 < 4.0:
            oracle.matvec(art, v64)
            n2 += 1
        dt2 = time.time() - t1
        result["cpu_baseline"] = {
            "value": nall / dtall, "unit": "matvec/s", "cores": cores, "kind": "oracle",
            "single_thread_value": n1 / dt1,
            "sample": "%d full 4096x14336 matvecs by the definition (oracle dense, float64) on %d threads "
                      "(row slices) in %.1f s; one thread: %d in %.1f s; oracle RSR multiply, one thread: "
                      "%.2f matvec/s; host reports %d cpus"
                      % (nall, cores, dtall, n1, dt1, n2 / dt2, os.cpu_count() or 0),
        }

    if args.traffic_probe:
        src = torch.ones(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()

    print(json.dumps(result))


if __name__ == "__main__":
    main()

#!/usr/bin/env python3
"""Benchmark of the Slim-DP communication-set path on one MI355X.

A step is one full reselect iteration of the hot path on the VGG-16-sized flat model
(138,357,544 binary32 parameters, W = 8 logical workers, core 10 %, explorer 2 % of the
rest): score -> select core -> sample W explorers -> pack W workers -> merge.  Inputs are
seeded synthetic vectors already resident in HBM when the timed region starts.

Prints ONE JSON line: whole-job throughput in Gparam/s (n / step time), the roofline of the
dominant kernel measured with events on the library's stream, per-stage times, the same
iteration in other states (first iteration of a fresh context, library options untouched,
other update vectors every step), and the CPU oracle timed on a bounded sample of the same
workload.

``--workload vgg16_loop20`` times the 20-iteration loop instead (a step = the whole loop:
fresh updates for every (iteration, worker), resident in HBM before the clock starts; core
reselected every 5 iterations, explorer every iteration).
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X published HBM3E bandwidth
STAGES = ["score", "select_core", "sample_explore", "pack", "merge"]
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "vgg16_flat_W8_hbm_traffic_pmc.txt")


def stage_bytes(n: int, W: int, k: int, m: int) -> dict:
    """Algorithmic bytes of every stage (stream model: a sorted gather at >= 10 % density
    touches nearly every line, so extracting from an update vector costs reading it)."""
    return {
        "score": 4 * n * (1 + W) + 4 * n,
        "select_core": 2 * 4 * n + 4 * k + n // 8,
        "sample_explore": W * (n // 8 + 4 * m),
        "pack": W * (4 * n + n // 8 + 4 * m + 4 * (k + m)),
        "merge": 4 * n + 4 * n + 4 * W * (k + m) + 4 * k + 4 * W * m,
    }


def measured_traffic(kernel: str):
    """HBM bytes per launch of `kernel` as the committed counter summary states them (a line
    'traffic_bytes_per_launch <kernel>: <bytes>'), or None.  Counters are read under rocprofv3, never in
    this process."""
    try:
        text = open(TRAFFIC_FILE).read()
    except OSError:
        return None
    m = re.search(r"^traffic_bytes_per_launch\s+" + re.escape(kernel) + r"\s*:\s*([0-9.eE+]+)", text, flags=re.M)
    return float(m.group(1)) if m else None


def cpu_baseline(sample_n: int, all_cores: bool) -> dict:
    """The oracle as it stands, one iteration on a bounded sample: one thread; with all_cores the same calls
    spread over the host cores where the units are independent (workers)."""
    import oracle
    from paper_1709_09393_amd import workloads
    wl = workloads.VGG16.scaled(sample_n)
    w = wl.weights()
    g = wl.gradients(0)
    k, m = wl.k, wl.m
    oracle.lib()

    def note(what, t0):      # progress of a long CPU leg, from the work itself
        if sample_n >= 50_000_000:
            print("cpu_baseline: %s done at %.1f s" % (what, time.perf_counter() - t0), file=sys.stderr, flush=True)

    def one(pool):
        mp = (lambda f, xs: list(pool.map(f, xs))) if pool else (lambda f, xs: [f(x) for x in xs])
        t0 = time.perf_counter()
        S = oracle.score(w, g, wl.c)
        note("score", t0)
        core = oracle.select_core(S, k)
        note("core selection", t0)

        def explore(q):
            r = oracle.sample_explore(wl.n, core, workloads.EXPLORE_SEED, 0, q, m)
            note("explorer of worker %d" % q, t0)
            return r
        ei = mp(explore, range(wl.W))
        packs = mp(lambda q: oracle.pack(g[q], core, ei[q]), range(wl.W))
        note("packs", t0)
        oracle.merge(w, wl.lr, core, [p[0] for p in packs], ei, [p[1] for p in packs])
        dt = time.perf_counter() - t0
        note("merge", t0)
        return dt

    dt = one(None)
    out = {"value": wl.n / dt / 1e9, "unit": "Gparam/s", "cores": 1, "kind": "oracle",
           "sample": "one full iteration of the same recipe at n=%d, W=%d (k=%d, m=%d), %.2f s" % (wl.n, wl.W, k, m, dt)}
    if all_cores:
        from concurrent.futures import ThreadPoolExecutor
        nproc = os.cpu_count() or 1
        threads = min(wl.W, nproc)
        with ThreadPoolExecutor(threads) as pool:        # the C calls release the interpreter lock
            dt2 = one(pool)
        out["all_cores"] = {"value": wl.n / dt2 / 1e9, "unit": "Gparam/s", "nproc": nproc, "threads_used": threads,
                            "what": "same calls, the W explorer rankings and packs on %d threads (the two global "
                                    "passes and the core ranking stay on one), %.2f s" % (threads, dt2)}
    return out


class Buffers:
    """Device buffers of one model: outputs of every stage, allocated once."""

    def __init__(self, torch, sd, n, W, k, m, dev):
        i32, f32 = torch.int32, torch.float32
        self.S = torch.empty(n, dtype=f32, device=dev)
        self.core_idx = torch.empty(k, dtype=i32, device=dev)
        self.core_bits = torch.empty((n + 31) // 32, dtype=i32, device=dev)
        self.core_off = torch.empty(sd.T + 1, dtype=i32, device=dev)
        self.expl_idx = [torch.empty(m, dtype=i32, device=dev) for _ in range(W)]
        self.expl_off = [torch.empty(sd.T + 1, dtype=i32, device=dev) for _ in range(W)]
        self.expl_idx2 = [torch.empty(m, dtype=i32, device=dev) for _ in range(W)]      # a request one iteration ahead
        self.expl_off2 = [torch.empty(sd.T + 1, dtype=i32, device=dev) for _ in range(W)]
        self.core_val = [torch.empty(k, dtype=f32, device=dev) for _ in range(W)]
        self.expl_val = [torch.empty(m, dtype=f32, device=dev) for _ in range(W)]


def reselect_step(sd, wl, b, w, g, ks, ms, t, ev=None, as_scored=True, announce=True):
    """score -> select -> explorers -> pack -> merge; ev: six events around the five stages."""
    def mark(j):
        if ev is not None:
            ev[j].record()
    W = len(g)
    mark(0)
    sd.score(w, g, wl.c, out=b.S)
    mark(1)
    _, _, _, epoch = sd.select_core(b.S, ks, reuse_histogram=True, core_idx=b.core_idx, core_bits=b.core_bits,
                                    core_off=b.core_off)
    mark(2)
    sd.sample_explore(b.core_bits, ks, t, ms, 0, W, expl_idx=b.expl_idx, expl_off=b.expl_off)
    if announce:       # the next iteration's random draw (integer work only) rides inside the next scoring pass
        sd.explore_hint(ks, t + 1, ms, 0, W)
    mark(3)
    sd.pack(g, b.core_idx, b.core_off, b.expl_idx, b.expl_off, epoch, core_val=b.core_val, expl_val=b.expl_val,
            updates_as_scored=as_scored)
    mark(4)
    sd.merge(w, wl.lr, epoch, b.core_idx, b.core_off, b.core_val, b.expl_idx, b.expl_off, b.expl_val)
    mark(5)
    return epoch


def device_updates(torch, wl, workloads, t, dev):
    """Fresh update vectors of iteration t with the workload's distribution, drawn on the device (bench only: the
    parity tests use the host recipe that the oracle sees too)."""
    out = []
    for q in range(wl.W):
        gen = torch.Generator(device=dev)
        gen.manual_seed(workloads.gradient_seed(t, q))
        x = torch.empty(wl.n, dtype=torch.float32, device=dev)
        x.normal_(0.0, wl.grad_sigma, generator=gen)
        if wl.grad_fp16:
            x = x.to(torch.float16).to(torch.float32)
        out.append(x)
    return out


def run_loop(torch, sd, wl, b, w, g_all, ks, ms):
    """The multi-iteration loop: core every reselect_every iterations from the current model and that iteration's
    updates, explorer every iteration, every draw announced one iteration ahead (inside the scoring pass of a
    reselecting iteration, otherwise on the library's side stream).  While the core stays, the explorer request of
    the next iteration is issued before this iteration's pack (two sets of list arrays) and runs beside pack and merge."""
    epoch = None
    W = wl.W
    lists = [(b.expl_idx, b.expl_off), (b.expl_idx2, b.expl_off2)]
    ahead = False
    for t in range(wl.iterations):
        g = g_all[t]
        resel = t % wl.reselect_every == 0
        ei, eo = lists[t & 1]
        if resel:
            sd.score(w, g, wl.c, out=b.S)
            _, _, _, epoch = sd.select_core(b.S, ks, reuse_histogram=True, core_idx=b.core_idx, core_bits=b.core_bits,
                                            core_off=b.core_off)
        if not ahead:
            sd.sample_explore(b.core_bits, ks, t, ms, 0, W, expl_idx=ei, expl_off=eo)
        next_resel = (t + 1) % wl.reselect_every == 0
        sd.set_option("explore_hint_mode", 0 if next_resel else 1)
        sd.explore_hint(ks, t + 1, ms, 0, W)
        ahead = not next_resel and t + 1 < wl.iterations
        if ahead:
            sd.sample_explore(b.core_bits, ks, t + 1, ms, 0, W, expl_idx=lists[(t + 1) & 1][0], expl_off=lists[(t + 1) & 1][1])
        sd.pack(g, b.core_idx, b.core_off, ei, eo, epoch, core_val=b.core_val, expl_val=b.expl_val,
                updates_as_scored=resel)
        sd.merge(w, wl.lr, epoch, b.core_idx, b.core_off, b.core_val, ei, eo, b.expl_val)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--n", type=int, default=0, help="override the parameter count (profiling runs)")
    ap.add_argument("--cpu-sample", type=int, default=16_000_000, help="oracle sample size; 0 skips the CPU leg")
    ap.add_argument("--cpu-full", action="store_true",
                    help="time the oracle once at the workload's full size instead of a sample (minutes)")
    ap.add_argument("--workload", default="vgg16_flat", help="another named configuration (not the headline): "
                    "tiny, googlenet_seg57, tie_stress, vgg16_loop20 (a step = the whole 20-iteration loop)")
    ap.add_argument("--opt", action="append", default=[], help="library option name=value (tuning runs)")
    ap.add_argument("--no-variants", action="store_true", help="headline only (profiling runs)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain 1 GiB device copy (known traffic) so that hardware byte counters "
                         "read under rocprofv3 --pmc can be scaled")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (W logical workers share it); --gpus %d is not supported"
              % args.gpus, file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_1709_09393_amd import binding, workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    wl = workloads.BY_NAME[args.workload]
    if args.n:
        wl = wl.scaled(args.n)
    n, W, k, m = wl.n, wl.W, wl.k, wl.m
    ks, ms = [int(x) for x in wl.k_seg()], [int(x) for x in wl.m_seg()]
    seg_off = [int(x) for x in wl.segment_offsets()]

    def new_context(capture=True):
        c = binding.SlimDP(n, W, seg_off=seg_off, seed=workloads.EXPLORE_SEED)
        if capture:
            c.set_option("speculative_pack", 1)   # the scoring pass keeps the likely core's update values for the pack
            c.set_option("explore_async", 1)      # explorer requests on the library's side stream, beside the pack
        for kv in args.opt:
            name, value = kv.split("=")
            c.set_option(name, int(value))
        return c

    sd = new_context()
    w0 = torch.from_numpy(wl.weights()).to(dev)
    w = w0.clone()
    b = Buffers(torch, sd, n, W, k, m, dev)
    sb = stage_bytes(n, W, k, m)
    total_bytes = sum(sb.values())

    if args.copy_calibration:
        a = torch.empty(1 << 28, dtype=torch.float32, device=dev).fill_(1.0)       # 1 GiB
        c = torch.empty_like(a)
        c.copy_(a)                                                                # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del a, c

    def timed(fn, reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for r in range(reps):
            fn(r)
        e1.record()
        torch.cuda.synchronize()
        sd.synchronize()
        return e0.elapsed_time(e1) / reps

    # ------------------------------------------------------------------------------------------------------
    if wl.iterations > 1:
        # the loop: all updates of all iterations resident before the clock starts
        g_all = [device_updates(torch, wl, workloads, t, dev) for t in range(wl.iterations)]
        torch.cuda.synchronize()
        for _ in range(max(1, args.warmup)):
            sd.explore_hint(ks, 0, ms, 0, W)
            run_loop(torch, sd, wl, b, w, g_all, ks, ms)
        sd.synchronize()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            sd.explore_hint(ks, 0, ms, 0, W)
            run_loop(torch, sd, wl, b, w, g_all, ks, ms)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        sd.synchronize()
        ms_per_step = (t1 - t0) * 1e3 / args.steps
        n_resel = (wl.iterations + wl.reselect_every - 1) // wl.reselect_every
        steady_bytes = sb["sample_explore"] + sb["pack"] + sb["merge"]
        loop_bytes = n_resel * total_bytes + (wl.iterations - n_resel) * steady_bytes
        out = {
            "metric": "Gparam/s score+select+pack+merge, % of HBM peak GB/s, 138M params, W=8",
            "value": n * wl.iterations / (ms_per_step * 1e-3) / 1e9, "unit": "Gparam/s", "n_gpus": 1,
            "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
            "config": {"workload": wl.name, "n": n, "W": W, "k": k, "m": m, "iterations": wl.iterations,
                       "reselect_every": wl.reselect_every, "updates": "fresh per (iteration, worker), drawn on the device"},
            "ms_per_iteration": ms_per_step / wl.iterations,
            "algorithmic_bytes_per_step": loop_bytes,
            "hbm_frac_whole_step": loop_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS,
            "roofline": None, "cpu_baseline": None,
        }
        sd.close()
        print(json.dumps(out))
        return 0

    # ------------------------------------------------------------------------------------------------------
    g = [torch.from_numpy(wl.gradient(0, q)).to(dev) for q in range(W)]
    sd.explore_hint(ks, 0, ms, 0, W)
    for t in range(args.warmup):
        reselect_step(sd, wl, b, w, g, ks, ms, t)
    sd.synchronize()

    events = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(args.steps):
        reselect_step(sd, wl, b, w, g, ks, ms, args.warmup + t, events[t])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    sd.synchronize()

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    stage_ms = {s: float(np.mean([events[t][j].elapsed_time(events[t][j + 1]) for t in range(args.steps)]))
                for j, s in enumerate(STAGES)}
    value = n / (ms_per_step * 1e-3) / 1e9

    # dominant kernel: k_score (one launch per step: reads w and the W updates, writes the score)
    score_gbs = sb["score"] / (stage_ms["score"] * 1e-3) / 1e9
    traffic = measured_traffic("k_score") if (not args.n and wl.name == "vgg16_flat") else None
    roofline = {"bound": "hbm", "kernel": "k_score", "achieved": score_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": score_gbs / HBM_PEAK_GBS, "traffic": traffic,
                "algorithmic_bytes_per_launch": sb["score"], "avg_launch_ms": stage_ms["score"]}

    def frac(bytes_, ms_):
        return bytes_ / (ms_ * 1e-3) / 1e9 / HBM_PEAK_GBS

    out = {
        "metric": "Gparam/s score+select+pack+merge, % of HBM peak GB/s, 138M params, W=8",
        "value": value, "unit": "Gparam/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": wl.name, "n": n, "W": W, "k": k, "m": m, "core_pct": wl.core_pct,
                   "explore_pct": wl.explore_pct, "c": wl.c, "lr": wl.lr, "tile": binding.TILE,
                   "state": "steady: options speculative_pack and explore_async on, every draw announced one step ahead, "
                            "the same update vectors every step"},
        "hbm_frac_whole_step": frac(total_bytes, ms_per_step),
        "algorithmic_bytes_per_step": total_bytes,
        "stage_ms": stage_ms,
        "stage_hbm_frac": {s: frac(sb[s], stage_ms[s]) for s in STAGES},
        "roofline": roofline,
    }
    reps = max(3, min(args.steps, 10))
    if not args.no_variants:
        # (1) other update vectors every step (two sets alternate): the capture bound comes from a selection on
        # different updates, as in a training loop
        g2 = [torch.from_numpy(wl.gradient(1, q)).to(dev) for q in range(W)]
        sets = [g, g2]
        sd.explore_hint(ks, 5000, ms, 0, W)
        reselect_step(sd, wl, b, w, sets[1], ks, ms, 5000)
        fresh_ms = timed(lambda r: reselect_step(sd, wl, b, w, sets[r & 1], ks, ms, 5001 + r), reps)
        out["fresh_updates_ms"] = fresh_ms
        out["fresh_updates_hbm_frac"] = frac(total_bytes, fresh_ms)
        del g2, sets
        # (2) the pack without the flag (it scans the update vectors), everything else as in the headline
        sd.explore_hint(ks, 6000, ms, 0, W)
        reselect_step(sd, wl, b, w, g, ks, ms, 6000, as_scored=False)
        scan_ms = timed(lambda r: reselect_step(sd, wl, b, w, g, ks, ms, 6001 + r, as_scored=False), reps)
        out["scanning_pack_ms"] = scan_ms
        out["scanning_pack_hbm_frac"] = frac(total_bytes, scan_ms)
        # (3) the iteration before a reselection as algorithm 1 has it (every worker pushes its whole update; dense
        # update, significance of the new model and selection: no pack, no sparse merge)
        def dense(_r):
            sd.dense_update_score(w, g, wl.lr, wl.c, out=b.S)
            sd.select_core(b.S, ks, reuse_histogram=True, core_idx=b.core_idx, core_bits=b.core_bits, core_off=b.core_off)
        dense(0)
        dense_ms = timed(dense, reps)
        out["paper_schedule_reselect"] = {"ms": dense_ms, "Gparam_per_s": n / (dense_ms * 1e-3) / 1e9,
                                          "what": "slimdp_dense_update_score + slimdp_select_core",
                                          "algorithmic_bytes": 4 * n * (W + 3) + 4 * n + 4 * k + n // 8}
        # (4) the steady iteration between two reselections (cached core keys, updates no scoring pass has seen:
        # explorers, pack by scanning the updates, merge); the next iteration's draw and explorer request run on the side
        # stream beside this iteration's pack and merge
        sd.set_option("explore_hint_mode", 1)
        _, _, _, epoch2 = sd.select_core(b.S, ks, core_idx=b.core_idx, core_bits=b.core_bits, core_off=b.core_off)
        lists = [(b.expl_idx, b.expl_off), (b.expl_idx2, b.expl_off2)]
        sd.explore_hint(ks, 10_000, ms, 0, W)
        sd.sample_explore(b.core_bits, ks, 10_000, ms, 0, W, expl_idx=lists[0][0], expl_off=lists[0][1])

        def steady(r):
            ei, eo = lists[r & 1]
            sd.explore_hint(ks, 10_001 + r, ms, 0, W)                       # next draw and next request: the side stream
            sd.sample_explore(b.core_bits, ks, 10_001 + r, ms, 0, W, expl_idx=lists[(r + 1) & 1][0], expl_off=lists[(r + 1) & 1][1])
            sd.pack(g, b.core_idx, b.core_off, ei, eo, epoch2, core_val=b.core_val, expl_val=b.expl_val)
            sd.merge(w, wl.lr, epoch2, b.core_idx, b.core_off, b.core_val, ei, eo, b.expl_val)
        steady_ms = timed(steady, reps)
        steady_bytes = sb["sample_explore"] + sb["pack"] + sb["merge"]
        out["steady_iteration"] = {"ms": steady_ms, "Gparam_per_s": n / (steady_ms * 1e-3) / 1e9,
                                   "what": "slimdp_sample_explore + slimdp_pack + slimdp_merge, core keys cached",
                                   "algorithmic_bytes": steady_bytes, "hbm_frac": frac(steady_bytes, steady_ms)}
        # (4b) the rest of the loop around the path: pull with local overwrite (section 3.3 steps 4, 5), one local
        # mini-batch step of all W workers with update accumulation (step 1), and the 8-bit wire codec (section 4.2)
        sd.set_option("explore_hint_mode", 0)
        w_local = [w0.clone() for _ in range(W)]
        delta = [torch.empty_like(w0) for _ in range(W)]
        sd.local_step(w_local, g, delta, 0.01, first=True)
        ls_ms = timed(lambda r: sd.local_step(w_local, g, delta, 0.01, first=False), reps)
        # the last local step before a push with the extraction in the same pass, against the two calls it replaces
        lsp_ms = timed(lambda r: sd.local_step_pack(w_local, g, delta, 0.01, False, b.core_idx, b.core_off, b.expl_idx,
                                                    b.expl_off, epoch2, core_val=b.core_val, expl_val=b.expl_val), reps)
        pk_ms = timed(lambda r: sd.pack(delta, b.core_idx, b.core_off, b.expl_idx, b.expl_off, epoch2, core_val=b.core_val,
                                        expl_val=b.expl_val), reps)
        pull_ms = timed(lambda r: sd.pull(w, epoch2, b.core_idx, b.core_off, b.expl_idx, b.expl_off, w_local=w_local,
                                          core_out=b.core_val, expl_out=b.expl_val), reps)
        # pull, local merge and the first local step of the next round in one pass, against the two calls it replaces
        pls_ms = timed(lambda r: sd.pull_local_step(w, epoch2, b.core_idx, b.core_off, b.expl_idx, b.expl_off, w_local, g,
                                                    delta, 0.01, first=True), reps)
        ls1_ms = timed(lambda r: sd.local_step(w_local, g, delta, 0.01, first=True), reps)
        del w_local, delta
        codes = sd.quantize(b.core_val, 0, 0)
        codes_e = sd.quantize(b.expl_val, 1, 0)

        def quant(_r):
            sd.quantize(b.core_val, 0, _r, code=codes[0], scale=codes[1])
            sd.quantize(b.expl_val, 1, _r, code=codes_e[0], scale=codes_e[1])

        def dequant(_r):
            sd.dequantize(codes[0], codes[1], out=b.core_val)
            sd.dequantize(codes_e[0], codes_e[1], out=b.expl_val)
        q_ms = timed(quant, reps)
        dq_ms = timed(dequant, reps)
        nvals = W * (k + m)
        out["worker_side"] = {
            "local_step": {"ms": ls_ms, "algorithmic_bytes": 20 * n * W, "hbm_frac": frac(20 * n * W, ls_ms)},
            "local_step_and_pack_in_one_pass": {"ms": lsp_ms, "two_calls_ms": ls_ms + pk_ms,
                                                "algorithmic_bytes": 20 * n * W + sb["pack"] - 4 * n * W,
                                                "hbm_frac": frac(20 * n * W + sb["pack"] - 4 * n * W, lsp_ms)},
            "pull_with_local_overwrite": {"ms": pull_ms},
            "pull_and_first_local_step_in_one_pass": {"ms": pls_ms, "two_calls_ms": pull_ms + ls1_ms,
                                                      "algorithmic_bytes": 16 * n * W + 4 * n,
                                                      "hbm_frac": frac(16 * n * W + 4 * n, pls_ms)},
            "quantize": {"ms": q_ms, "algorithmic_bytes": 5 * nvals, "hbm_frac": frac(5 * nvals, q_ms)},
            "dequantize": {"ms": dq_ms, "algorithmic_bytes": 5 * nvals, "hbm_frac": frac(5 * nvals, dq_ms)},
            "wire_bytes_per_worker": {"plain": binding.wire_bytes(k, m, False), "quantized": binding.wire_bytes(k, m, True),
                                      "dense": 4 * n},
        }
        del codes, codes_e
    sd.close()
    if not args.no_variants:
        # (5) the very first iteration of a fresh context: no selection before it (its draw is announced: that needs
        # nothing but the sizes)
        cold = []
        for _ in range(3):
            c = new_context()
            w.copy_(w0)
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            c.explore_hint(ks, 0, ms, 0, W)
            e0.record()
            reselect_step(c, wl, b, w, g, ks, ms, 0, announce=False)
            e1.record()
            torch.cuda.synchronize()
            c.synchronize()
            cold.append(e0.elapsed_time(e1))
            c.close()
        out["cold_iteration_ms"] = float(np.mean(cold))
        out["cold_iteration_hbm_frac"] = frac(total_bytes, out["cold_iteration_ms"])
        # (6) library options untouched (no capture in the scoring pass; the pack scans), draws still announced
        c = new_context(capture=False)
        c.explore_hint(ks, 0, ms, 0, W)
        for t in range(2):
            reselect_step(c, wl, b, w, g, ks, ms, t, as_scored=False)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for t in range(reps):
            reselect_step(c, wl, b, w, g, ks, ms, 2 + t, as_scored=False)
        e1.record()
        torch.cuda.synchronize()
        c.synchronize()
        out["default_options_ms"] = e0.elapsed_time(e1) / reps
        out["default_options_hbm_frac"] = frac(total_bytes, out["default_options_ms"])
        c.close()
    del w, g, b
    if args.cpu_full:
        out["cpu_baseline"] = cpu_baseline(n, all_cores=True)
    elif args.cpu_sample > 0:
        out["cpu_baseline"] = cpu_baseline(args.cpu_sample, all_cores=True)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())

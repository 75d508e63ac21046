#!/usr/bin/env python3
"""Benchmark of the fused Marsit one-bit synchronisation pass on one MI355X.

A step = one pass of the whole hot path (compensate, sign, the M-1 merges of every part's chain,
decode, global compensation) over one batch of synthetic gradients of all M simulated workers; it
is one call of a whole-pass entry point of the C ABI (one kernel launch for whole packed words).
Inputs are resident in HBM before the timed region starts.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload resnet50]

The default run is the headline: marsit_ring_step_sim on the resnet50 workload (M = 8,
d = 25.6 M, ring).  The switches --entry, --M, --d, --grid-x and --ld-pad time the other
whole-pass entry points, other worker counts and schedules (those without a compiled
specialisation run the any-schedule kernel) and rows that do not start on 128-byte lines;
they exist so that every figure quoted for those kernels comes from this file.
--split-workers is a probe of the memory system (the rows taken as separate synchronisations).
"""

from __future__ import annotations

import argparse
import dataclasses
import glob
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0      # MI355X HBM3E, vendor figure
# Integer vector peak for the kernels that only draw: 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz 32-bit
# lane operations per second; one Philox4x32-10 call compiles to 40 vector instructions (per round
# two 32 x 32 -> 64-bit multiply-adds and two three-input XORs), priced here at one issue slot each.
PHILOX_PEAK_CALLS_PER_S = 256 * 4 * 16 * 2.4e9 / 40

ENTRIES = ("ring_step_sim", "tree_step_sim", "ragged_torus_step_sim", "full_sync", "step_apply")


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="resnet50")
    ap.add_argument("--entry", default="ring_step_sim", choices=ENTRIES,
                    help="whole-pass entry point that is timed as the step (marsit_<entry>)")
    ap.add_argument("--M", type=int, default=0, help="override the workload's worker count")
    ap.add_argument("--d", type=int, default=0, help="override the workload's elements per gradient")
    ap.add_argument("--grid-x", type=int, default=-1, help="override the workload's torus columns (0: ring)")
    ap.add_argument("--ld-pad", type=int, default=0, help="row stride = d + this many elements")
    ap.add_argument("--fused-waves", type=int, default=0,
                    help="force this many one-wavefront workgroups per CU for the compiled fused kernels "
                         "(tuning hook marsit_set_fused_waves_per_cu; 0: the library's choice)")
    ap.add_argument("--split-workers", type=int, default=1,
                    help="memory-system probe: take the M workers as this many separate synchronisations of "
                         "M / N workers each, one launch after the other over row blocks of the same arrays "
                         "(NOT the result of one synchronisation of M workers; ring_step_sim and full_sync only). "
                         "Shows what the pass would cost with only M / N workers' streams open at a time")
    ap.add_argument("--per-launch-events", action="store_true",
                    help="record a HIP event after every timed step (per-launch min / median / max in the JSON) "
                         "instead of only before the first and after the last one; the extra records cost "
                         "1-2 % of the step time, so they are off by default")
    ap.add_argument("--seed", type=int, default=2022)
    ap.add_argument("--pool", type=int, default=10,
                    help="distinct gradient sets kept in HBM and cycled through (0: one per step)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch one plain device copy of one gradient set (known size: reads and "
                         "writes 4*M*ld bytes), the yardstick for the rocprofv3 --pmc byte counters")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-unfused", action="store_true", help="skip timing the hop-by-hop chain")
    ap.add_argument("--no-aux", action="store_true", help="skip timing the other entry points")
    ap.add_argument("--cpu-threads", type=int, default=0)
    return ap.parse_args()


def algorithmic_bytes(entry: str, M: int, d: int) -> int:
    """Bytes the pass has to move: g and c read, c' written per worker; the update (or, for
    step_apply, the model read and written instead) once; the final packed bitmap."""
    n_words = (d + 63) // 64
    if entry == "full_sync":
        return 12 * M * d + 4 * d
    if entry == "step_apply":
        return 12 * M * d + 8 * d + 8 * n_words
    return 12 * M * d + 4 * d + 8 * n_words


def measured_traffic(key: str):
    """HBM bytes per launch from the rocprofv3 counter summaries under profiles/, or None when no
    summary covers this run or the summary was made from other kernel sources than the ones here."""
    from paper_2204_06787_amd import build as hip_build
    digest = hip_build.fused_sources_digest()
    for path in sorted(glob.glob(os.path.join(ROOT, "profiles", "*.txt"))):
        text = open(path).read()
        if not re.search(r"^key: " + re.escape(key) + r"\s*$", text, flags=re.M):
            continue
        sha = re.search(r"^fused_sources_sha16: (\w+)", text, flags=re.M)
        val = re.search(r"^traffic_bytes_per_launch: (\d+)", text, flags=re.M)
        if sha and val and sha.group(1) == digest:
            return int(val.group(1)), os.path.relpath(path, ROOT)
        return None, f"{os.path.relpath(path, ROOT)} describes other kernel sources than this tree's"
    return None, "no counter summary under profiles/ for this configuration"


def cpu_baseline(wl, g_host, seed, threads):
    """The oracle, as it stands, on the host cores: full steps of the same workload."""
    import numpy as np
    from oracle import marsit_oracle as orc
    c_host = np.zeros_like(g_host)
    n_steps = max(1, min(wl.steps, 10))         # about 12 s on 16 cores at the headline size
    t0 = time.perf_counter()
    for t in range(n_steps):                    # the same gradients again, compensation carried over
        orc.sync_step(g_host, c_host, wl.scale, seed + t, grid_x=wl.grid_x, threads=threads)
    dt = (time.perf_counter() - t0) / n_steps
    gbps = wl.algorithmic_bytes() / dt / 1e9
    # the same on one thread, on the first 1/8 of the columns
    d8 = max(64, (wl.d // 8) // 64 * 64)
    g8 = np.ascontiguousarray(g_host[:, :d8])
    c8 = np.zeros_like(g8)
    t0 = time.perf_counter()
    orc.sync_step(g8, c8, wl.scale, seed, grid_x=wl.grid_x, threads=1)
    dt1 = time.perf_counter() - t0
    bytes8 = 12 * wl.M * d8 + 4 * d8 + d8 // 8
    cpu_model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    cpu_model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    return {
        "value": gbps, "unit": "GB/s", "cores": threads, "kind": "oracle",
        "sample": f"{n_steps} full steps of {wl.name} (M={wl.M}, d={wl.d}) on {threads} OpenMP threads",
        "seconds": dt * n_steps, "seconds_per_step": dt, "worker_elements_per_s": wl.M * wl.d / dt,
        "cpu_model": cpu_model, "host_cores_visible": os.cpu_count(),
        "single_thread": {"value": bytes8 / dt1 / 1e9, "unit": "GB/s", "seconds": dt1,
                          "sample": f"1 step on the first {d8} columns"},
    }


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build simulates the M workers inside ONE GPU; there is no multi-GPU "
              "path to time (--gpus must be 1).", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2204_06787_amd import marsit, workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    marsit.load_library()          # raises if the HIP library has not been built
    torch.cuda.set_device(0)
    # One 256-element call now, so that the runtime loads the library's code object for this device
    # here and not at the first warm-up step: that load takes milliseconds, the GPU would sit idle
    # between the input generation and the steps, and the device's clock transient after an idle
    # period would then fall into the timed region of a short run.
    probe = torch.zeros(256, dtype=torch.float32, device="cuda")
    marsit.marsit_apply_update(probe, probe.clone())
    torch.cuda.synchronize()
    del probe
    if args.fused_waves:
        marsit.marsit_set_fused_waves_per_cu(args.fused_waves)
    wl = workloads.WORKLOADS[args.workload]
    custom = {}
    if args.M > 0:
        custom["M"] = args.M
    if args.d > 0:
        custom["d"] = args.d
    if args.grid_x >= 0:
        custom["grid_x"] = args.grid_x
    if custom:
        wl = dataclasses.replace(wl, name=wl.name + "+" + ",".join(f"{k}={v}" for k, v in custom.items()), **custom)
    entry = args.entry
    if entry == "tree_step_sim" and wl.grid_x:
        wl = dataclasses.replace(wl, grid_x=0)
    M, d, ld = wl.M, wl.d, wl.d + args.ld_pad
    headline = (entry == "ring_step_sim" and not custom and args.ld_pad == 0 and not args.fused_waves
                and args.split_workers == 1)
    split = args.split_workers
    if split != 1 and (split < 1 or M % split or wl.grid_x or entry not in ("ring_step_sim", "full_sync")):
        print("bench.py: --split-workers must divide M and goes with a ring or the full-precision round", file=sys.stderr)
        sys.exit(2)
    K, Wm = args.steps, args.warmup
    total = K + Wm
    pool = args.pool if args.pool > 0 else total
    pool = max(1, min(pool, total, int(64e9 // (4 * M * ld))))

    # inputs: resident in HBM before anything is timed
    grads = [workloads.make_gradients(wl, t, args.seed, device="cuda", ld=ld) for t in range(pool)]
    c = workloads.zero_compensation(wl, device="cuda", ld=ld)
    update = torch.empty(d, dtype=torch.float32, device="cuda")
    bits = marsit.new_bitmap(d)
    x_model = torch.zeros(d, dtype=torch.float32, device="cuda") if entry == "step_apply" else None
    stream = torch.cuda.current_stream()

    def step(t):
        g, seed = grads[t % pool], workloads.step_seed(args.seed, t)
        if split > 1:
            rows = M // split
            for k in range(split):
                gk, ck = g[k * rows:(k + 1) * rows], c[k * rows:(k + 1) * rows]
                if entry == "ring_step_sim":
                    marsit.marsit_ring_step_sim(gk, ck, update, bits, wl.scale, seed, d=d, stream=stream)
                else:
                    marsit.marsit_full_sync(gk, ck, update, d=d, stream=stream)
        elif entry == "ring_step_sim":
            marsit.marsit_ring_step_sim(g, c, update, bits, wl.scale, seed, grid_x=wl.grid_x, d=d, stream=stream)
        elif entry == "tree_step_sim":
            marsit.marsit_tree_step_sim(g, c, update, bits, wl.scale, seed, d=d, stream=stream)
        elif entry == "ragged_torus_step_sim":
            marsit.marsit_ragged_torus_step_sim(g, c, update, bits, wl.scale, seed, wl.grid_x or M, d=d, stream=stream)
        elif entry == "full_sync":
            marsit.marsit_full_sync(g, c, update, d=d, stream=stream)
        else:   # one round of Algorithm 2 in one pass, one-bit branch (t = 1, K = 2), update not written
            marsit.marsit_step_apply(1, 2, g, c, x_model, None, bits, wl.scale, seed, grid_x=wl.grid_x, d=d,
                                     stream=stream)

    if args.copy_calibration:
        scratch = torch.empty_like(grads[0])
        scratch.copy_(grads[0])
        torch.cuda.synchronize()
        del scratch

    for t in range(Wm):
        step(t)
    torch.cuda.synchronize()

    # HIP events on the stream the kernels are launched on: one before the first timed step and one
    # after the last (or one after every step with --per-launch-events)
    every = 1 if args.per_launch_events else K
    events = [torch.cuda.Event(enable_timing=True) for _ in range(K // every + 1)]
    t0 = time.perf_counter()
    events[0].record(stream)
    for i in range(K):
        step(Wm + i)
        if (i + 1) % every == 0:
            events[(i + 1) // every].record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    per_launch_ms = [events[i].elapsed_time(events[i + 1]) / every for i in range(K // every)]
    avg_kernel_ms = sum(per_launch_ms) / len(per_launch_ms)
    ms_per_step = wall * 1e3 / K
    nbytes = algorithmic_bytes(entry, M, d) if split == 1 else split * algorithmic_bytes(entry, M // split, d)
    value = nbytes / (ms_per_step * 1e-3) / 1e9
    achieved = nbytes / (avg_kernel_ms * 1e-3) / 1e9
    schedule = "tree" if entry == "tree_step_sim" else ("ring" if not wl.grid_x or wl.grid_x == M else
                                                        f"torus {wl.grid_x} columns x {-(-M // wl.grid_x)} rows")
    key = f"entry={entry} M={M} d={d} grid_x={wl.grid_x} ld_pad={args.ld_pad}" + (
        f" fused_waves={args.fused_waves}" if args.fused_waves else "") + (
        f" split_workers={split}" if split > 1 else "")
    traffic, traffic_source = measured_traffic(key)

    out = {
        "metric": "fused Marsit sync pass GB/s (algorithmic bytes / time)",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{wl.name}: M={M} simulated workers, d={d} fp32, {schedule}, "
                               f"{wl.dist} gradients, compensation carried over steps, one seed per step",
                   "entry_point": "marsit_" + entry, "M": M, "d": d, "ld": ld, "grid_x": wl.grid_x,
                   "scale": wl.scale, "gradient_sets_in_hbm": pool,
                   **({"fused_waves_per_cu": args.fused_waves} if args.fused_waves else {}),
                   **({"split_workers": split, "note": "probe: separate synchronisations of M / split workers each, "
                       "launches_timed counts steps of `split` launches"} if split > 1 else {})},
        "worker_elements_per_s": M * d / (ms_per_step * 1e-3),
        "elements_per_s": d / (ms_per_step * 1e-3),
        "algorithmic_bytes_per_step": nbytes,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": traffic, "traffic_source": traffic_source,
                     "kernel": "sync_step_kernel" if headline else f"the kernel marsit_{entry} launches for this shape",
                     "avg_launch_ms": avg_kernel_ms, "launches_timed": K,
                     "events": "one per launch" if args.per_launch_events else "first and last"},
    }
    if args.per_launch_events:
        out["roofline"].update(median_launch_ms=sorted(per_launch_ms)[K // 2], min_launch_ms=min(per_launch_ms),
                               max_launch_ms=max(per_launch_ms))

    if not args.no_unfused and entry == "ring_step_sim":
        # what the fusion buys: the same pass hop by hop (M compress, M(M-1) hop merges, M decodes)
        ws = torch.empty(marsit.marsit_chain_workspace_words(M, d, wl.grid_x), dtype=torch.int64,
                         device="cuda")
        c2 = workloads.zero_compensation(wl, device="cuda", ld=ld)

        def chain(t):
            marsit.marsit_chain_step_sim(grads[t % pool], c2, update, bits, ws, wl.scale,
                                         workloads.step_seed(args.seed, t), grid_x=wl.grid_x, d=d, stream=stream)
        for t in range(2):
            chain(t)
        torch.cuda.synchronize()
        n_chain = 5
        t0 = time.perf_counter()
        for t in range(n_chain):
            chain(2 + t)
        torch.cuda.synchronize()
        chain_ms = (time.perf_counter() - t0) * 1e3 / n_chain

        def replayed_ms(call):
            """The step recorded once into a HIP graph; ms per replay (no host code between launches)."""
            try:
                graph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(graph):
                    call(torch.cuda.current_stream())
                for _ in range(2):
                    graph.replay()
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(n_chain):
                    graph.replay()
                torch.cuda.synchronize()
                return (time.perf_counter() - t0) * 1e3 / n_chain
            except Exception as exc:        # an extra figure must not cost the line
                return f"not measured: {type(exc).__name__}: {exc}"[:200]

        out["unfused_chain"] = {"ms_per_step": chain_ms, "value": nbytes / (chain_ms * 1e-3) / 1e9,
                                "unit": "GB/s (same algorithmic bytes)", "steps": n_chain,
                                "launches_per_step": 2 * M + M * (M - 1) + M,
                                "ms_per_step_in_a_graph": replayed_ms(lambda st: marsit.marsit_chain_step_sim(
                                    grads[0], c2, update, bits, ws, wl.scale, workloads.step_seed(args.seed, 0),
                                    grid_x=wl.grid_x, d=d, stream=st))}

        # the same pass as ONE exchange step: M compress, one fold per part, M decodes
        def exchange(t):
            marsit.marsit_exchange_step_sim(grads[t % pool], c2, update, bits, ws, wl.scale,
                                            workloads.step_seed(args.seed, t), grid_x=wl.grid_x, d=d, stream=stream)
        for t in range(2):
            exchange(t)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for t in range(n_chain):
            exchange(2 + t)
        torch.cuda.synchronize()
        ex_ms = (time.perf_counter() - t0) * 1e3 / n_chain
        Xb = wl.grid_x or M
        out["unfused_exchange_step"] = {
            "ms_per_step": ex_ms, "value": nbytes / (ex_ms * 1e-3) / 1e9,
            "unit": "GB/s (same algorithmic bytes)", "steps": n_chain,
            "launches_per_step": 2 * M + M + (M if M // Xb > 1 else 0),
            "ms_per_step_in_a_graph": replayed_ms(lambda st: marsit.marsit_exchange_step_sim(
                grads[0], c2, update, bits, ws, wl.scale, workloads.step_seed(args.seed, 0), grid_x=wl.grid_x, d=d,
                stream=st))}
        del ws, c2

    if not args.no_aux and entry == "ring_step_sim" and args.ld_pad == 0:
        try:
            out["other_entry_points"] = other_entry_points(torch, marsit, workloads, wl, grads, update, bits,
                                                           stream, args.seed, nbytes)
        except Exception as exc:            # the headline figures above stand on their own
            out["other_entry_points"] = {"error": f"{type(exc).__name__}: {exc}"[:300]}

    if not args.no_cpu_baseline and entry == "ring_step_sim":
        threads = args.cpu_threads or min(16, os.cpu_count() or 1)
        g_host = grads[0][:, :d].contiguous().cpu().numpy()
        out["cpu_baseline"] = cpu_baseline(wl, g_host, workloads.step_seed(args.seed, 0), threads)
    print(json.dumps(out))


def other_entry_points(torch, marsit, workloads, wl, grads, update, bits, stream, seed0, nbytes):
    """The other entry points on the same workload, each timed with events.

    Per-worker kernels work on one worker's vectors (102 MB each at the headline size), which the
    256 MB memory-side cache would hold from one launch to the next.  They are therefore timed
    over a ROTATION of buffers: launch i takes worker i mod M of gradient set (i / M) mod pool, and
    the model and update vectors rotate over M copies, so every launch finds its operands in HBM
    (more than 1.5 GB goes through between two uses of a buffer) -- "cache_resident": false."""
    M, d, pool = wl.M, wl.d, len(grads)

    def timed(fn, reps=10, warm=2):
        for i in range(warm):
            fn(i)
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ev0.record(stream)
        for i in range(reps):
            fn(warm + i)
        ev1.record(stream)
        torch.cuda.synchronize()
        return ev0.elapsed_time(ev1) / reps

    def graph_us_per_launch(fn, n=40, replays=10):
        """fn(i, stream) recorded n times into one HIP graph; microseconds per launch over replays of it
        (what a hop costs when no host code runs between the launches)."""
        try:
            graph = torch.cuda.CUDAGraph()
            fn(0, stream)                                   # first use outside the capture
            torch.cuda.synchronize()
            with torch.cuda.graph(graph):
                for i in range(n):
                    fn(i, torch.cuda.current_stream())
            for _ in range(3):
                graph.replay()
            ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            ev0.record(stream)
            for _ in range(replays):
                graph.replay()
            ev1.record(stream)
            torch.cuda.synchronize()
            return ev0.elapsed_time(ev1) * 1e3 / (replays * n)
        except Exception as exc:            # an extra figure must not cost the line
            return f"not measured: {type(exc).__name__}: {exc}"[:200]

    def entry(ms, nb, **extra):
        e = {"ms": ms, "GB/s": nb / (ms * 1e-3) / 1e9, "frac_of_hbm_peak": nb / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
             "algorithmic_bytes": nb}
        e.update(extra)
        return e

    c3 = workloads.zero_compensation(wl, device="cuda")
    x = torch.zeros(d, dtype=torch.float32, device="cuda")
    one_bits = marsit.new_bitmap(d)
    aux = {}
    # the whole-pass kernels get the same long warm-up as the headline
    aux["marsit_full_sync"] = entry(timed(lambda i: marsit.marsit_full_sync(grads[i % pool], c3, update, stream=stream),
                                          reps=20, warm=25), 12 * M * d + 4 * d)
    # one round of Algorithm 2 in one pass (one-bit branch: t = 1, K = 2): model read and written in the fused kernel
    aux["marsit_step_apply"] = entry(timed(lambda i: marsit.marsit_step_apply(
        1, 2, grads[i % pool], c3, x, None, one_bits, wl.scale, seed0 + i, grid_x=wl.grid_x, stream=stream),
        reps=20, warm=25), 12 * M * d + 8 * d + d // 8)
    c3.zero_()
    aux["marsit_tree_step_sim"] = entry(timed(lambda i: marsit.marsit_tree_step_sim(
        grads[i % pool], c3, update, one_bits, wl.scale, seed0 + i, stream=stream), reps=20, warm=25), nbytes)
    c3.zero_()
    scaled = torch.empty_like(c3)
    aux["marsit_local_momentum"] = entry(timed(lambda i: marsit.marsit_local_momentum(
        c3, grads[i % pool], scaled, 0.5, 0.1, stream=stream)), 16 * M * d)
    c3.zero_()
    mom2 = torch.zeros_like(c3)
    aux["marsit_local_adam"] = entry(timed(lambda i: marsit.marsit_local_adam(
        c3, mom2, grads[i % pool], scaled, 0.9, 0.999, 1e-8, 0.1, 1.0 - 0.9 ** (i + 1), 1.0 - 0.999 ** (i + 1),
        stream=stream)), 24 * M * d)
    del mom2
    c3.zero_()

    # ---- per-worker kernels, operands rotated so that none is cache resident ----
    xs = scaled                                    # reuse as M model vectors
    xs.zero_()
    upds = torch.empty((M, d), dtype=torch.float32, device="cuda")
    maps = torch.empty((M, marsit.n_words(d)), dtype=torch.int64, device="cuda")
    for m in range(M):
        marsit.marsit_compress(grads[0][m], None, maps[m], stream=stream)      # valid bitmaps to decode

    def row(i):
        return grads[(i // M) % pool][i % M], i % M
    rot = {"cache_resident": False, "operands": f"rotating over {M} workers x {pool} gradient sets"}
    reps, warm = 4 * M, M

    def f_compress(i):
        g, m = row(i)
        marsit.marsit_compress(g, c3[m], maps[m], stream=stream)
    aux["marsit_compress"] = entry(timed(f_compress, reps, warm), 8 * d + d // 8, **rot)

    def f_decode(i):
        g, m = row(i)
        marsit.marsit_decode_compensate(maps[m], g, c3[m], wl.scale, upds[m], c3[m], stream=stream)
    aux["marsit_decode_compensate"] = entry(timed(f_decode, reps, warm), 16 * d + d // 8, **rot)
    c3.zero_()

    def f_decode_apply(i):
        g, m = row(i)
        marsit.marsit_decode_compensate_apply(maps[m], g, c3[m], wl.scale, xs[m], None, c3[m], stream=stream)
    aux["marsit_decode_compensate_apply"] = entry(timed(f_decode_apply, reps, warm), 20 * d + d // 8, **rot)
    c3.zero_()

    def f_apply(i):
        m = i % M
        marsit.marsit_apply_update(xs[m], upds[m], stream=stream)
    aux["marsit_apply_update"] = entry(timed(f_apply, reps, warm), 12 * d, **rot)

    # one ring hop of a worker: its signs of one part folded into the received segment
    W = marsit.n_words(d)
    seg = W // M
    n_part = seg * 64
    recv = torch.zeros((M, seg), dtype=torch.int64, device="cuda")

    def f_chm(i):
        g, m = row(i)
        lo = (i % M) * n_part
        marsit.marsit_compress_hop_merge(recv[m], g[lo:lo + n_part], c3[m][lo:lo + n_part], recv[m],
                                         (i % M) * seg, 3, 2, seed0, stream=stream)
    aux["marsit_compress_hop_merge"] = entry(timed(f_chm, reps, warm), 8 * n_part + 16 * seg, **rot)
    aux["marsit_compress_hop_merge"]["note"] = (
        f"one part of {n_part} elements ({8 * seg} B message) per launch: launch-bound at this size")

    def g_chm(i, st):
        g, m = row(i)
        lo = (i % M) * n_part
        marsit.marsit_compress_hop_merge(recv[m], g[lo:lo + n_part], c3[m][lo:lo + n_part], recv[m],
                                         (i % M) * seg, 3, 2, seed0, stream=st)
    aux["marsit_compress_hop_merge"]["us_per_launch_in_a_graph"] = graph_us_per_launch(g_chm)

    # the same kernel over a whole vector (fold of a whole bitmap), where HBM is the bound
    full_recv = torch.zeros((M, W), dtype=torch.int64, device="cuda")

    def f_chm_full(i):
        g, m = row(i)
        marsit.marsit_compress_hop_merge(full_recv[m], g, c3[m], full_recv[m], 0, 3, 2, seed0, stream=stream)
    aux["marsit_compress_hop_merge_whole_vector"] = entry(timed(f_chm_full, reps, warm), 8 * d + 16 * W, **rot)

    # merges on packed words only: 16 Philox calls per packed word per hop and 24 bytes moved
    aux["marsit_hop_merge"] = entry(timed(lambda i: marsit.marsit_hop_merge(
        recv[i % M], maps[i % M][:seg], recv[i % M], 0, seg, 3, 2, seed0, stream=stream)), 24 * seg)
    aux["marsit_hop_merge"].update(
        us_per_launch_in_a_graph=graph_us_per_launch(lambda i, st: marsit.marsit_hop_merge(
            recv[i % M], maps[i % M][:seg], recv[i % M], 0, seg, 3, 2, seed0, stream=st)),
        note=f"one part of {seg} packed words ({8 * seg} B message): launch-bound",
        bound="launch latency at this size; integer ALU (Philox) on large inputs, see the whole-bitmap rows")
    whole = torch.empty(W, dtype=torch.int64, device="cuda")
    ms = timed(lambda i: marsit.marsit_hop_merge(maps[i % M], maps[(i + 1) % M], whole, 0, W, 3, 2, seed0,
                                                 stream=stream), reps=20, warm=4)
    aux["marsit_hop_merge_whole_bitmap"] = entry(ms, 24 * W, bound="alu", philox_calls=16 * W,
                                                 philox_calls_per_s=16 * W / (ms * 1e-3),
                                                 alu_peak_calls_per_s=PHILOX_PEAK_CALLS_PER_S,
                                                 frac_of_alu_peak=16 * W / (ms * 1e-3) / PHILOX_PEAK_CALLS_PER_S,
                                                 note="operands are 3.2 MB bitmaps: cache resident by nature")
    ms = timed(lambda i: marsit.marsit_fold_segments(maps, M, i % M, whole, 0, W, 0, seed0 + i, stream=stream),
               reps=20, warm=4)
    aux["marsit_fold_segments_whole_bitmap"] = entry(ms, 8 * (M + 1) * W, bound="alu", philox_calls=16 * (M - 1) * W,
                                                     philox_calls_per_s=16 * (M - 1) * W / (ms * 1e-3),
                                                     alu_peak_calls_per_s=PHILOX_PEAK_CALLS_PER_S,
                                                     frac_of_alu_peak=16 * (M - 1) * W / (ms * 1e-3) / PHILOX_PEAK_CALLS_PER_S,
                                                     note=f"the {M - 1}-hop chain of all {W} words in one launch")
    del full_recv, recv, whole, upds, maps

    # the schedule as M workers on M streams, hop by hop (what a transport would sequence)
    X = wl.grid_x or M
    Y = M // X
    with marsit.RingPipeline(M) as pipe:
        wsp = torch.empty(pipe.workspace_words(d, wl.grid_x), dtype=torch.int64, device="cuda")
        ms = timed(lambda i: pipe.step(grads[i % pool], c3, update, one_bits, wsp, wl.scale, seed0 + i,
                                       grid_x=wl.grid_x, stream=stream), reps=5)
        torch.cuda.synchronize()
    aux["marsit_pipeline_step"] = {
        "ms_per_step": ms, "streams": M,
        "launches_per_step": M + M * (X - 1) + M * (Y - 1) + M,
        "hop_steps": X + (Y - 1) + 1,
        "note": f"1 compress+send step, {X - 1} row hops (sign step fused into the merge), {Y - 1} column hops, 1 decode step; "
                f"row segments of {8 * ((d // 64) // X)} B"}

    # context, not product: PyTorch's own elementwise kernels on arrays of one gradient set's size
    # (rows of the same tensors, so nothing new is allocated but the output)
    if pool >= 2:
        a_flat, b_flat = grads[0].view(-1), grads[1].view(-1)
        out_flat = c3.view(-1)
        n = out_flat.numel()
        ms_add = timed(lambda i: torch.add(a_flat, b_flat, out=out_flat))
        ms_copy = timed(lambda i: out_flat.copy_(a_flat if i % 2 else b_flat))
        aux["context_torch_elementwise"] = {
            "note": "PyTorch's library kernels on the same box, for scale; not part of the path",
            "add_2_reads_1_write": entry(ms_add, 12 * n), "copy_1_read_1_write": entry(ms_copy, 8 * n)}
    return aux


if __name__ == "__main__":
    main()

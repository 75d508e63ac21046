#!/usr/bin/env python3
"""Benchmark of the fused Marsit one-bit synchronisation pass on one MI355X.

A step = one pass of the whole hot path (compensate, sign, the M-1 merges of every part's chain,
decode, global compensation) over one batch of synthetic gradients of all M simulated workers; it
is one launch of the fused kernel through the C ABI.  Inputs are resident in HBM before the timed
region starts.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload resnet50]
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

HBM_PEAK_GBPS = 8000.0      # MI355X HBM3E, vendor figure

# HBM traffic of one launch of the fused kernel in bytes, from rocprofv3 --pmc FETCH_SIZE and
# WRITE_SIZE runs scaled by a copy kernel of known size (figures and commands: profiles/).
# None where no counter run has been made for that workload.
MEASURED_TRAFFIC_BYTES = {
    "resnet50": 2_563_238_687,   # profiles/sync_step_kernel_resnet50_hbm_traffic.txt
    "torus4x4": 5_020_856_830,   # profiles/sync_step_kernel_torus4x4_hbm_traffic.txt
}


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="resnet50")
    ap.add_argument("--seed", type=int, default=2022)
    ap.add_argument("--pool", type=int, default=10,
                    help="distinct gradient sets kept in HBM and cycled through (0: one per step)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch one plain device copy of one gradient set (known size: reads and "
                         "writes 4*M*d bytes), the yardstick for the rocprofv3 --pmc byte counters")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-unfused", action="store_true", help="skip timing the hop-by-hop chain")
    ap.add_argument("--no-aux", action="store_true", help="skip timing the other entry points")
    ap.add_argument("--cpu-threads", type=int, default=0)
    return ap.parse_args()


def cpu_baseline(wl, g_host, seed, threads):
    """The oracle, as it stands, on the host cores: one full step of the same workload."""
    import numpy as np
    from oracle import marsit_oracle as orc
    c_host = np.zeros_like(g_host)
    n_steps = max(1, min(wl.steps, 8))          # about 10 s on 16 cores at the headline size
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
    wl = workloads.WORKLOADS[args.workload]
    K, Wm = args.steps, args.warmup
    total = K + Wm
    pool = args.pool if args.pool > 0 else total
    pool = max(1, min(pool, total, int(64e9 // (4 * wl.M * wl.d))))

    # inputs: resident in HBM before anything is timed
    grads = [workloads.make_gradients(wl, t, args.seed, device="cuda") for t in range(pool)]
    c = workloads.zero_compensation(wl, device="cuda")
    update = torch.empty(wl.d, dtype=torch.float32, device="cuda")
    bits = marsit.new_bitmap(wl.d)
    stream = torch.cuda.current_stream()

    def step(t):
        marsit.marsit_ring_step_sim(grads[t % pool], c, update, bits, wl.scale,
                                    workloads.step_seed(args.seed, t), grid_x=wl.grid_x,
                                    stream=stream)

    if args.copy_calibration:
        scratch = torch.empty_like(grads[0])
        scratch.copy_(grads[0])
        torch.cuda.synchronize()
        del scratch

    for t in range(Wm):
        step(t)
    torch.cuda.synchronize()

    events = [torch.cuda.Event(enable_timing=True) for _ in range(K + 1)]
    t0 = time.perf_counter()
    events[0].record(stream)
    for i in range(K):
        step(Wm + i)
        events[i + 1].record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    per_launch_ms = [events[i].elapsed_time(events[i + 1]) for i in range(K)]
    avg_kernel_ms = sum(per_launch_ms) / K
    ms_per_step = wall * 1e3 / K
    nbytes = wl.algorithmic_bytes()
    value = nbytes / (ms_per_step * 1e-3) / 1e9
    achieved = nbytes / (avg_kernel_ms * 1e-3) / 1e9

    out = {
        "metric": "fused Marsit sync pass GB/s (algorithmic bytes / time)",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": K, "warmup": Wm,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"{wl.name}: M={wl.M} simulated workers, d={wl.d} fp32, "
                               f"{'ring' if not wl.grid_x else f'torus {wl.grid_x}x{wl.M // wl.grid_x}'}, "
                               f"{wl.dist} gradients, compensation carried over steps, one seed per step",
                   "M": wl.M, "d": wl.d, "grid_x": wl.grid_x, "scale": wl.scale,
                   "gradient_sets_in_hbm": pool},
        "worker_elements_per_s": wl.M * wl.d / (ms_per_step * 1e-3),
        "elements_per_s": wl.d / (ms_per_step * 1e-3),
        "algorithmic_bytes_per_step": nbytes,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS,
                     "traffic": MEASURED_TRAFFIC_BYTES.get(wl.name),
                     "kernel": "sync_step_kernel", "avg_launch_ms": avg_kernel_ms,
                     "median_launch_ms": sorted(per_launch_ms)[K // 2],
                     "min_launch_ms": min(per_launch_ms), "max_launch_ms": max(per_launch_ms)},
    }

    if not args.no_unfused:
        # what the fusion buys: the same pass hop by hop (M compress, M(M-1) hop merges, M decodes)
        ws = torch.empty(marsit.marsit_chain_workspace_words(wl.M, wl.d, wl.grid_x), dtype=torch.int64,
                         device="cuda")
        c2 = workloads.zero_compensation(wl, device="cuda")

        def chain(t):
            marsit.marsit_chain_step_sim(grads[t % pool], c2, update, bits, ws, wl.scale,
                                         workloads.step_seed(args.seed, t), grid_x=wl.grid_x, stream=stream)
        for t in range(2):
            chain(t)
        torch.cuda.synchronize()
        n_chain = 5
        t0 = time.perf_counter()
        for t in range(n_chain):
            chain(2 + t)
        torch.cuda.synchronize()
        chain_ms = (time.perf_counter() - t0) * 1e3 / n_chain
        out["unfused_chain"] = {"ms_per_step": chain_ms, "value": nbytes / (chain_ms * 1e-3) / 1e9,
                                "unit": "GB/s (same algorithmic bytes)", "steps": n_chain,
                                "launches_per_step": 2 * wl.M + wl.M * (wl.M - 1) + wl.M}

        # the same pass as ONE exchange step: M compress, one fold per part, M decodes
        def exchange(t):
            marsit.marsit_exchange_step_sim(grads[t % pool], c2, update, bits, ws, wl.scale,
                                            workloads.step_seed(args.seed, t), grid_x=wl.grid_x, stream=stream)
        for t in range(2):
            exchange(t)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for t in range(n_chain):
            exchange(2 + t)
        torch.cuda.synchronize()
        ex_ms = (time.perf_counter() - t0) * 1e3 / n_chain
        Xb = wl.grid_x or wl.M
        out["unfused_exchange_step"] = {
            "ms_per_step": ex_ms, "value": nbytes / (ex_ms * 1e-3) / 1e9,
            "unit": "GB/s (same algorithmic bytes)", "steps": n_chain,
            "launches_per_step": 2 * wl.M + wl.M + (wl.M if wl.M // Xb > 1 else 0)}
        del ws, c2

    if not args.no_aux:
        # the other entry points on the same workload, each timed with events over 10 launches
        def timed(fn, reps=10, warm=2):
            for _ in range(warm):
                fn()
            ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            ev0.record(stream)
            for _ in range(reps):
                fn()
            ev1.record(stream)
            torch.cuda.synchronize()
            return ev0.elapsed_time(ev1) / reps

        def entry(ms, nb):
            return {"ms": ms, "GB/s": nb / (ms * 1e-3) / 1e9, "frac_of_hbm_peak": nb / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                    "algorithmic_bytes": nb}
        M, d = wl.M, wl.d
        c3 = workloads.zero_compensation(wl, device="cuda")
        x = torch.zeros(d, dtype=torch.float32, device="cuda")
        one_bits = marsit.new_bitmap(d)
        aux = {}
        # the two whole-pass kernels get the same long warm-up as the headline (the device runs the
        # first ~25 launches of a burst 5-8 % slower)
        aux["marsit_full_sync"] = entry(timed(lambda: marsit.marsit_full_sync(grads[0], c3, update, stream=stream),
                                              reps=20, warm=25), 12 * M * d + 4 * d)
        # one round of Algorithm 2 in one pass (one-bit branch: t = 1, K = 2): model read and written in the fused kernel
        aux["marsit_step_apply"] = entry(timed(lambda: marsit.marsit_step_apply(
            1, 2, grads[0], c3, x, None, one_bits, wl.scale, args.seed, grid_x=wl.grid_x, stream=stream),
            reps=20, warm=25), 12 * M * d + 8 * d + d // 8)
        c3.zero_()
        aux["marsit_apply_update"] = entry(timed(lambda: marsit.marsit_apply_update(x, update, stream=stream)), 12 * d)
        scaled = torch.empty_like(c3)
        aux["marsit_local_momentum"] = entry(timed(lambda: marsit.marsit_local_momentum(
            c3, grads[0], scaled, 0.5, 0.1, stream=stream)), 16 * M * d)
        c3.zero_()
        del scaled
        aux["marsit_compress"] = entry(timed(lambda: marsit.marsit_compress(grads[0][0], c3[0], one_bits, stream=stream)),
                                       8 * d + d // 8)
        aux["marsit_decode_compensate"] = entry(timed(lambda: marsit.marsit_decode_compensate(
            one_bits, grads[0][0], c3[0], wl.scale, update, c3[0], stream=stream)), 16 * d + d // 8)
        aux["marsit_decode_compensate_apply"] = entry(timed(lambda: marsit.marsit_decode_compensate_apply(
            one_bits, grads[0][0], c3[0], wl.scale, x, None, c3[0], stream=stream)), 20 * d + d // 8)
        seg = (d // 64) // M
        aux["marsit_hop_merge"] = entry(timed(lambda: marsit.marsit_hop_merge(
            one_bits[:seg], bits[:seg], one_bits[:seg], 0, seg, 3, 2, args.seed, stream=stream)), 24 * seg)
        aux["marsit_hop_merge"]["note"] = f"one part of {seg} packed words ({8 * seg} B message); ALU-bound by design"
        aux["marsit_tree_step_sim"] = entry(timed(lambda: marsit.marsit_tree_step_sim(
            grads[0], c3, update, one_bits, wl.scale, args.seed, stream=stream), reps=20, warm=25), nbytes)
        # the schedule as M workers on M streams, hop by hop (what a transport would sequence)
        X = wl.grid_x or M
        Y = M // X
        with marsit.RingPipeline(M) as pipe:
            wsp = torch.empty(pipe.workspace_words(d, wl.grid_x), dtype=torch.int64, device="cuda")
            ms = timed(lambda: pipe.step(grads[0], c3, update, one_bits, wsp, wl.scale, args.seed,
                                         grid_x=wl.grid_x, stream=stream), reps=5)
            torch.cuda.synchronize()
        aux["marsit_pipeline_step"] = {
            "ms_per_step": ms, "streams": M,
            "launches_per_step": M + M * (X - 1) + M * (Y - 1) + M,
            "hop_steps": X + (Y - 1) + 1,
            "note": f"1 compress+send step, {X - 1} row hops (sign step fused into the merge), {Y - 1} column hops, 1 decode step; "
                    f"row segments of {8 * ((d // 64) // X)} B"}
        del wsp
        out["other_entry_points"] = aux
        del c3, x, one_bits

    if not args.no_cpu_baseline:
        threads = args.cpu_threads or min(16, os.cpu_count() or 1)
        g_host = grads[0].cpu().numpy()
        out["cpu_baseline"] = cpu_baseline(wl, g_host, workloads.step_seed(args.seed, 0), threads)
    print(json.dumps(out))


if __name__ == "__main__":
    main()

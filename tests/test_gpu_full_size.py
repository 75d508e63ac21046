"""Parity at the full sizes of the five workloads, in the launch configuration bench.py times
(same entry point, same buffers layout, consecutive steps with compensation carried over).

The oracle runs on all host cores (its loop over packed words is counter-based, so threads do not
change results); every output element is compared, not a sample.
"""

import os

import numpy as np
import pytest
import torch

from oracle import marsit_oracle as orc
from paper_2204_06787_amd import marsit, workloads
from gpu_util import assert_f32_parity, host_bits, host_f32

pytestmark = pytest.mark.gpu

THREADS = min(16, os.cpu_count() or 1)


@pytest.mark.parametrize("name", ["resnet18", "resnet50", "torus4x4", "large"])
def test_full_size_workload(name):
    """Every workload as stated: 10 / 10 / 5 / 3 consecutive steps, compensation carried over, a
    fresh seed and fresh gradients per step, every output element of every step compared."""
    wl = workloads.WORKLOADS[name]
    steps = wl.steps
    print(f"full-size parity: {name} M={wl.M} d={wl.d} grid_x={wl.grid_x} steps={steps}", flush=True)
    c = workloads.zero_compensation(wl, device="cuda")
    update = torch.empty(wl.d, dtype=torch.float32, device="cuda")
    bits = marsit.new_bitmap(wl.d)
    c_h = np.zeros((wl.M, wl.d), dtype=np.float32)
    for t in range(steps):
        g = workloads.make_gradients(wl, t, seed=2022, device="cuda")
        seed = workloads.step_seed(2022, t)
        marsit.marsit_ring_step_sim(g, c, update, bits, wl.scale, seed, grid_x=wl.grid_x)
        torch.cuda.synchronize()
        g_h = host_f32(g)
        del g
        want_u, want_b, _ = orc.sync_step(g_h, c_h, wl.scale, seed, grid_x=wl.grid_x, threads=THREADS)
        del g_h
        assert np.array_equal(host_bits(bits), want_b), f"{name}: merged bitmap, step {t}"
        assert np.array_equal(host_f32(update).view(np.uint32), want_u.view(np.uint32)), f"{name}: update, step {t}"
        del want_u, want_b
        got_c = host_f32(c)
        assert_f32_parity(got_c, c_h, f"{name}: compensation, step {t}")
        del got_c
        # a property that holds at any size: the update is +-scale everywhere
        assert bool((update.abs() == np.float32(wl.scale)).all())
        print(f"  step {t} ok", flush=True)


def test_workload_generators_have_the_stated_statistics():
    """The synthetic gradients are what the recipe says (so the timed inputs are the stated ones)."""
    wl = workloads.WORKLOADS["resnet18"]
    g = workloads.make_gradients(wl, 0, seed=5, device="cuda", d=2_000_000)
    assert abs(float(g.std()) - 0.1) < 2e-3 and abs(float(g.mean())) < 1e-3
    wl = workloads.WORKLOADS["resnet50"]
    g = workloads.make_gradients(wl, 0, seed=5, device="cuda", d=1_600_000)
    stds = workloads.layer_stds(wl, 5)
    assert float(stds.min()) >= 1e-4 * 0.999 and float(stds.max()) <= 1e-1 * 1.001
    per_layer = g[0].view(workloads.N_LAYERS, -1).std(dim=1).cpu()
    assert torch.allclose(per_layer, stds, rtol=0.05)
    wl = workloads.WORKLOADS["large"]
    g = workloads.make_gradients(wl, 0, seed=5, device="cuda", d=4_000_000)
    frac_big = float((g.abs() > 1.0).float().mean())          # only the Student-t part reaches |x| > 10 sigma
    assert 1e-5 < frac_big < 5e-4


def _rand_rows(M, d, seed, std=0.1):
    gen = torch.Generator(device="cuda").manual_seed(seed)
    g = torch.empty((M, d), dtype=torch.float32, device="cuda")
    for m in range(M):
        g[m].normal_(mean=0.0, std=std, generator=gen)
    return g


@pytest.mark.parametrize("entry,M,grid_x,d", [
    ("tree", 8, 0, 25_600_000),            # tree_step_kernel<8>, the size bench.py --entry tree_step_sim times
    ("ragged", 13, 4, 12_800_000 + 37),    # staged kernel, short last row, ragged last word
    ("ring", 32, 0, 6_400_000 + 5),        # staged kernel, batches of 8
    ("ring", 64, 0, 3_200_000 + 63),       # gather-and-sweep kernel
    ("torus", 24, 6, 8_000_000),           # staged kernel, 6 x 4 torus
])
def test_other_kernels_at_large_sizes(entry, M, grid_x, d):
    """The kernels behind bench.py's --entry / --M / --grid-x switches at sizes that run for
    thousands of workgroups per CU: two consecutive steps with the compensation carried over,
    every output element compared."""
    print(f"large-size parity: {entry} M={M} grid_x={grid_x} d={d}", flush=True)
    scale = 1e-3
    c = torch.zeros((M, d), dtype=torch.float32, device="cuda")
    c_h = np.zeros((M, d), dtype=np.float32)
    update = torch.empty(d, dtype=torch.float32, device="cuda")
    bits = marsit.new_bitmap(d)
    for t in range(2):
        g = _rand_rows(M, d, seed=1000 * M + t)
        seed = workloads.step_seed(77, t)
        if entry == "tree":
            marsit.marsit_tree_step_sim(g, c, update, bits, scale, seed)
        elif entry == "ragged":
            marsit.marsit_ragged_torus_step_sim(g, c, update, bits, scale, seed, grid_x)
        else:
            marsit.marsit_ring_step_sim(g, c, update, bits, scale, seed, grid_x=grid_x)
        torch.cuda.synchronize()
        g_h = host_f32(g)
        del g
        if entry == "tree":
            want_u, want_b = orc.tree_step(g_h, c_h, scale, seed)
        elif entry == "ragged":
            want_u, want_b = orc.ragged_torus_step(g_h, c_h, scale, seed, grid_x, threads=THREADS)
        else:
            want_u, want_b, _ = orc.sync_step(g_h, c_h, scale, seed, grid_x=grid_x, threads=THREADS)
        del g_h
        assert np.array_equal(host_bits(bits), want_b), f"merged bitmap, step {t}"
        assert np.array_equal(host_f32(update).view(np.uint32), want_u.view(np.uint32)), f"update, step {t}"
        assert_f32_parity(host_f32(c), c_h, f"compensation, step {t}")


def test_round_of_algorithm_2_at_the_headline_size():
    """marsit_round at M = 8, d = 25.6 M with the model update in the same pass: one full-precision
    round (t = 0) and two one-bit rounds, model, update and compensation compared in full."""
    wl = workloads.WORKLOADS["resnet50"]
    M, d, K = wl.M, wl.d, 4
    x = torch.zeros(d, dtype=torch.float32, device="cuda")
    x_h = np.zeros(d, dtype=np.float32)
    c = torch.zeros((M, d), dtype=torch.float32, device="cuda")
    c_h = np.zeros((M, d), dtype=np.float32)
    update = torch.empty(d, dtype=torch.float32, device="cuda")
    bits = marsit.new_bitmap(d)
    for t in range(3):
        g = workloads.make_gradients(wl, t, seed=31, device="cuda")
        seed = workloads.step_seed(31, t)
        marsit.marsit_round(t, K, marsit.SCHEDULE_RING, 0, g, c, x, update, bits, wl.scale, seed)
        torch.cuda.synchronize()
        g_h = host_f32(g)
        del g
        if t % K == 0:
            want_u = orc.full_sync(g_h, c_h)
        else:
            want_u, want_b, _ = orc.sync_step(g_h, c_h, wl.scale, seed, threads=THREADS)
            assert np.array_equal(host_bits(bits), want_b), t
        del g_h
        x_h = orc.apply_update(x_h, want_u)
        assert np.array_equal(host_f32(update).view(np.uint32), want_u.view(np.uint32)), t
        assert np.array_equal(host_f32(x).view(np.uint32), x_h.view(np.uint32)), t
        assert_f32_parity(host_f32(c), c_h, f"compensation, round {t}")

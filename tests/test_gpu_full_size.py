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

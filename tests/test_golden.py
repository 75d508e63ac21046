"""Stored digests of the oracle's outputs (written by tests/golden/make_golden.py, which calls only
the oracle): the oracle must still produce them, and the HIP path must produce the same."""

import importlib.util
import json
import os

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
spec = importlib.util.spec_from_file_location("make_golden", os.path.join(HERE, "golden", "make_golden.py"))
make_golden = importlib.util.module_from_spec(spec)
spec.loader.exec_module(make_golden)

with open(os.path.join(HERE, "golden", "oracle_digests.json")) as fh:
    STORED = json.load(fh)


@pytest.mark.parametrize("case", make_golden.CASES, ids=[c[0] for c in make_golden.CASES])
def test_oracle_still_produces_the_stored_digests(case):
    name, M, d, gx, scale, seed, steps = case
    assert make_golden.run_case(M, d, gx, scale, seed, steps) == STORED[name]


@pytest.mark.gpu
@pytest.mark.parametrize("case", make_golden.CASES, ids=[c[0] for c in make_golden.CASES])
def test_hip_path_produces_the_stored_digests(case):
    import torch
    from paper_2204_06787_amd import marsit
    name, M, d, gx, scale, seed, steps = case
    c = torch.zeros((M, d), dtype=torch.float32, device="cuda")
    u = torch.empty(d, dtype=torch.float32, device="cuda")
    b = marsit.new_bitmap(d)
    for t in range(steps):
        g = torch.from_numpy(make_golden.inputs(M, d, t)).cuda()
        if gx < 0:
            marsit.marsit_tree_step_sim(g, c, u, b, scale, seed + t)
        else:
            marsit.marsit_ring_step_sim(g, c, u, b, scale, seed + t, grid_x=gx)
        torch.cuda.synchronize()
        got = {"bits": make_golden.digest(b.cpu().numpy().view(np.uint64)),
               "update": make_golden.digest(u.cpu().numpy()), "c": make_golden.digest(c.cpu().numpy())}
        assert got == STORED[name][t], (name, t)


@pytest.mark.parametrize("case", make_golden.EXTRA, ids=[c[0] for c in make_golden.EXTRA])
def test_oracle_still_produces_the_stored_digests_of_the_other_rounds(case):
    name, kind, M, d, param, steps = case
    assert make_golden.run_extra(kind, M, d, param, steps) == STORED[name]


@pytest.mark.gpu
@pytest.mark.parametrize("case", make_golden.EXTRA, ids=[c[0] for c in make_golden.EXTRA])
def test_hip_path_produces_the_stored_digests_of_the_other_rounds(case):
    import torch
    from paper_2204_06787_amd import marsit
    name, kind, M, d, param, steps = case
    c = torch.zeros((M, d), dtype=torch.float32, device="cuda")
    s1, s2 = torch.zeros_like(c), torch.zeros_like(c)
    u = torch.empty(d, dtype=torch.float32, device="cuda")
    b = marsit.new_bitmap(d)
    dig = make_golden.digest
    for t in range(steps):
        g = torch.from_numpy(make_golden.inputs(M, d, t)).cuda()
        if kind == "ragged":
            marsit.marsit_ragged_torus_step_sim(g, c, u, b, 1e-3, 31 + t, param)
            torch.cuda.synchronize()
            got = {"bits": dig(b.cpu().numpy().view(np.uint64)), "update": dig(u.cpu().numpy()), "c": dig(c.cpu().numpy())}
        elif kind == "full":
            c += torch.from_numpy(make_golden.inputs(M, d, 100 + t) * np.float32(0.25)).cuda()
            marsit.marsit_full_sync(g, c, u)
            torch.cuda.synchronize()
            got = {"update": dig(u.cpu().numpy()), "c": dig(c.cpu().numpy())}
        elif kind == "adam":
            step = torch.empty_like(g)
            marsit.marsit_local_adam(s1, s2, g, step, 0.9, 0.999, 1e-8, 0.01, 1.0 - 0.9 ** (t + 1), 1.0 - 0.999 ** (t + 1))
            torch.cuda.synchronize()
            got = {"step": dig(step.cpu().numpy()), "mom1": dig(s1.cpu().numpy()), "mom2": dig(s2.cpu().numpy())}
        else:
            step = torch.empty_like(g)
            marsit.marsit_local_momentum(s1, g, step, 0.9, 0.05)
            torch.cuda.synchronize()
            got = {"step": dig(step.cpu().numpy()), "buf": dig(s1.cpu().numpy())}
        assert got == STORED[name][t], (name, t)

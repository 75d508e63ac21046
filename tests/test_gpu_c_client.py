"""The C ABI used from a plain C program (no Python, no torch on its side): the client under
tests/helpers reads seeded inputs from a file, runs the fused pass on the GPU and writes its results;
they are compared with the oracle here."""

import os
import struct
import subprocess

import numpy as np
import pytest

from oracle import marsit_oracle as orc
from paper_2204_06787_amd import build as hip_build
from paper_2204_06787_amd import workloads

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("M,grid_x,d,ld", [(3, 0, 65_536, 65_536), (8, 0, 100_003, 100_004), (6, 3, 7001, 7001)])
def test_plain_c_client_matches_the_oracle(tmp_path, M, grid_x, d, ld):
    assert os.path.exists(hip_build.C_CLIENT), "run __graft_entry__.build() first: the C client is not built"
    steps, scale, seed0 = 2, 1e-3, 424242
    wl = workloads.Workload("c_client", M=M, d=d, grid_x=grid_x, steps=steps, scale=scale, dist="normal", std=0.1)
    grads = [workloads.make_gradients(wl, t, seed=9, device="cpu", d=d, ld=ld).numpy() for t in range(steps)]
    src, dst = tmp_path / "in.bin", tmp_path / "out.bin"
    with open(src, "wb") as f:
        f.write(struct.pack("<IIQQfIQ", M, grid_x, d, ld, scale, steps, seed0))
        for g in grads:
            f.write(np.ascontiguousarray(g, dtype=np.float32).tobytes())
    print(f"c client: M={M} grid_x={grid_x} d={d} ld={ld}", flush=True)
    proc = subprocess.run([hip_build.C_CLIENT, str(src), str(dst)], capture_output=True, text=True, timeout=100)
    assert proc.returncode == 0, proc.stdout + proc.stderr

    c_h = np.zeros((M, ld), dtype=np.float32)
    for t in range(steps):
        want_u, want_b, _ = orc.sync_step(grads[t].copy(), c_h, scale, seed0 + t, grid_x=grid_x, d=d)
    W = orc.n_words(d)
    raw = dst.read_bytes()
    assert len(raw) == 4 * d + 8 * W + 4 * M * ld
    got_u = np.frombuffer(raw, dtype=np.float32, count=d)
    got_b = np.frombuffer(raw, dtype=np.uint64, count=W, offset=4 * d)
    got_c = np.frombuffer(raw, dtype=np.float32, count=M * ld, offset=4 * d + 8 * W).reshape(M, ld)
    assert np.array_equal(got_b, want_b)
    assert np.array_equal(got_u.view(np.uint32), want_u.view(np.uint32))
    assert np.array_equal(got_c[:, :d].view(np.uint32), c_h[:, :d].view(np.uint32))
    assert not got_c[:, d:].any()                       # padding columns of c stay as the client left them (zero)

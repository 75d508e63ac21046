#!/usr/bin/env python3
"""Writes ``tests/golden/oracle_digests.json``: digests of what the CPU oracle computes for small,
machine-independent inputs.  Calls ONLY the oracle (never the HIP path).  The stored digests guard
against an unnoticed change of the oracle's arithmetic; the GPU tests compare the HIP path with the
same digests as well.

    python tests/golden/make_golden.py
"""

import hashlib
import json
import os
import sys

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, os.path.dirname(os.path.dirname(HERE)))

from oracle import marsit_oracle as orc   # noqa: E402

CASES = [
    # name, M, d, grid_x (0: ring, -1: tree), scale, seed, steps
    ("ring_M3_d65536", 3, 65_536, 0, 1e-3, 2022, 2),
    ("ring_M8_d20011", 8, 20_011, 0, 1e-3, 7, 3),
    ("torus_4x4_d30003", 16, 30_003, 4, 2.5e-3, 99, 2),
    ("torus_3x2_d4100", 6, 4_100, 3, 1e-3, 5, 2),
    ("tree_M8_d20011", 8, 20_011, -1, 1e-3, 7, 2),
    ("tree_M5_d777", 5, 777, -1, 1e-3, 11, 2),
]


def inputs(M: int, d: int, step: int) -> np.ndarray:
    """Integer-hash based values in [-1, 1): identical on every machine and library version."""
    m = np.arange(M, dtype=np.uint64)[:, None]
    e = np.arange(d, dtype=np.uint64)[None, :]
    offset = np.uint64((step * 0x94D049BB133111EB + 12345) & 0xFFFFFFFFFFFFFFFF)
    x = m * np.uint64(0x9E3779B97F4A7C15) + e * np.uint64(0xBF58476D1CE4E5B9) + offset
    x ^= x >> np.uint64(31)
    x *= np.uint64(0xD6E8FEB86659FD93)
    x ^= x >> np.uint64(29)
    v = (x >> np.uint64(40)).astype(np.int64) - (1 << 23)          # 24-bit signed
    return (v.astype(np.float64) / float(1 << 23)).astype(np.float32)


def digest(a: np.ndarray) -> str:
    return hashlib.sha256(np.ascontiguousarray(a).tobytes()).hexdigest()


def run_case(M, d, grid_x, scale, seed, steps):
    c = np.zeros((M, d), dtype=np.float32)
    out = []
    for t in range(steps):
        g = inputs(M, d, t)
        if grid_x < 0:
            update, bits = orc.tree_step(g, c, scale, seed + t)
        else:
            update, bits, _ = orc.sync_step(g, c, scale, seed + t, grid_x=grid_x)
        out.append({"bits": digest(bits), "update": digest(update), "c": digest(c)})
    return out


# The other rounds and schedules: name, kind, M, d, parameter (ragged: columns of the torus), steps
EXTRA = [
    ("ragged_torus_M13_x4_d9001", "ragged", 13, 9_001, 4, 2),
    ("ragged_torus_M7_x3_d640", "ragged", 7, 640, 3, 2),
    ("full_precision_M5_d5003", "full", 5, 5_003, 0, 2),
    ("local_adam_M3_d4099", "adam", 3, 4_099, 0, 3),
    ("local_momentum_M3_d4099", "momentum", 3, 4_099, 0, 3),
]


def run_extra(kind, M, d, param, steps):
    c = np.zeros((M, d), dtype=np.float32)
    state1 = np.zeros((M, d), dtype=np.float32)
    state2 = np.zeros((M, d), dtype=np.float32)
    out = []
    for t in range(steps):
        g = inputs(M, d, t)
        if kind == "ragged":
            update, bits = orc.ragged_torus_step(g, c, 1e-3, 31 + t, param, d=d)
            out.append({"bits": digest(bits), "update": digest(update), "c": digest(c)})
        elif kind == "full":
            c += inputs(M, d, 100 + t) * np.float32(0.25)              # a non-zero compensation to fold in
            update = orc.full_sync(g, c, d=d)
            out.append({"update": digest(update), "c": digest(c)})
        elif kind == "adam":
            step = orc.local_adam(state1, state2, g, 0.9, 0.999, 1e-8, 0.01, 1.0 - 0.9 ** (t + 1), 1.0 - 0.999 ** (t + 1))
            out.append({"step": digest(step), "mom1": digest(state1), "mom2": digest(state2)})
        else:
            step = orc.local_momentum(state1, g, 0.9, 0.05)
            out.append({"step": digest(step), "buf": digest(state1)})
    return out


def main():
    table = {name: run_case(M, d, gx, scale, seed, steps) for name, M, d, gx, scale, seed, steps in CASES}
    table.update({name: run_extra(kind, M, d, param, steps) for name, kind, M, d, param, steps in EXTRA})
    path = os.path.join(HERE, "oracle_digests.json")
    with open(path, "w") as fh:
        json.dump(table, fh, indent=1, sort_keys=True)
        fh.write("\n")
    print("wrote", path)


if __name__ == "__main__":
    main()

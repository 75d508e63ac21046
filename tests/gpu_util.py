"""Helpers shared by the GPU parity tests (test code only)."""

import numpy as np
import torch

from oracle import marsit_oracle as orc
from paper_2204_06787_amd import marsit

REL_TOL = 1e-6          # stated bar for decoded updates and compensation vectors (fp32 relative error)


def dev(a: np.ndarray) -> torch.Tensor:
    if a.dtype == np.uint64:
        a = a.view(np.int64)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host_bits(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().numpy().view(np.uint64)


def host_f32(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().numpy()


def unaligned_rows(M: int, ld: int, offset_elems: int = 1) -> torch.Tensor:
    """[M, ld] float32 view whose base pointer is offset_elems * 4 bytes past a 256-byte boundary."""
    base = torch.zeros(M * ld + 8, dtype=torch.float32, device="cuda")
    return base[offset_elems:offset_elems + M * ld].view(M, ld)


def assert_f32_parity(got: np.ndarray, want: np.ndarray, what: str):
    """Within 1e-6 relative (the stated bar) -- and, because every step is a single fp32 rounding
    of identical operands, in fact bit for bit."""
    got = np.asarray(got)
    want = np.asarray(want)
    assert got.shape == want.shape, what
    finite = np.isfinite(want)
    assert np.array_equal(np.isfinite(got), finite), what
    denom = np.maximum(np.abs(want[finite]).astype(np.float64), np.finfo(np.float32).tiny)
    err = np.abs(got[finite].astype(np.float64) - want[finite].astype(np.float64)) / denom
    assert err.size == 0 or err.max() <= REL_TOL, f"{what}: max rel err {err.max():.3e}"
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), f"{what}: not bit-identical"


def oracle_step(g_host: np.ndarray, c_host: np.ndarray, scale, seed, grid_x=0, d=None, threads=8):
    """Runs the oracle on host copies; c_host is updated in place."""
    return orc.sync_step(g_host, c_host, scale, seed, grid_x=grid_x, d=d, threads=threads)


def fused_step(g: torch.Tensor, c: torch.Tensor, scale, seed, grid_x=0, d=None, want_bits=True):
    d = g.shape[1] if d is None else d
    update = torch.full((max(d, 1),), 7.0, dtype=torch.float32, device="cuda")[:d]
    bits = marsit.new_bitmap(d) if want_bits else None
    if bits is not None:
        bits.fill_(-1)
    marsit.marsit_ring_step_sim(g, c, update, bits, scale, seed, grid_x=grid_x, d=d)
    torch.cuda.synchronize()
    return update, bits


def unfused_step(g: torch.Tensor, c: torch.Tensor, scale, seed, grid_x=0, d=None):
    """The same pass as a chain of the three per-worker entry points along the schedule."""
    M = g.shape[0]
    d = g.shape[1] if d is None else d
    W = marsit.n_words(d)
    X = grid_x or M
    Y = M // X
    maps = [marsit.marsit_compress(g[m], c[m], marsit.new_bitmap(d), d=d) for m in range(M)]
    fine = marsit.marsit_split_bounds(W, M, grid_x)
    rows = [marsit.new_bitmap(d) for _ in range(Y)]
    for a in range(X):
        lo, hi = fine[a * Y], fine[(a + 1) * Y]
        if hi == lo:
            continue
        for y in range(Y):
            r = rows[y][lo:hi]
            r.copy_(maps[y * X + a][lo:hi])
            for h in range(1, X):
                marsit.marsit_hop_merge(r, maps[y * X + (a + h) % X][lo:hi], r, lo, hi - lo, h + 1,
                                        (y << 8) | h, seed)
    final = marsit.new_bitmap(d)
    for a in range(X):
        for b in range(Y):
            lo, hi = fine[a * Y + b], fine[a * Y + b + 1]
            if hi == lo:
                continue
            r = final[lo:hi]
            r.copy_(rows[b][lo:hi])
            for k in range(1, Y):
                marsit.marsit_hop_merge(r, rows[(b + k) % Y][lo:hi], r, lo, hi - lo, k + 1,
                                        (1 << 16) | k, seed)
    update = torch.empty(d, dtype=torch.float32, device="cuda")
    for m in range(M):
        marsit.marsit_decode_compensate(final, g[m], c[m], scale, update if m == 0 else None, c[m], d=d)
    torch.cuda.synchronize()
    return update, final, maps

"""Other multi-hop schedules on the GPU against the oracle: the weighted merge and the reduction tree."""

import numpy as np
import pytest
import torch

from oracle import marsit_oracle as orc
from paper_2204_06787_amd import marsit, workloads
from gpu_util import assert_f32_parity, dev, host_bits, host_f32, unaligned_rows

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("w_recv,w_local", [(0, 1), (1, 1), (2, 1), (1, 2), (4, 4), (3, 4), (7, 1), (1, 63), (40, 24)])
@pytest.mark.parametrize("n_words", [1, 17, 5000])
def test_hop_merge_weighted(w_recv, w_local, n_words):
    rng = np.random.default_rng(n_words + 100 * w_recv + w_local)
    recv = rng.integers(0, 2**64, size=n_words, dtype=np.uint64)
    local = rng.integers(0, 2**64, size=n_words, dtype=np.uint64)
    hop, seed, begin = orc.tree_hop_id(2, 8), 0x1234ABCD5678, 77
    want = orc.hop_merge_weighted(recv, local, begin, w_recv, w_local, hop, seed)
    out = torch.zeros(n_words, dtype=torch.int64, device="cuda")
    marsit.marsit_hop_merge_weighted(dev(recv), dev(local), out, begin, n_words, w_recv, w_local, hop, seed)
    torch.cuda.synchronize()
    assert np.array_equal(host_bits(out), want)


def _check_tree(M, d, ld=None, aligned=True, steps=2, scale=1e-3, seed=0x7EE):
    ld = d if ld is None else ld
    rng = np.random.default_rng(M * 977 + d)
    g_h = rng.standard_normal((M, ld)).astype(np.float32)
    c_h = (0.3 * rng.standard_normal((M, ld))).astype(np.float32)
    if aligned:
        g_d, c_d = dev(g_h), dev(c_h)
    else:
        g_d, c_d = unaligned_rows(M, ld), unaligned_rows(M, ld)
        g_d.copy_(dev(g_h))
        c_d.copy_(dev(c_h))
    pad = c_h[:, d:].copy()
    u = torch.empty(d, dtype=torch.float32, device="cuda")
    b = marsit.new_bitmap(d)
    for t in range(steps):
        sd = workloads.step_seed(seed, t)
        b.fill_(-1)
        marsit.marsit_tree_step_sim(g_d, c_d, u, b, scale, sd, d=d)
        torch.cuda.synchronize()
        want_u, want_b = orc.tree_step(g_h, c_h, scale, sd, d=d)
        assert np.array_equal(host_bits(b), want_b), (M, d, t)
        assert np.array_equal(host_f32(u).view(np.uint32), want_u.view(np.uint32)), (M, d, t)
        assert_f32_parity(host_f32(c_d)[:, :d], c_h[:, :d], f"compensation (tree), step {t}")
    assert np.array_equal(host_f32(c_d)[:, d:], pad)


@pytest.mark.parametrize("M", [1, 2, 3, 4, 5, 6, 7, 8, 12, 16])
@pytest.mark.parametrize("d", [5, 64, 1000, 65_536 + 9])
def test_tree_step_compiled_schedules(M, d):
    _check_tree(M, d)


@pytest.mark.parametrize("M", [9, 10, 11, 13, 24, 33, 41, 48, 49, 64])
@pytest.mark.parametrize("d", [7, 4100, 50_001])
def test_tree_step_generic(M, d):
    _check_tree(M, d)


@pytest.mark.parametrize("M,d,ld", [(8, 1000, 1001), (5, 4099, 4102), (16, 20_000, 20_004)])
def test_tree_step_row_stride_and_misaligned_base(M, d, ld):
    _check_tree(M, d, ld=ld)
    _check_tree(M, d, ld=ld, aligned=False)


def test_tree_step_full_size_headline_shape():
    """M = 8, d = 25.6 M, one step, every element compared."""
    wl = workloads.WORKLOADS["resnet50"]
    g = workloads.make_gradients(wl, 0, seed=2022, device="cuda")
    c = workloads.zero_compensation(wl, device="cuda")
    u = torch.empty(wl.d, dtype=torch.float32, device="cuda")
    b = marsit.new_bitmap(wl.d)
    marsit.marsit_tree_step_sim(g, c, u, b, wl.scale, 99)
    torch.cuda.synchronize()
    g_h = host_f32(g)
    c_h = np.zeros_like(g_h)
    want_u, want_b = orc.tree_step(g_h, c_h, wl.scale, 99)
    assert np.array_equal(host_bits(b), want_b)
    assert np.array_equal(host_f32(u), want_u)
    assert_f32_parity(host_f32(c), c_h, "compensation (tree, full size)")


# ------------------------------------------------------------------------------------------------
# torus whose last row is short (M not a multiple of the number of columns)
# ------------------------------------------------------------------------------------------------

@pytest.mark.parametrize("M,grid_x", [(3, 2), (5, 2), (5, 3), (7, 3), (5, 4), (11, 4), (13, 5), (23, 6), (41, 7),
                                      (64, 9), (63, 8), (6, 3), (8, 8), (4, 1), (9, 2), (23, 4), (47, 5), (50, 7), (50, 12)])
@pytest.mark.parametrize("d,ld,offset", [(7, 7, 0), (64 * 40, 64 * 40, 0), (33_333, 33_336, 0), (5001, 5003, 1)])
def test_ragged_torus_step(M, grid_x, d, ld, offset):
    """Short last row, weighted column merges; staged (M <= 48) and gather-and-sweep (M > 48)
    kernels, up to four rows (row draws shared by a lane's bits) and more (drawn per bit), ragged sizes, padded and misaligned rows, two steps with the compensation carried over; the
    dividing shapes take the plain torus kernels and must agree with the same oracle routine."""
    rng = np.random.default_rng(M * 100 + grid_x + d)
    c_h = np.zeros((M, ld), dtype=np.float32)
    if offset:
        c_d = unaligned_rows(M, ld, offset)
    else:
        c_d = torch.zeros((M, ld), dtype=torch.float32, device="cuda")
    x_h = rng.standard_normal(d).astype(np.float32)
    x_d = dev(x_h)
    u_d = torch.empty(d, dtype=torch.float32, device="cuda")
    bits = marsit.new_bitmap(d)
    for t in range(2):
        g_h = rng.standard_normal((M, ld)).astype(np.float32)
        if offset:
            g_d = unaligned_rows(M, ld, offset)
            g_d.copy_(dev(g_h))
        else:
            g_d = dev(g_h)
        want_u, want_b = orc.ragged_torus_step(g_h, c_h, 1e-3, 500 + t, grid_x, d=d, threads=8)
        if t == 0:
            marsit.marsit_ragged_torus_step_sim(g_d, c_d, u_d, bits, 1e-3, 500 + t, grid_x, d=d)
        else:
            marsit.marsit_ragged_torus_step_apply(g_d, c_d, x_d, u_d, bits, 1e-3, 500 + t, grid_x, d=d)
            x_h = orc.apply_update(x_h, want_u)
        torch.cuda.synchronize()
        assert np.array_equal(host_bits(bits), want_b), t
        assert np.array_equal(host_f32(u_d).view(np.uint32), want_u.view(np.uint32)), t
        assert_f32_parity(host_f32(c_d)[:, :d], c_h[:, :d], f"compensation, step {t}")
        assert np.array_equal(host_f32(c_d)[:, d:], c_h[:, d:])
        assert_f32_parity(host_f32(x_d), x_h, f"model, step {t}")

"""Matching-rate diagnostics (Section 3.2.2, Fig. 2b) on the GPU against the oracle, and the
closed-form matching rate of the merged signs at scale."""

import numpy as np
import pytest
import torch

from oracle import marsit_oracle as orc
from paper_2204_06787_amd import marsit, workloads
from gpu_util import dev, fused_step, host_bits, host_f32, unaligned_rows

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("M,d,ld,aligned", [(1, 5, 5, True), (2, 64, 64, True), (3, 1000, 1001, True), (8, 100_003, 100_004, True),
                                             (16, 4097, 4100, False), (64, 300, 300, True), (7, 65_536, 65_536, True)])
def test_votes_and_matching_count(M, d, ld, aligned):
    rng = np.random.default_rng(M * 1000 + d)
    g_h = rng.standard_normal((M, ld)).astype(np.float32)
    c_h = (0.5 * rng.standard_normal((M, ld))).astype(np.float32)
    g_h[:, :min(d, 3)] = 0.0
    c_h[:, :min(d, 3)] = -0.0
    if aligned:
        g_d, c_d = dev(g_h), dev(c_h)
    else:
        g_d, c_d = unaligned_rows(M, ld), unaligned_rows(M, ld)
        g_d.copy_(dev(g_h))
        c_d.copy_(dev(c_h))
    agg = marsit.marsit_aggregate_sign(g_d, c_d, marsit.new_bitmap(d).fill_(-1), d=d)
    maj = marsit.marsit_majority_vote(g_d, c_d, marsit.new_bitmap(d).fill_(-1), d=d)
    count = torch.full((1,), 123, dtype=torch.int64, device="cuda")
    marsit.marsit_count_matching(agg, maj, d, count)
    torch.cuda.synchronize()
    want_agg, want_maj = orc.aggregate_sign(g_h, c_h, d=d), orc.majority_vote(g_h, c_h, d=d)
    assert np.array_equal(host_bits(agg), want_agg)
    assert np.array_equal(host_bits(maj), want_maj)
    assert int(count.item()) == orc.count_matching(want_agg, want_maj, d)
    marsit.marsit_count_matching(agg, agg, d, count)
    torch.cuda.synchronize()
    assert int(count.item()) == d


def test_matching_rate_of_merged_signs_at_scale():
    """On i.i.d. Gaussian gradients the merged bit is the sign of a uniformly drawn worker, so its
    matching rate is 1/2 + arcsin(1/sqrt(M))/pi; the majority vote does better, as the paper's
    Fig. 2(b) ordering has it.  M = 8, d = 11.2 M."""
    wl = workloads.WORKLOADS["resnet18"]
    g = workloads.make_gradients(wl, 0, seed=9, device="cuda")
    c = workloads.zero_compensation(wl, device="cuda")
    ref = marsit.marsit_aggregate_sign(g, c, marsit.new_bitmap(wl.d))
    maj = marsit.marsit_majority_vote(g, c, marsit.new_bitmap(wl.d))
    _, bits = fused_step(g, c, wl.scale, 4321)
    count = torch.zeros(1, dtype=torch.int64, device="cuda")
    marsit.marsit_count_matching(bits, ref, wl.d, count)
    torch.cuda.synchronize()
    rate = int(count.item()) / wl.d
    want = 0.5 + np.arcsin(1.0 / np.sqrt(wl.M)) / np.pi
    assert abs(rate - want) <= 5 * np.sqrt(want * (1 - want) / wl.d)
    marsit.marsit_count_matching(maj, ref, wl.d, count)
    torch.cuda.synchronize()
    assert int(count.item()) / wl.d > rate + 0.05


# ------------------------------------------------------------------------------------------------
# the strawman of Section 3.2: SSDM stochastic sign, cascading compression
# ------------------------------------------------------------------------------------------------

@pytest.mark.parametrize("n,offset", [(1, 0), (5, 0), (64, 0), (1000, 0), (4099, 1), (300_001, 0)])
def test_ssdm_cascade_hop(n, offset):
    rng = np.random.default_rng(n)
    g_h = rng.standard_normal(n + 1).astype(np.float32)
    c_h = (0.1 * rng.standard_normal(n + 1)).astype(np.float32)
    g1 = np.ascontiguousarray(g_h[offset:offset + n])
    c1 = np.ascontiguousarray(c_h[offset:offset + n])
    gd, cd = dev(g_h)[offset:offset + n], dev(c_h)[offset:offset + n]
    ws = marsit.new_cascade_workspace()
    seed, begin = 0xC0FFEE, 12345
    # first holder
    t0 = orc.add_compensation(g1, c1)
    norm0 = orc.l2_norm(t0)
    want0 = orc.ssdm_sign(t0, norm0, begin, orc.cascade_hop_id(0), seed)
    bits = marsit.new_bitmap(n).fill_(-1)
    norm_a = torch.zeros(1, dtype=torch.float32, device="cuda")
    norm_b = torch.zeros(1, dtype=torch.float32, device="cuda")
    marsit.marsit_ssdm_cascade_hop(None, None, gd, cd, bits, norm_a, ws, begin, n, orc.cascade_hop_id(0), seed)
    torch.cuda.synchronize()
    assert float(norm_a.item()) == norm0
    assert np.array_equal(host_bits(bits), want0)
    # a later hop, in place on the bitmap
    signs = np.where(((want0[np.arange(n) // 64] >> (np.arange(n) % 64).astype(np.uint64)) & np.uint64(1)) == 1,
                     np.float32(norm0), np.float32(-norm0)).astype(np.float32)
    t1 = (signs + t0).astype(np.float32)
    norm1 = orc.l2_norm(t1)
    want1 = orc.ssdm_sign(t1, norm1, begin, orc.cascade_hop_id(1), seed)
    marsit.marsit_ssdm_cascade_hop(bits, norm_a, gd, cd, bits, norm_b, ws, begin, n, orc.cascade_hop_id(1), seed)
    torch.cuda.synchronize()
    assert float(norm_b.item()) == norm1
    assert np.array_equal(host_bits(bits), want1)


@pytest.mark.parametrize("M,d", [(1, 100), (3, 65_536), (8, 400_000 + 21), (5, 7), (4, 64 * 4)])
def test_cascade_ring_step(M, d):
    rng = np.random.default_rng(M + d)
    g_h = rng.standard_normal((M, d)).astype(np.float32)
    c_h = (0.2 * rng.standard_normal((M, d))).astype(np.float32)
    want_u, want_b, want_n = orc.cascade_ring_step(g_h, c_h, 31337)
    u = torch.zeros(d, dtype=torch.float32, device="cuda")
    b = marsit.new_bitmap(d).fill_(0)
    norms = torch.zeros(M, dtype=torch.float32, device="cuda")
    marsit.marsit_cascade_ring_step_sim(dev(g_h), dev(c_h), u, b, norms, marsit.new_cascade_workspace(), 31337)
    torch.cuda.synchronize()
    assert np.array_equal(host_f32(norms), want_n)
    assert np.array_equal(host_bits(b), want_b)
    assert np.array_equal(host_f32(u).view(np.uint32), want_u.view(np.uint32))


def test_matching_rate_ordering_at_scale():
    """Fig. 2(b)'s ordering on synthetic gradients, M = 8, d = 11.2 M: cascading compression is close
    to a coin flip, Marsit's merged signs sit at the closed-form rate, the majority vote is highest."""
    wl = workloads.WORKLOADS["resnet18"]
    g = workloads.make_gradients(wl, 0, seed=10, device="cuda")
    c = workloads.zero_compensation(wl, device="cuda")
    ref = marsit.marsit_aggregate_sign(g, c, marsit.new_bitmap(wl.d))
    maj = marsit.marsit_majority_vote(g, c, marsit.new_bitmap(wl.d))
    cas = marsit.new_bitmap(wl.d)
    marsit.marsit_cascade_ring_step_sim(g, c, torch.empty(wl.d, device="cuda"), cas,
                                        torch.empty(wl.M, device="cuda"), marsit.new_cascade_workspace(), 17)
    _, mar = fused_step(g, c, wl.scale, 17)
    count = torch.zeros(1, dtype=torch.int64, device="cuda")
    rates = {}
    for name, bits in (("cascading", cas), ("marsit", mar), ("majority", maj)):
        marsit.marsit_count_matching(bits, ref, wl.d, count)
        torch.cuda.synchronize()
        rates[name] = int(count.item()) / wl.d
    print("matching rates:", rates, flush=True)
    assert abs(rates["cascading"] - 0.5) < 0.01
    assert abs(rates["marsit"] - (0.5 + np.arcsin(1 / np.sqrt(wl.M)) / np.pi)) < 1e-3
    assert rates["cascading"] < rates["marsit"] < rates["majority"]

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

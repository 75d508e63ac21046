"""Sizes beyond 2^32 elements per vector: every index and offset of the fused kernel has to be 64-bit.
The oracle cannot run 8.6 G elements in test time, so sampled packed words are checked against the
oracle's one-word routines and the rest through properties that hold at any size."""

import numpy as np
import pytest
import torch

from oracle import marsit_oracle as orc
from paper_2204_06787_amd import marsit

pytestmark = pytest.mark.gpu


def test_more_than_2_to_32_elements_per_worker():
    M, d, scale, seed = 2, (1 << 32) + 64 * 3 + 5, 1e-3, 0xB16B00B5
    free, _ = torch.cuda.mem_get_info()
    if free < 150 * (1 << 30):
        pytest.skip("needs about 150 GB of device memory")
    print(f"huge: M={M} d={d}", flush=True)
    gen = torch.Generator(device="cuda").manual_seed(5)
    g = torch.empty((M, d), dtype=torch.float32, device="cuda")
    c = torch.empty((M, d), dtype=torch.float32, device="cuda")
    for m in range(M):
        g[m].normal_(generator=gen)
        c[m].normal_(generator=gen).mul_(0.25)
    s = g + c                                           # compensated gradient, fp32, by a different implementation
    c_in = None
    update = torch.empty(d, dtype=torch.float32, device="cuda")
    bits = marsit.new_bitmap(d)
    marsit.marsit_ring_step_sim(g, c, update, bits, scale, seed)
    torch.cuda.synchronize()

    # properties at full size
    assert bool((update.abs() == np.float32(scale)).all())                      # +-scale everywhere
    assert bool((c[0] == s[0] - update).all()) and bool((c[1] == s[1] - update).all())   # compensation update
    plus = update > 0
    pos0, pos1 = s[0] >= 0, s[1] >= 0
    agree = pos0 == pos1
    assert bool((~agree | (plus == pos0)).all())                 # same sign in both: unchanged (Section 1)
    # the share of disagreeing elements that took worker 1's sign is about one half
    n_dis = int((~agree).sum().item())
    n_took1 = int((~agree & (plus == pos1)).sum().item())
    assert abs(n_took1 / n_dis - 0.5) < 1e-3
    del plus, pos0, pos1, agree

    # sampled packed words against the oracle, among them the first, the last and the ones around
    # the part boundary and the 2^32-element mark
    W = orc.n_words(d)
    bounds = [int(x) for x in orc.split_bounds(0, W, M)]
    rng = np.random.default_rng(1)
    words = set(int(x) for x in rng.integers(0, W, size=1500))
    words |= {0, 1, W - 1, W - 2, W - 3, bounds[1] - 1, bounds[1], (1 << 26) - 1, 1 << 26, (1 << 26) + 1}
    words = sorted(words)
    idx = torch.tensor(words, dtype=torch.int64, device="cuda")
    got_words = bits[idx].cpu().numpy().view(np.uint64)
    for n, w in enumerate(words):
        lo, hi = w * 64, min(d, w * 64 + 64)
        sw = s[:, lo:hi].cpu().numpy()
        i = 0 if w < bounds[1] else 1                                        # part -> first holder
        first = orc.sign_pack(np.ascontiguousarray(sw[i]))
        local = orc.sign_pack(np.ascontiguousarray(sw[1 - i]))
        want = orc.merge_word(int(first[0]), int(local[0]), 2, 1, seed, w)
        assert int(got_words[n]) == want, w
        want_u = orc.decode(np.array([want], dtype=np.uint64), scale, hi - lo)
        assert np.array_equal(update[lo:hi].cpu().numpy(), want_u), w

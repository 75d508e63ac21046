"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, and its host-side
logic (argument validation, Philox, part bounds) behaves as include/marsit.h says.  No kernel is
launched here."""

import os
import re

import numpy as np
import pytest

from oracle import marsit_oracle as orc
from paper_2204_06787_amd import marsit
import philox_ref

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x10000          # a non-NULL, 16-byte aligned "device pointer" that is never dereferenced


@pytest.fixture(scope="module")
def lib():
    return marsit.load_library()


def test_library_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "marsit.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(marsit_[a-z0-9_]+)\s*\(", header))
    assert declared == set(marsit.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_version_and_status_strings(lib):
    assert marsit.marsit_version() >= 100
    assert lib.marsit_status_string(0) == b"ok"
    for code in (-1, -2, -3, -99):
        assert len(lib.marsit_status_string(code)) > 0


def test_host_philox_matches_other_implementations():
    for line in open(os.path.join(ROOT, "tests", "golden", "philox4x32_10_kat.txt")):
        if line.startswith("#") or not line.strip():
            continue
        v = [int(x, 16) for x in line.split()]
        assert marsit.marsit_philox4x32_10(v[0:4], v[4:6]) == v[6:10]
    rng = np.random.default_rng(21)
    for _ in range(300):
        ctr = [int(x) for x in rng.integers(0, 2**32, size=4)]
        key = [int(x) for x in rng.integers(0, 2**32, size=2)]
        want = philox_ref.philox4x32_10(ctr, key)
        assert marsit.marsit_philox4x32_10(ctr, key) == want
        assert [int(x) for x in orc.philox4x32_10(ctr, key)] == want


@pytest.mark.parametrize("W,M,gx", [(1024, 3, 0), (400_000, 8, 0), (2_156_250, 8, 0), (400_000, 16, 4),
                                    (5, 8, 0), (7, 6, 3), (0, 4, 2), (1001, 12, 4), (999, 64, 8)])
def test_split_bounds_match_oracle(W, M, gx):
    got = marsit.marsit_split_bounds(W, M, gx)
    X = gx or M
    Y = M // X
    rows = [int(x) for x in orc.split_bounds(0, W, X)]
    want = []
    for a in range(X):
        sub = [int(x) for x in orc.split_bounds(rows[a], rows[a + 1] - rows[a], Y)]
        want.extend(sub[:-1])
    want.append(W)
    assert got == want


def test_split_bounds_rejects_bad_shapes(lib):
    import ctypes
    buf = (ctypes.c_uint64 * 65)()
    assert lib.marsit_split_bounds(10, 0, 0, buf) == marsit.EINVAL
    assert lib.marsit_split_bounds(10, 65, 0, buf) == marsit.EINVAL
    assert lib.marsit_split_bounds(10, 6, 4, buf) == marsit.EINVAL
    assert lib.marsit_split_bounds(10, 6, 0, None) == marsit.EINVAL


def test_ring_step_argument_validation(lib):
    ok = dict(g=FAKE, c=FAKE, u=FAKE, b=None, M=8, d=64, ld=64, scale=1e-3, seed=1, gx=0)

    def call(**kw):
        a = dict(ok, **kw)
        return lib.marsit_ring_step_sim(a["g"], a["c"], a["u"], a["b"], a["M"], a["d"], a["ld"],
                                        a["scale"], a["seed"], a["gx"], None)
    assert call(g=None) == marsit.EINVAL
    assert call(c=None) == marsit.EINVAL
    assert call(u=None) == marsit.EINVAL
    assert call(M=0) == marsit.EINVAL
    assert call(M=65) == marsit.EINVAL
    assert call(ld=63) == marsit.EINVAL
    assert call(gx=3) == marsit.EINVAL
    assert call(scale=float("inf")) == marsit.EINVAL
    assert call(scale=float("nan")) == marsit.EINVAL
    assert call(d=marsit.MAX_ELEMENTS + 1, ld=marsit.MAX_ELEMENTS + 1) == marsit.EINVAL
    assert call(g=FAKE + 2) == marsit.EALIGN
    assert call(b=FAKE + 4) == marsit.EALIGN
    assert call(d=0) == marsit.OK            # empty input: success, nothing launched


def test_size_limit_is_what_one_launch_can_cover(lib):
    """Every kernel covers its vector with one launch of at most one work-item per 4 elements in
    whole workgroups of 256, and a launch must stay below 2^32 work-items in x.  The limit in the
    header is exactly the largest d for which that holds; larger sizes are refused as invalid
    arguments by every entry point, before anything is launched."""
    header = open(os.path.join(ROOT, "include", "marsit.h")).read()
    limit = int(re.search(r"#define\s+MARSIT_MAX_ELEMENTS\s+(\d+)ull", header).group(1))
    assert limit == marsit.MAX_ELEMENTS == (1 << 34) - 1024

    def work_items(d, block):          # the launch geometry, recomputed here
        cols = (d + 3) // 4
        return (cols + block - 1) // block * block
    for d in (1, 4, 5, 1023, 1024, 1025, 25_600_000, (1 << 32) + 197, (1 << 34) - 1028, limit - 4, limit - 1, limit):
        assert lib.marsit_grid_work_items(d) == work_items(d, 256), d
        assert work_items(d, 256) < (1 << 32) and work_items(d, 64) < (1 << 32), d
        # the per-word kernels: 16 work-items per packed word, 64 per 4 words in marsit_compress
        words = (d + 63) // 64
        assert (words * 16 + 255) // 256 * 256 < (1 << 32)
        assert ((words + 3) // 4 * 64 + 255) // 256 * 256 < (1 << 32)
    assert work_items(limit + 1, 256) == (1 << 32)                   # the first size one launch cannot cover
    for d in (limit + 1, 1 << 34, (1 << 34) + 4, 1 << 37, (1 << 37) + 1, (1 << 64) - 1):
        assert lib.marsit_grid_work_items(d) == 0, d
    assert lib.marsit_grid_work_items(0) == 0

    for d in (limit + 1, 1 << 34, 1 << 37):
        E = marsit.EINVAL
        assert lib.marsit_ring_step_sim(FAKE, FAKE, FAKE, None, 1, d, d, 1e-3, 1, 0, None) == E
        assert lib.marsit_tree_step_sim(FAKE, FAKE, FAKE, None, 1, d, d, 1e-3, 1, None) == E
        assert lib.marsit_ragged_torus_step_sim(FAKE, FAKE, FAKE, None, 3, d, d, 1e-3, 1, 2, None) == E
        assert lib.marsit_full_sync(FAKE, FAKE, FAKE, 1, d, d, None) == E
        assert lib.marsit_step(1, 2, FAKE, FAKE, FAKE, None, 1, d, d, 1e-3, 1, 0, None) == E
        assert lib.marsit_step_apply(1, 2, FAKE, FAKE, FAKE, None, None, 1, d, d, 1e-3, 1, 0, None) == E
        assert lib.marsit_round(1, 2, 0, 0, FAKE, FAKE, FAKE, None, None, 1, d, d, 1e-3, 1, None) == E
        assert lib.marsit_round(0, 2, 2, 0, FAKE, FAKE, FAKE, None, None, 1, d, d, 1e-3, 1, None) == E
        assert lib.marsit_compress(FAKE, None, FAKE, d, None) == E
        assert lib.marsit_decode_compensate(FAKE, FAKE, None, 1.0, None, FAKE, d, None) == E
        assert lib.marsit_decode_compensate_apply(FAKE, FAKE, None, 1.0, FAKE + 64, None, FAKE, d, None) == E
        assert lib.marsit_compress_hop_merge(FAKE, FAKE, None, FAKE, 0, d, 2, 1, 1, None) == E
        assert lib.marsit_hop_merge(FAKE, FAKE, FAKE, 0, d // 64 + 1, 2, 1, 5, None) == E
        assert lib.marsit_hop_merge_weighted(FAKE, FAKE, FAKE, 0, d // 64 + 1, 2, 1, 1, 5, None) == E
        assert lib.marsit_fold_segments(FAKE, d, 2, 0, FAKE, 0, d // 64 + 1, 0, 5, None) == E
        assert lib.marsit_apply_update(FAKE, FAKE, d, None) == E
        assert lib.marsit_local_momentum(FAKE, FAKE + 64, FAKE + 64, 1, d, d, 0.5, 0.1, None) == E
        assert lib.marsit_local_adam(FAKE, FAKE + 64, FAKE + 128, FAKE + 128, 1, d, d, 0.9, 0.99, 1e-8, 0.1, 0.1, 0.01, None) == E
        assert lib.marsit_chain_step_sim(FAKE, FAKE, FAKE, FAKE, FAKE, 1, d, d, 1.0, 1, 0, None) == E
        assert lib.marsit_exchange_step_sim(FAKE, FAKE, FAKE, FAKE, FAKE, 1, d, d, 1.0, 1, 0, None) == E
        assert lib.marsit_exchange_step_sim_static(FAKE, FAKE, FAKE, FAKE, 1, d, d, 1.0, 1, 0, None) == E
        assert lib.marsit_aggregate_sign(FAKE, FAKE, FAKE, 1, d, d, None) == E
        assert lib.marsit_majority_vote(FAKE, FAKE, FAKE, 1, d, d, None) == E
        assert lib.marsit_count_matching(FAKE, FAKE, d, FAKE, None) == E
        assert lib.marsit_ssdm_cascade_hop(None, None, FAKE, FAKE, FAKE, FAKE, FAKE, 0, d, 1, 1, None) == E
        assert lib.marsit_cascade_ring_step_sim(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 1, d, d, 1, None) == E
        assert marsit.marsit_chain_workspace_words(1, d, 0) == 0
        assert lib.marsit_pipeline_workspace_words(1, d, 0) == 0


def test_fused_waves_hook_validation(lib):
    assert lib.marsit_set_fused_waves_per_cu(1) == marsit.EINVAL
    assert lib.marsit_set_fused_waves_per_cu(33) == marsit.EINVAL
    assert lib.marsit_set_fused_waves_per_cu(2) == marsit.OK
    assert lib.marsit_set_fused_waves_per_cu(32) == marsit.OK
    assert lib.marsit_set_fused_waves_per_cu(0) == marsit.OK          # back to the built-in choice


def test_other_entry_points_argument_validation(lib):
    assert lib.marsit_compress(None, None, FAKE, 64, None) == marsit.EINVAL
    assert lib.marsit_compress(FAKE, None, None, 64, None) == marsit.EINVAL
    assert lib.marsit_compress(FAKE + 1, None, FAKE, 64, None) == marsit.EALIGN
    assert lib.marsit_compress(FAKE, None, FAKE, 0, None) == marsit.OK

    assert lib.marsit_hop_merge(FAKE, FAKE, FAKE, 0, 10, 0, 1, 5, None) == marsit.EINVAL      # fold 0
    assert lib.marsit_hop_merge(None, FAKE, FAKE, 0, 10, 2, 1, 5, None) == marsit.EINVAL
    assert lib.marsit_hop_merge(FAKE + 4, FAKE, FAKE, 0, 10, 2, 1, 5, None) == marsit.EALIGN
    assert lib.marsit_hop_merge(FAKE, FAKE, FAKE, 0, 0, 2, 1, 5, None) == marsit.OK

    assert lib.marsit_decode_compensate(None, FAKE, None, 1.0, None, FAKE, 64, None) == marsit.EINVAL
    assert lib.marsit_decode_compensate(FAKE, FAKE, None, 1.0, None, None, 64, None) == marsit.EINVAL
    assert lib.marsit_decode_compensate(FAKE, FAKE, None, float("inf"), None, FAKE, 64, None) == marsit.EINVAL
    assert lib.marsit_decode_compensate(FAKE, FAKE, None, 1.0, None, FAKE, 0, None) == marsit.OK

    assert lib.marsit_full_sync(FAKE, FAKE, FAKE, 0, 64, 64, None) == marsit.EINVAL
    assert lib.marsit_full_sync(FAKE, FAKE, FAKE, 4, 64, 32, None) == marsit.EINVAL
    assert lib.marsit_full_sync(FAKE, FAKE, FAKE, 4, 0, 0, None) == marsit.OK

    assert lib.marsit_step(3, 0, FAKE, FAKE, FAKE, None, 4, 64, 64, 1.0, 1, 0, None) == marsit.EINVAL   # K = 0
    assert lib.marsit_step(3, 5, FAKE, FAKE, FAKE, None, 0, 64, 64, 1.0, 1, 0, None) == marsit.EINVAL
    assert lib.marsit_step(5, 5, FAKE, FAKE, FAKE, None, 4, 64, 64, float("nan"), 1, 0, None) == marsit.EINVAL
    assert lib.marsit_step(5, 5, FAKE, FAKE, FAKE, None, 4, 0, 0, 1.0, 1, 0, None) == marsit.OK

    assert lib.marsit_chain_step_sim(FAKE, FAKE, FAKE, FAKE, None, 4, 64, 64, 1.0, 1, 0, None) == marsit.EINVAL
    assert lib.marsit_chain_step_sim(FAKE, FAKE, FAKE, None, FAKE, 4, 64, 64, 1.0, 1, 0, None) == marsit.EINVAL
    assert lib.marsit_chain_step_sim(FAKE, FAKE, FAKE, FAKE, FAKE, 4, 64, 64, 1.0, 1, 3, None) == marsit.EINVAL
    assert lib.marsit_chain_step_sim(FAKE, FAKE, FAKE, FAKE, FAKE + 4, 4, 64, 64, 1.0, 1, 0, None) == marsit.EALIGN
    assert lib.marsit_chain_step_sim(FAKE, FAKE, FAKE, FAKE, FAKE, 4, 0, 64, 1.0, 1, 0, None) == marsit.OK
    assert marsit.marsit_chain_workspace_words(8, 25_600_000, 0) == 8 * 400_000
    assert marsit.marsit_chain_workspace_words(16, 25_600_000, 4) == 20 * 400_000
    assert marsit.marsit_chain_workspace_words(6, 100, 4) == 0

    assert lib.marsit_compress_hop_merge(None, FAKE, FAKE, FAKE, 0, 64, 2, 1, 1, None) == marsit.EINVAL   # recv needed
    assert lib.marsit_compress_hop_merge(FAKE, FAKE, FAKE, FAKE, 0, 64, 0, 1, 1, None) == marsit.EINVAL   # fold 0
    assert lib.marsit_compress_hop_merge(FAKE, None, FAKE, FAKE, 0, 64, 2, 1, 1, None) == marsit.EINVAL
    assert lib.marsit_compress_hop_merge(FAKE + 4, FAKE, FAKE, FAKE, 0, 64, 2, 1, 1, None) == marsit.EALIGN
    assert lib.marsit_compress_hop_merge(FAKE, FAKE, FAKE, FAKE, 0, 0, 2, 1, 1, None) == marsit.OK

    assert lib.marsit_decode_compensate_apply(FAKE, FAKE, FAKE, 1.0, None, FAKE, FAKE, 64, None) == marsit.EINVAL
    assert lib.marsit_decode_compensate_apply(FAKE, FAKE, FAKE, 1.0, FAKE, FAKE, FAKE + 1024, 64, None) == marsit.EINVAL   # x aliases update
    assert lib.marsit_decode_compensate_apply(FAKE, FAKE, FAKE, 1.0, FAKE + 2, None, FAKE, 64, None) == marsit.EALIGN
    assert lib.marsit_decode_compensate_apply(FAKE, FAKE, FAKE, 1.0, FAKE + 1024, None, FAKE, 0, None) == marsit.OK

    assert lib.marsit_fold_segments(None, 64, 4, 0, FAKE, 0, 64, 0, 1, None) == marsit.EINVAL
    assert lib.marsit_fold_segments(FAKE, 64, 0, 0, FAKE, 0, 64, 0, 1, None) == marsit.EINVAL      # no operands
    assert lib.marsit_fold_segments(FAKE, 64, 4, 4, FAKE, 0, 64, 0, 1, None) == marsit.EINVAL      # first >= K
    assert lib.marsit_fold_segments(FAKE, 32, 4, 0, FAKE, 0, 64, 0, 1, None) == marsit.EINVAL      # operands overlap
    assert lib.marsit_fold_segments(FAKE, 64, 4, 0, FAKE, 0, 64, 3, 1, None) == marsit.EINVAL      # hop bits in the base
    assert lib.marsit_fold_segments(FAKE + 4, 64, 4, 0, FAKE, 0, 64, 0, 1, None) == marsit.EALIGN
    assert lib.marsit_fold_segments(FAKE, 64, 4, 0, FAKE, 0, 0, 0, 1, None) == marsit.OK
    assert lib.marsit_exchange_step_sim(FAKE, FAKE, FAKE, FAKE, None, 4, 64, 64, 1.0, 1, 0, None) == marsit.EINVAL
    assert lib.marsit_exchange_step_sim(FAKE, FAKE, FAKE, FAKE, FAKE, 4, 64, 64, 1.0, 1, 3, None) == marsit.EINVAL
    assert lib.marsit_exchange_step_sim(FAKE, FAKE, FAKE, FAKE, FAKE, 4, 0, 64, 1.0, 1, 0, None) == marsit.OK

    assert lib.marsit_tree_step_apply(FAKE, FAKE, None, FAKE, FAKE, 4, 64, 64, 1.0, 1, None) == marsit.EINVAL
    assert lib.marsit_tree_step_apply(FAKE, FAKE, FAKE, FAKE, FAKE, 4, 64, 64, 1.0, 1, None) == marsit.EINVAL   # x aliases update
    assert lib.marsit_tree_step_apply(FAKE, FAKE, FAKE + 2, None, FAKE, 4, 64, 64, 1.0, 1, None) == marsit.EALIGN
    assert lib.marsit_tree_step_apply(FAKE, FAKE, FAKE, None, None, 4, 0, 64, 1.0, 1, None) == marsit.OK
    assert lib.marsit_tree_step_sim(FAKE, FAKE, None, FAKE, 4, 64, 64, 1.0, 1, None) == marsit.EINVAL

    assert lib.marsit_ragged_torus_step_sim(FAKE, FAKE, FAKE, FAKE, 5, 64, 64, 1.0, 1, 0, None) == marsit.EINVAL    # grid_x = 0
    assert lib.marsit_ragged_torus_step_sim(FAKE, FAKE, FAKE, FAKE, 5, 64, 64, 1.0, 1, 6, None) == marsit.EINVAL    # grid_x > M
    assert lib.marsit_ragged_torus_step_sim(FAKE, FAKE, None, FAKE, 5, 64, 64, 1.0, 1, 2, None) == marsit.EINVAL
    assert lib.marsit_ragged_torus_step_sim(FAKE, FAKE, FAKE, FAKE, 5, 64, 32, 1.0, 1, 2, None) == marsit.EINVAL    # ld < d
    assert lib.marsit_ragged_torus_step_sim(FAKE, FAKE, FAKE + 2, FAKE, 5, 64, 64, 1.0, 1, 2, None) == marsit.EALIGN
    assert lib.marsit_ragged_torus_step_sim(FAKE, FAKE, FAKE, FAKE, 5, 0, 64, 1.0, 1, 2, None) == marsit.OK
    assert lib.marsit_ragged_torus_step_apply(FAKE, FAKE, None, FAKE, FAKE, 5, 64, 64, 1.0, 1, 2, None) == marsit.EINVAL
    assert lib.marsit_ragged_torus_step_apply(FAKE, FAKE, FAKE, None, None, 5, 0, 64, 1.0, 1, 2, None) == marsit.OK

    assert lib.marsit_pipeline_create(None, 4) == marsit.EINVAL
    assert lib.marsit_pipeline_destroy(None) == marsit.EINVAL
    assert lib.marsit_pipeline_ring_step(None, FAKE, FAKE, FAKE, FAKE, FAKE, 64, 64, 1.0, 1, None) == marsit.EINVAL
    assert lib.marsit_pipeline_step(None, FAKE, FAKE, FAKE, FAKE, FAKE, 64, 64, 1.0, 1, 0, None) == marsit.EINVAL
    assert lib.marsit_pipeline_workspace_words(8, 25_600_000, 0) == 8 * 400_000 + 16 * 50_001
    # 4 x 4 torus: own maps, row send buffers, 4 row results, column send buffers
    assert lib.marsit_pipeline_workspace_words(16, 25_600_000, 4) == (
        16 * 400_000 + 32 * 100_001 + 4 * 400_000 + 32 * 25_001)
    assert lib.marsit_pipeline_workspace_words(0, 100, 0) == 0
    assert lib.marsit_pipeline_workspace_words(6, 100, 4) == 0

    assert lib.marsit_aggregate_sign(FAKE, None, FAKE, 4, 64, 64, None) == marsit.EINVAL
    assert lib.marsit_majority_vote(FAKE, FAKE, FAKE, 65, 64, 64, None) == marsit.EINVAL
    assert lib.marsit_majority_vote(FAKE, FAKE, FAKE + 4, 4, 64, 64, None) == marsit.EALIGN
    assert lib.marsit_aggregate_sign(FAKE, FAKE, FAKE, 4, 0, 0, None) == marsit.OK
    assert lib.marsit_count_matching(FAKE, FAKE, 64, None, None) == marsit.EINVAL

    assert lib.marsit_hop_merge_weighted(FAKE, FAKE, FAKE, 0, 10, 3, 0, 1, 5, None) == marsit.EINVAL   # w_local 0
    assert lib.marsit_hop_merge_weighted(FAKE, FAKE, FAKE, 0, 0, 3, 1, 1, 5, None) == marsit.OK
    assert lib.marsit_tree_step_sim(FAKE, FAKE, FAKE, None, 0, 64, 64, 1.0, 1, None) == marsit.EINVAL
    assert lib.marsit_tree_step_sim(FAKE, FAKE, FAKE, None, 8, 64, 32, 1.0, 1, None) == marsit.EINVAL
    assert lib.marsit_tree_step_sim(FAKE, FAKE + 2, FAKE, None, 8, 64, 64, 1.0, 1, None) == marsit.EALIGN
    assert lib.marsit_tree_step_sim(FAKE, FAKE, FAKE, None, 8, 0, 64, 1.0, 1, None) == marsit.OK

    assert lib.marsit_ssdm_cascade_hop(None, None, FAKE, FAKE, FAKE, None, FAKE, 0, 64, 1, 5, None) == marsit.EINVAL
    assert lib.marsit_ssdm_cascade_hop(FAKE, None, FAKE, FAKE, FAKE, FAKE, FAKE, 0, 64, 1, 5, None) == marsit.EINVAL
    assert lib.marsit_ssdm_cascade_hop(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 0, 64, 1, 5, None) == marsit.EINVAL
    assert lib.marsit_ssdm_cascade_hop(None, None, FAKE, FAKE, FAKE, FAKE, FAKE, 0, 0, 1, 5, None) == marsit.OK
    assert lib.marsit_cascade_ring_step_sim(FAKE, FAKE, FAKE, FAKE, FAKE, None, 4, 64, 64, 5, None) == marsit.EINVAL
    assert lib.marsit_cascade_ring_step_sim(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 4, 0, 64, 5, None) == marsit.OK

    assert lib.marsit_hop_merge_device_seed(FAKE, FAKE, FAKE, 0, 10, 2, 1, None, None) == marsit.EINVAL
    assert lib.marsit_hop_merge_device_seed(FAKE, FAKE, FAKE, 0, 10, 2, 1, FAKE + 4, None) == marsit.EALIGN
    assert lib.marsit_set_device_seed(None, 5, None) == marsit.EINVAL

    assert lib.marsit_step_apply(1, 4, FAKE, FAKE, None, FAKE, FAKE, 4, 64, 64, 1.0, 1, 0, None) == marsit.EINVAL   # no model
    assert lib.marsit_step_apply(1, 0, FAKE, FAKE, FAKE, FAKE + 1024, FAKE, 4, 64, 64, 1.0, 1, 0, None) == marsit.EINVAL   # K = 0
    assert lib.marsit_step_apply(1, 4, FAKE, FAKE, FAKE, FAKE, FAKE, 4, 64, 64, 1.0, 1, 0, None) == marsit.EINVAL   # x aliases update
    assert lib.marsit_step_apply(1, 4, FAKE, FAKE, FAKE + 2, None, FAKE, 4, 64, 64, 1.0, 1, 0, None) == marsit.EALIGN
    assert lib.marsit_step_apply(0, 4, FAKE, FAKE, FAKE + 2, None, FAKE, 4, 64, 64, 1.0, 1, 0, None) == marsit.EALIGN
    assert lib.marsit_step_apply(1, 4, FAKE, FAKE, FAKE, None, FAKE, 4, 64, 64, 1.0, 1, 3, None) == marsit.EINVAL   # 3 does not divide 4
    assert lib.marsit_step_apply(1, 4, FAKE, FAKE, FAKE, None, None, 4, 0, 64, 1.0, 1, 0, None) == marsit.OK
    assert lib.marsit_step_apply(0, 4, FAKE, FAKE, FAKE, None, None, 4, 0, 64, 1.0, 1, 0, None) == marsit.OK
    assert lib.marsit_apply_update(None, FAKE, 64, None) == marsit.EINVAL
    assert lib.marsit_apply_update(FAKE, FAKE, 0, None) == marsit.OK
    assert lib.marsit_local_momentum(FAKE, FAKE + 64, None, 2, 64, 64, 0.9, 0.1, None) == marsit.EINVAL
    assert lib.marsit_local_momentum(FAKE, FAKE, FAKE + 64, 2, 64, 64, 0.9, 0.1, None) == marsit.EINVAL   # buf aliases grad
    assert lib.marsit_local_momentum(FAKE, FAKE + 64, FAKE + 64, 2, 64, 32, 0.9, 0.1, None) == marsit.EINVAL   # ld < d
    assert lib.marsit_local_momentum(FAKE, FAKE + 64, FAKE + 64, 2, 64, 64, float("nan"), 0.1, None) == marsit.EINVAL
    assert lib.marsit_local_momentum(FAKE, FAKE + 62, FAKE + 64, 2, 64, 64, 0.9, 0.1, None) == marsit.EALIGN
    assert lib.marsit_local_momentum(FAKE, FAKE + 64, FAKE + 64, 2, 0, 64, 0.9, 0.1, None) == marsit.OK
    adam = lib.marsit_local_adam
    ok_args = (2, 64, 64, 0.9, 0.999, 1e-8, 0.1, 0.1, 0.001, None)
    assert adam(FAKE, FAKE + 1024, FAKE + 2048, None, *ok_args) == marsit.EINVAL
    assert adam(FAKE, FAKE, FAKE + 2048, FAKE + 2048, *ok_args) == marsit.EINVAL                 # moments alias
    assert adam(FAKE, FAKE + 1024, FAKE, FAKE + 2048, *ok_args) == marsit.EINVAL                 # moment aliases grad
    assert adam(FAKE, FAKE + 1024, FAKE + 2048, FAKE + 1024, *ok_args) == marsit.EINVAL          # moment aliases output
    assert adam(FAKE, FAKE + 1024, FAKE + 2048, FAKE + 2048, 2, 64, 32, 0.9, 0.999, 1e-8, 0.1, 0.1, 0.001, None) == marsit.EINVAL
    assert adam(FAKE, FAKE + 1024, FAKE + 2048, FAKE + 2048, 2, 64, 64, 0.9, 0.999, 1e-8, 0.1, 0.0, 0.001, None) == marsit.EINVAL   # bias1 = 0
    assert adam(FAKE, FAKE + 1024, FAKE + 2048, FAKE + 2048, 2, 64, 64, 0.9, float("inf"), 1e-8, 0.1, 0.1, 0.001, None) == marsit.EINVAL
    assert adam(FAKE, FAKE + 1022, FAKE + 2048, FAKE + 2048, *ok_args) == marsit.EALIGN
    assert adam(FAKE, FAKE + 1024, FAKE + 2048, FAKE + 2048, 2, 0, 64, 0.9, 0.999, 1e-8, 0.1, 0.1, 0.001, None) == marsit.OK


def test_missing_library_fails_loudly(tmp_path):
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        marsit.load_library(str(tmp_path / "libmarsit.so"))


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2204_06787_amd")
    for dirpath, _, files in os.walk(pkg):
        for name in files:
            if name.endswith((".py", ".hip", ".hpp", ".h", ".cpp")):
                text = open(os.path.join(dirpath, name)).read()
                assert "oracle" not in text.lower() or name == "workloads.py", name
    text = open(os.path.join(pkg, "workloads.py")).read()
    assert "import oracle" not in text and "from oracle" not in text


def test_header_is_valid_c(tmp_path):
    """include/marsit.h compiles as plain C11 (the boundary has no C++ in it)."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    src = tmp_path / "use_header.c"
    src.write_text('#include "marsit.h"\nint main(void) { return marsit_version() == 0; }\n')
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    proc = subprocess.run(["gcc", "-std=c11", "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only",
                           "-I", os.path.join(root, "include"), str(src)], capture_output=True, text=True)
    assert proc.returncode == 0, proc.stderr


def test_bench_refuses_more_than_one_gpu():
    """bench.py times one GPU's share; asking for more exits with a message that says so (before
    anything touches a GPU)."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    proc = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                          capture_output=True, text=True, timeout=120)
    assert proc.returncode != 0
    assert "ONE GPU" in proc.stderr and "--gpus must be 1" in proc.stderr
    assert proc.stdout.strip() == ""


def test_bench_byte_model_and_traffic_lookup(tmp_path, monkeypatch):
    """bench.py's algorithmic bytes are the stated per-element figures, and roofline.traffic is
    taken from a counter summary only when that summary was made from this tree's kernel sources."""
    import importlib
    import sys
    if ROOT not in sys.path:
        sys.path.insert(0, ROOT)
    bench = importlib.import_module("bench")
    M, d = 8, 25_600_000
    assert bench.algorithmic_bytes("ring_step_sim", M, d) == 12 * M * d + 4 * d + d // 8 == 2_563_200_000
    assert bench.algorithmic_bytes("tree_step_sim", M, d) == 2_563_200_000
    assert bench.algorithmic_bytes("full_sync", M, d) == 12 * M * d + 4 * d
    assert bench.algorithmic_bytes("step_apply", M, d) == 12 * M * d + 8 * d + d // 8
    assert bench.algorithmic_bytes("ring_step_sim", 3, 65) == 12 * 3 * 65 + 4 * 65 + 16     # ragged: 2 words

    from paper_2204_06787_amd import build
    digest = build.fused_sources_digest()
    assert len(digest) == 16 and int(digest, 16) >= 0
    prof = tmp_path / "profiles"
    prof.mkdir()
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    key = "entry=ring_step_sim M=8 d=25600000 grid_x=0 ld_pad=0"
    assert bench.measured_traffic(key)[0] is None                                   # nothing there
    (prof / "a.txt").write_text(f"x\nkey: {key}\ntraffic_bytes_per_launch: 123456\nfused_sources_sha16: {digest}\n")
    assert bench.measured_traffic(key) == (123456, os.path.join("profiles", "a.txt"))
    assert bench.measured_traffic(key.replace("M=8", "M=9"))[0] is None             # another shape
    (prof / "a.txt").write_text(f"key: {key}\ntraffic_bytes_per_launch: 123456\nfused_sources_sha16: {'0' * 16}\n")
    value, why = bench.measured_traffic(key)
    assert value is None and "other kernel sources" in why                          # stale summary

"""Parity of the HIP path against the CPU oracle, through the C ABI, on the same seeded inputs.

Bar: packed bitmaps, merged signs and decoded updates bit-exact; compensation within 1e-6 relative
(checked, and additionally bit for bit because each value is one fp32 rounding of the same
operands on both sides).
"""

import numpy as np
import pytest
import torch

from oracle import marsit_oracle as orc
from paper_2204_06787_amd import marsit, workloads
from gpu_util import (assert_f32_parity, dev, fused_step, host_bits, host_f32, oracle_step,
                      unaligned_rows, unfused_step)

pytestmark = pytest.mark.gpu

SPECIALS = np.array([0.0, -0.0, np.inf, -np.inf, 1e-45, -1e-45, 1e-40, -1e-40, 3.4e38, -3.4e38,
                     1.17549435e-38, -1.17549435e-38], dtype=np.float32)


def _inputs(M, d, ld=None, seed=0, c_scale=0.3):
    ld = d if ld is None else ld
    rng = np.random.default_rng(seed * 7919 + M * 131 + d)
    g = rng.standard_normal((M, ld)).astype(np.float32)
    c = (c_scale * rng.standard_normal((M, ld))).astype(np.float32)
    return g, c


# ------------------------------------------------------------------------------------------------
# marsit_compress
# ------------------------------------------------------------------------------------------------

@pytest.mark.parametrize("d", [1, 2, 63, 64, 65, 255, 256, 257, 1023, 4097, 65536 + 5, 1_000_003])
@pytest.mark.parametrize("with_c", [True, False])
def test_compress(d, with_c):
    g, c = _inputs(1, d, seed=1)
    g, c = g[0], c[0]
    n = min(d, SPECIALS.size)
    g[:n] = SPECIALS[:n]
    c[:n] = 0.0
    if d > 40:
        g[20:30] = 1.5
        c[20:30] = -1.5          # exact cancellation -> +0 -> bit 1
    want = orc.sign_pack(orc.add_compensation(g, c if with_c else None))
    bits = marsit.new_bitmap(d)
    bits.fill_(-1)
    marsit.marsit_compress(dev(g), dev(c) if with_c else None, bits, d=d)
    torch.cuda.synchronize()
    assert np.array_equal(host_bits(bits), want)


def test_compress_unaligned_pointer():
    d = 5000
    g, c = _inputs(1, d + 3, seed=2)
    gd, cd = dev(g[0]), dev(c[0])
    for off in (1, 2, 3):
        want = orc.sign_pack(orc.add_compensation(np.ascontiguousarray(g[0, off:off + d]),
                                                  np.ascontiguousarray(c[0, off:off + d])))
        bits = marsit.new_bitmap(d)
        marsit.marsit_compress(gd[off:off + d], cd[off:off + d], bits, d=d)
        torch.cuda.synchronize()
        assert np.array_equal(host_bits(bits), want)


# ------------------------------------------------------------------------------------------------
# marsit_hop_merge
# ------------------------------------------------------------------------------------------------

@pytest.mark.parametrize("n_words", [1, 2, 15, 16, 17, 63, 1000, 50_000])
@pytest.mark.parametrize("fold,hop", [(1, 0), (2, 1), (3, 2), (5, 4), (8, 7), (16, (1 << 16) | 3),
                                      (4, (3 << 8) | 3), (64, 63)])
def test_hop_merge(n_words, fold, hop):
    rng = np.random.default_rng(n_words * 100 + fold)
    recv = rng.integers(0, 2**64, size=n_words, dtype=np.uint64)
    local = rng.integers(0, 2**64, size=n_words, dtype=np.uint64)
    seed = 0xABCDEF0123456789
    for word_begin in (0, 341, (1 << 33) + 7):
        want = orc.hop_merge(recv, local, word_begin, fold, hop, seed)
        out = torch.zeros(n_words, dtype=torch.int64, device="cuda")
        marsit.marsit_hop_merge(dev(recv), dev(local), out, word_begin, n_words, fold, hop, seed)
        torch.cuda.synchronize()
        assert np.array_equal(host_bits(out), want), (word_begin,)


def test_hop_merge_in_place():
    rng = np.random.default_rng(3)
    n = 777
    recv = rng.integers(0, 2**64, size=n, dtype=np.uint64)
    local = rng.integers(0, 2**64, size=n, dtype=np.uint64)
    want = orc.hop_merge(recv, local, 12, 3, 2, 99)
    r, l = dev(recv), dev(local)
    marsit.marsit_hop_merge(r, l, r, 12, n, 3, 2, 99)           # out aliases recv
    torch.cuda.synchronize()
    assert np.array_equal(host_bits(r), want)
    assert np.array_equal(host_bits(l), local)
    r2 = dev(recv)
    marsit.marsit_hop_merge(r2, l, l, 12, n, 3, 2, 99)          # out aliases local
    torch.cuda.synchronize()
    assert np.array_equal(host_bits(l), want)


# ------------------------------------------------------------------------------------------------
# marsit_decode_compensate
# ------------------------------------------------------------------------------------------------

@pytest.mark.parametrize("d", [1, 3, 4, 5, 63, 64, 65, 1023, 4100, 100_003])
@pytest.mark.parametrize("offset", [0, 1])
def test_decode_compensate(d, offset):
    rng = np.random.default_rng(d)
    g, c = _inputs(1, d + 1, seed=4)
    g1 = np.ascontiguousarray(g[0, offset:offset + d])
    c1 = np.ascontiguousarray(c[0, offset:offset + d])
    n = min(d, SPECIALS.size)
    g1[:n] = SPECIALS[:n]
    c1[:n] = 0.0
    bits = rng.integers(0, 2**64, size=orc.n_words(d), dtype=np.uint64)
    scale = 2.5e-3
    want_u = orc.decode(bits, scale, d)
    want_c = orc.compensate(orc.add_compensation(g1, c1), want_u)

    gd = torch.zeros(d + 1, dtype=torch.float32, device="cuda")
    cd = torch.zeros(d + 1, dtype=torch.float32, device="cuda")
    gd[offset:offset + d] = dev(g1)
    cd[offset:offset + d] = dev(c1)
    ud = torch.zeros(d + 1, dtype=torch.float32, device="cuda")
    gv, cv, uv = gd[offset:offset + d], cd[offset:offset + d], ud[offset:offset + d]
    marsit.marsit_decode_compensate(dev(bits), gv, cv, scale, uv, cv, d=d)      # in place on c
    torch.cuda.synchronize()
    assert np.array_equal(host_f32(uv).view(np.uint32), want_u.view(np.uint32))
    assert_f32_parity(host_f32(cv), want_c, "c_out")

    # c = NULL and update_out = NULL
    want_c0 = orc.compensate(orc.add_compensation(g1, None), want_u)
    out = torch.zeros(d, dtype=torch.float32, device="cuda")
    marsit.marsit_decode_compensate(dev(bits), gv, None, scale, None, out, d=d)
    torch.cuda.synchronize()
    assert_f32_parity(host_f32(out), want_c0, "c_out (c = NULL)")


@pytest.mark.parametrize("d", [1, 3, 4, 5, 63, 64, 65, 1023, 4100, 100_003])
@pytest.mark.parametrize("offset", [0, 1])
def test_decode_compensate_apply(d, offset):
    """Decode, compensation update and model update in one pass = the oracle's three steps."""
    rng = np.random.default_rng(d + 7)
    g, c = _inputs(1, d + 1, seed=5)
    g1 = np.ascontiguousarray(g[0, offset:offset + d])
    c1 = np.ascontiguousarray(c[0, offset:offset + d])
    x1 = rng.standard_normal(d).astype(np.float32)
    bits = rng.integers(0, 2**64, size=orc.n_words(d), dtype=np.uint64)
    scale = 2.5e-3
    want_u = orc.decode(bits, scale, d)
    want_c = orc.compensate(orc.add_compensation(g1, c1), want_u)
    want_x = orc.apply_update(x1.copy(), want_u)

    buf = [torch.zeros(d + 1, dtype=torch.float32, device="cuda") for _ in range(4)]
    gv, cv, xv, uv = (b[offset:offset + d] for b in buf)
    gv.copy_(dev(g1))
    cv.copy_(dev(c1))
    xv.copy_(dev(x1))
    marsit.marsit_decode_compensate_apply(dev(bits), gv, cv, scale, xv, uv, cv, d=d)
    torch.cuda.synchronize()
    assert np.array_equal(host_f32(uv).view(np.uint32), want_u.view(np.uint32))
    assert_f32_parity(host_f32(cv), want_c, "c_out")
    assert_f32_parity(host_f32(xv), want_x, "x")
    # without the update output: a second application moves the model once more
    cv.copy_(dev(c1))
    marsit.marsit_decode_compensate_apply(dev(bits), gv, cv, scale, xv, None, cv, d=d)
    torch.cuda.synchronize()
    assert_f32_parity(host_f32(xv), orc.apply_update(want_x.copy(), want_u), "x (second round)")
    assert_f32_parity(host_f32(cv), want_c, "c_out (second round)")


# ------------------------------------------------------------------------------------------------
# fused pass vs oracle
# ------------------------------------------------------------------------------------------------

def _check_fused(M, d, grid_x, ld=None, aligned=True, scale=1e-3, seed=0x5EED, steps=1, specials=False):
    ld = d if ld is None else ld
    g_h, c_h = _inputs(M, d, ld=ld, seed=seed & 0xFFFF)
    if specials and d >= SPECIALS.size:
        for m in range(M):
            g_h[m, :SPECIALS.size] = np.roll(SPECIALS, m)
            c_h[m, :SPECIALS.size] = 0.0
    if aligned:
        g_d, c_d = dev(g_h), dev(c_h)
    else:
        g_d, c_d = unaligned_rows(M, ld), unaligned_rows(M, ld)
        g_d.copy_(dev(g_h))
        c_d.copy_(dev(c_h))
    c_before_pad = c_h[:, d:].copy()
    for t in range(steps):
        sd = workloads.step_seed(seed, t)
        want_u, want_b, _ = oracle_step(g_h, c_h, scale, sd, grid_x=grid_x, d=d)
        got_u, got_b = fused_step(g_d, c_d, scale, sd, grid_x=grid_x, d=d)
        assert np.array_equal(host_bits(got_b), want_b), f"bitmap, step {t}"
        assert np.array_equal(host_f32(got_u).view(np.uint32), want_u.view(np.uint32)), f"update, step {t}"
        assert_f32_parity(host_f32(c_d)[:, :d], c_h[:, :d], f"compensation, step {t}")
    if ld > d:
        assert np.array_equal(host_f32(c_d)[:, d:], c_before_pad), "padding columns were touched"


def test_tiny_ring_config():
    """M=3, d=65,536, N(0,1), c=0, scale 1e-3, one step."""
    wl = workloads.WORKLOADS["tiny_ring"]
    g = workloads.make_gradients(wl, 0, seed=1, device="cuda")
    c = workloads.zero_compensation(wl, device="cuda")
    g_h, c_h = host_f32(g).copy(), host_f32(c).copy()
    sd = workloads.step_seed(2022, 0)
    want_u, want_b, want_maps = orc.sync_step(g_h, c_h, wl.scale, sd, want_sign_maps=True)
    got_u, got_b = fused_step(g, c, wl.scale, sd)
    assert np.array_equal(host_bits(got_b), want_b)
    assert np.array_equal(host_f32(got_u).view(np.uint32), want_u.view(np.uint32))
    assert_f32_parity(host_f32(c), c_h, "compensation")
    # the un-fused chain gives the same, and its per-worker bitmaps are the oracle's
    c2 = workloads.zero_compensation(wl, device="cuda")
    u2, b2, maps = unfused_step(g, c2, wl.scale, sd)
    for m in range(wl.M):
        assert np.array_equal(host_bits(maps[m]), want_maps[m])
    assert np.array_equal(host_bits(b2), want_b)
    assert torch.equal(u2, got_u) and torch.equal(c2, c)


@pytest.mark.parametrize("d", [1, 3, 4, 5, 63, 64, 65, 255, 1023, 1024, 4100, 16384 + 1, 100_003])
@pytest.mark.parametrize("M", [1, 2, 3, 5, 8, 16])
def test_fused_ring_shapes(M, d):
    _check_fused(M, d, grid_x=0, seed=0x1000 + M)


@pytest.mark.parametrize("X,Y", [(2, 2), (3, 2), (2, 3), (4, 2), (2, 4), (3, 3), (4, 4)])
@pytest.mark.parametrize("d", [5, 64, 1000, 64 * 4 * 16 + 3, 50_001])
def test_fused_torus_shapes(X, Y, d):
    _check_fused(X * Y, d, grid_x=X, seed=0x2000 + X * 10 + Y)


@pytest.mark.parametrize("M", [4, 6, 7, 9, 10, 11, 12, 13, 14, 15])
@pytest.mark.parametrize("d", [64 * 7 + 5, 100_003])
def test_fused_ring_every_compiled_worker_count(M, d):
    _check_fused(M, d, grid_x=0, seed=0x1800 + M)


@pytest.mark.parametrize("M,grid_x", [(10, 5), (10, 2), (24, 6), (64, 0), (64, 8), (7, 1), (17, 0), (20, 4), (21, 7),
                                      (33, 0), (40, 0), (41, 0), (48, 6), (48, 0), (49, 0), (49, 7), (60, 5), (63, 0)])
@pytest.mark.parametrize("d", [7, 640, 33_333])
def test_fused_generic_schedule(M, grid_x, d):
    """Schedules without a compiled specialisation run the any-schedule kernels: staged in LDS in
    batches of 4, 8 or 16 workers up to 48 workers, gather-and-sweep above; tori of up to four rows
    share the row draws among a lane's bits, taller ones draw per bit."""
    _check_fused(M, d, grid_x=grid_x, seed=0x3000 + M)


@pytest.mark.parametrize("M,grid_x", [(8, 0), (16, 4), (3, 0)])
def test_fused_results_do_not_depend_on_the_occupancy_hook(M, grid_x):
    """marsit_set_fused_waves_per_cu only changes how many workgroups share a CU."""
    try:
        for waves in (2, 3, 5, 8, 32):
            marsit.marsit_set_fused_waves_per_cu(waves)
            _check_fused(M, 64 * 300 + 9, grid_x=grid_x, seed=0x7000 + M)
    finally:
        marsit.marsit_set_fused_waves_per_cu(0)


@pytest.mark.parametrize("M,grid_x", [(3, 0), (8, 0), (16, 4), (9, 3)])
@pytest.mark.parametrize("d,ld", [(1000, 1001), (4099, 4102), (64, 67), (20_000, 20_004)])
def test_fused_row_stride_and_misaligned_base(M, grid_x, d, ld):
    _check_fused(M, d, grid_x=grid_x, ld=ld, seed=0x4000 + M)
    _check_fused(M, d, grid_x=grid_x, ld=ld, aligned=False, seed=0x4100 + M)


@pytest.mark.parametrize("M,grid_x", [(3, 0), (8, 0), (16, 4)])
def test_fused_special_values_and_scales(M, grid_x):
    for scale in (1e-3, -2.0, 0.0, 1e-42, 3.0e38):
        _check_fused(M, 4096 + 17, grid_x=grid_x, scale=scale, specials=True, seed=0x5000 + M)


@pytest.mark.parametrize("M,grid_x", [(3, 0), (8, 0), (16, 4), (12, 0)])
def test_fused_compensation_carried_over_steps(M, grid_x):
    _check_fused(M, 70_000 + 9, grid_x=grid_x, steps=4, seed=0x6000 + M)


def test_fused_without_bitmap_output():
    M, d = 8, 10_000
    g_h, c_h = _inputs(M, d, seed=7)
    g_d, c_d = dev(g_h), dev(c_h)
    want_u, _, _ = oracle_step(g_h, c_h, 1e-3, 5)
    got_u, _ = fused_step(g_d, c_d, 1e-3, 5, want_bits=False)
    assert np.array_equal(host_f32(got_u), want_u)
    assert_f32_parity(host_f32(c_d), c_h, "compensation")


def test_empty_input_is_a_no_op():
    lib = marsit.load_library()
    g = torch.ones(4, 8, device="cuda")
    c = torch.ones(4, 8, device="cuda")
    u = torch.ones(8, device="cuda")
    rc = lib.marsit_ring_step_sim(g.data_ptr(), c.data_ptr(), u.data_ptr(), None, 4, 0, 8, 1.0, 1, 0,
                                  torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert rc == 0 and bool((c == 1).all()) and bool((u == 1).all())


def test_runs_on_a_side_stream():
    M, d = 8, 200_000
    g_h, c_h = _inputs(M, d, seed=8)
    g_d, c_d = dev(g_h), dev(c_h)
    u = torch.empty(d, device="cuda")
    b = marsit.new_bitmap(d)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        marsit.marsit_ring_step_sim(g_d, c_d, u, b, 1e-3, 77)
    side.synchronize()
    want_u, want_b, _ = oracle_step(g_h, c_h, 1e-3, 77)
    assert np.array_equal(host_bits(b), want_b) and np.array_equal(host_f32(u), want_u)


def test_host_threads_on_their_own_streams():
    """Four host threads, each with its own stream and buffers, run carried steps of different
    shapes at the same time (the library keeps no mutable state between calls; its error slot is per
    thread).  Every thread's results equal the oracle's for its inputs."""
    import threading
    shapes = [(8, 0, 200_000), (16, 4, 90_001), (20, 0, 30_000), (5, 0, 123_457)]
    steps = 6
    work = []
    for k, (M, grid_x, d) in enumerate(shapes):
        g_h, c_h = _inputs(M, d, seed=100 + k)
        work.append({"M": M, "grid_x": grid_x, "d": d, "g_h": g_h, "c_h": c_h, "g": dev(g_h), "c": dev(c_h),
                     "u": [torch.empty(d, device="cuda") for _ in range(steps)],
                     "b": [marsit.new_bitmap(d) for _ in range(steps)], "stream": torch.cuda.Stream(), "error": None})
    torch.cuda.synchronize()
    print("threads:", [(w["M"], w["grid_x"], w["d"]) for w in work], flush=True)

    def run(w):
        try:
            for t in range(steps):
                marsit.marsit_ring_step_sim(w["g"], w["c"], w["u"][t], w["b"][t], 1e-3, 500 + t, grid_x=w["grid_x"],
                                            stream=w["stream"])
            w["stream"].synchronize()
        except Exception as exc:        # reported by the main thread
            w["error"] = exc

    threads = [threading.Thread(target=run, args=(w,)) for w in work]
    for th in threads:
        th.start()
    for th in threads:
        th.join(timeout=100)
        assert not th.is_alive(), "a worker thread did not finish"
    torch.cuda.synchronize()
    for w in work:
        assert w["error"] is None, w["error"]
        c_ref = w["c_h"].copy()
        for t in range(steps):
            want_u, want_b, _ = oracle_step(w["g_h"], c_ref, 1e-3, 500 + t, grid_x=w["grid_x"])
            what = f"M={w['M']} grid_x={w['grid_x']} d={w['d']} step {t}"
            assert np.array_equal(host_bits(w["b"][t]), want_b), what
            assert np.array_equal(host_f32(w["u"][t]).view(np.uint32), want_u.view(np.uint32)), what
        assert np.array_equal(host_f32(w["c"]).view(np.uint32), c_ref.view(np.uint32)), f"compensation, M={w['M']}"


# ------------------------------------------------------------------------------------------------
# fused pass == chain of the un-fused entry points (bit for bit), moderate sizes
# ------------------------------------------------------------------------------------------------

@pytest.mark.parametrize("M,grid_x,d", [(8, 0, 1_000_000 + 37), (16, 4, 500_000 + 1), (5, 0, 300_001),
                                        (6, 3, 250_000), (10, 5, 99_999)])
def test_fused_equals_unfused_chain(M, grid_x, d):
    g_h, c_h = _inputs(M, d, seed=9)
    g1, c1 = dev(g_h), dev(c_h)
    g2, c2 = dev(g_h), dev(c_h)
    u1, b1 = fused_step(g1, c1, 1e-3, 4242, grid_x=grid_x)
    u2, b2, _ = unfused_step(g2, c2, 1e-3, 4242, grid_x=grid_x)
    assert torch.equal(b1, b2) and torch.equal(u1, u2) and torch.equal(c1, c2)


# ------------------------------------------------------------------------------------------------
# the native hop-by-hop chain (marsit_chain_step_sim) vs oracle and vs the fused kernel
# ------------------------------------------------------------------------------------------------

@pytest.mark.parametrize("M,grid_x,d", [(3, 0, 65_536), (8, 0, 400_000 + 21), (16, 4, 200_003), (6, 3, 64 * 5 + 1),
                                        (5, 0, 7), (9, 3, 33_333), (4, 1, 5000), (12, 0, 100)])
def test_chain_step(M, grid_x, d):
    g_h, c_h = _inputs(M, d, seed=11)
    g1, c1 = dev(g_h), dev(c_h)
    g2, c2 = dev(g_h), dev(c_h)
    ws = torch.empty(marsit.marsit_chain_workspace_words(M, d, grid_x), dtype=torch.int64, device="cuda")
    u1 = torch.empty(d, dtype=torch.float32, device="cuda")
    b1 = marsit.new_bitmap(d)
    for t in range(2):
        sd = workloads.step_seed(909, t)
        marsit.marsit_chain_step_sim(g1, c1, u1, b1, ws, 1e-3, sd, grid_x=grid_x)
        u2, b2 = fused_step(g2, c2, 1e-3, sd, grid_x=grid_x)
        want_u, want_b, _ = oracle_step(g_h, c_h, 1e-3, sd, grid_x=grid_x)
        assert np.array_equal(host_bits(b1), want_b) and torch.equal(b1, b2)
        assert np.array_equal(host_f32(u1), want_u) and torch.equal(u1, u2)
        assert_f32_parity(host_f32(c1), c_h, "compensation (chain)")
        assert torch.equal(c1, c2)


@pytest.mark.parametrize("K,first,n_words,hop_base", [(1, 0, 100, 0), (2, 1, 1, 0), (3, 2, 17, 0), (8, 5, 3000, 0),
                                                      (4, 0, 999, 3 << 8), (4, 3, 64, 1 << 16), (64, 63, 130, 0),
                                                      (16, 7, 12_501, 2 << 8)])
def test_fold_segments(K, first, n_words, hop_base):
    """The owner-side fold of K received segments in one launch = the oracle's chain of K - 1 hop
    merges in the same order (start at `first`, hop h folds operand (first + h) mod K)."""
    rng = np.random.default_rng(K * 1000 + n_words)
    stride = n_words + 5                                           # operands need not be densely packed
    maps_h = rng.integers(0, 2**64, size=(K, stride), dtype=np.uint64)
    word_begin, seed = 77_000, 0x1234ABCD5678
    want = maps_h[first, :n_words].copy()
    for h in range(1, K):
        want = orc.hop_merge(want, np.ascontiguousarray(maps_h[(first + h) % K, :n_words]), word_begin, h + 1,
                             hop_base | h, seed)
    out = torch.full((n_words + 2,), -1, dtype=torch.int64, device="cuda")
    marsit.marsit_fold_segments(dev(maps_h), K, first, out[:n_words], word_begin, n_words, hop_base, seed)
    torch.cuda.synchronize()
    assert np.array_equal(host_bits(out[:n_words]), want)
    assert bool((out[n_words:] == -1).all())                       # nothing written past the segment


@pytest.mark.parametrize("M,grid_x,d", [(3, 0, 65_536), (8, 0, 400_000 + 21), (16, 4, 200_003), (6, 3, 64 * 5 + 1),
                                        (5, 0, 7), (9, 3, 33_333), (4, 1, 5000), (12, 0, 100), (64, 8, 70_001),
                                        (1, 0, 1000)])
def test_exchange_step(M, grid_x, d):
    """One exchange step (signs, one fold per part, decode) against the oracle and the fused pass."""
    g_h, c_h = _inputs(M, d, seed=16)
    g1, c1 = dev(g_h), dev(c_h)
    g2, c2 = dev(g_h), dev(c_h)
    ws = torch.empty(marsit.marsit_chain_workspace_words(M, d, grid_x), dtype=torch.int64, device="cuda")
    u1 = torch.empty(d, dtype=torch.float32, device="cuda")
    b1 = marsit.new_bitmap(d)
    for t in range(2):
        sd = workloads.step_seed(606, t)
        marsit.marsit_exchange_step_sim(g1, c1, u1, b1, ws, 1e-3, sd, grid_x=grid_x)
        u2, b2 = fused_step(g2, c2, 1e-3, sd, grid_x=grid_x)
        want_u, want_b, _ = oracle_step(g_h, c_h, 1e-3, sd, grid_x=grid_x)
        assert np.array_equal(host_bits(b1), want_b) and torch.equal(b1, b2)
        assert np.array_equal(host_f32(u1), want_u) and torch.equal(u1, u2)
        assert_f32_parity(host_f32(c1), c_h, "compensation (exchange step)")
        assert torch.equal(c1, c2)


# ------------------------------------------------------------------------------------------------
# the ring as M workers on M streams (marsit_pipeline_*) vs oracle and vs the fused kernel
# ------------------------------------------------------------------------------------------------

@pytest.mark.parametrize("M,d", [(1, 1000), (2, 64 * 9 + 3), (3, 65_536), (5, 7), (8, 400_000 + 21), (8, 64 * 3),
                                 (16, 200_003)])
def test_ring_pipeline(M, d):
    g_h, c_h = _inputs(M, d, seed=12)
    g1, c1 = dev(g_h), dev(c_h)
    g2, c2 = dev(g_h), dev(c_h)
    u1 = torch.empty(d, dtype=torch.float32, device="cuda")
    b1 = marsit.new_bitmap(d)
    with marsit.RingPipeline(M) as pipe:
        ws = torch.empty(pipe.workspace_words(d), dtype=torch.int64, device="cuda")
        for t in range(3):                                   # the same events are used again every step
            sd = workloads.step_seed(4711, t)
            pipe.ring_step(g1, c1, u1, b1, ws, 1e-3, sd)
            torch.cuda.synchronize()
            u2, b2 = fused_step(g2, c2, 1e-3, sd)
            want_u, want_b, _ = oracle_step(g_h, c_h, 1e-3, sd)
            assert np.array_equal(host_bits(b1), want_b) and torch.equal(b1, b2), t
            assert np.array_equal(host_f32(u1), want_u) and torch.equal(u1, u2), t
            assert_f32_parity(host_f32(c1), c_h, f"compensation (pipeline), step {t}")


@pytest.mark.parametrize("M,X,d", [(8, 4, 400_000 + 21), (8, 2, 64 * 37 + 5), (16, 4, 200_003), (6, 3, 65_536),
                                   (6, 2, 7), (4, 1, 64 * 9 + 3), (4, 4, 1000), (12, 4, 64 * 5), (9, 3, 1),
                                   (64, 8, 70_001)])
def test_torus_pipeline(M, X, d):
    """Row rings, then column rings among the last holders, on one stream per worker."""
    g_h, c_h = _inputs(M, d, seed=14)
    g1, c1 = dev(g_h), dev(c_h)
    g2, c2 = dev(g_h), dev(c_h)
    u1 = torch.empty(d, dtype=torch.float32, device="cuda")
    b1 = marsit.new_bitmap(d)
    with marsit.RingPipeline(M) as pipe:
        ws = torch.empty(pipe.workspace_words(d, X), dtype=torch.int64, device="cuda")
        for t in range(3):
            sd = workloads.step_seed(815, t)
            pipe.step(g1, c1, u1, b1, ws, 1e-3, sd, grid_x=X)
            torch.cuda.synchronize()
            u2, b2 = fused_step(g2, c2, 1e-3, sd, grid_x=X)
            want_u, want_b, _ = oracle_step(g_h, c_h, 1e-3, sd, grid_x=X)
            assert np.array_equal(host_bits(b1), want_b) and torch.equal(b1, b2), t
            assert np.array_equal(host_f32(u1), want_u) and torch.equal(u1, u2), t
            assert_f32_parity(host_f32(c1), c_h, f"compensation (torus pipeline), step {t}")


def test_ring_pipeline_orders_with_the_callers_stream():
    """Work enqueued on the caller's stream after the step sees the results without a device sync."""
    M, d = 8, 300_000
    g_h, c_h = _inputs(M, d, seed=13)
    g1, c1 = dev(g_h), dev(c_h)
    u1 = torch.empty(d, dtype=torch.float32, device="cuda")
    b1 = marsit.new_bitmap(d)
    with marsit.RingPipeline(M) as pipe:
        ws = torch.empty(pipe.workspace_words(d), dtype=torch.int64, device="cuda")
        torch.cuda.synchronize()
        pipe.ring_step(g1, c1, u1, b1, ws, 1e-3, 5)
        u_copy = u1.clone()                                  # on the current stream, ordered after the step
        torch.cuda.synchronize()
    want_u, _, _ = oracle_step(g_h, c_h, 1e-3, 5)
    assert np.array_equal(host_f32(u_copy), want_u)


@pytest.mark.parametrize("n", [1, 3, 4, 63, 64, 65, 255, 1000, 64 * 300, 64 * 300 + 17, 1_000_003])
@pytest.mark.parametrize("fold,offset", [(1, 0), (2, 0), (5, 0), (8, 1)])
def test_compress_hop_merge(n, fold, offset):
    """The sign step fused into a merge = the oracle's sign-pack followed by its hop merge, from an
    aligned and from a misaligned base, with and without compensation, in place over recv."""
    rng = np.random.default_rng(n * 31 + fold)
    W = marsit.n_words(n)
    g_h = rng.standard_normal(n).astype(np.float32)
    c_h = (0.5 * rng.standard_normal(n)).astype(np.float32)
    recv_h = rng.integers(0, 2**64, size=W, dtype=np.uint64)
    if n % 64:
        recv_h[-1] &= np.uint64((1 << (n % 64)) - 1)
    word_begin, hop_id, seed = 123_456, (2 << 8) | 3, 0xABCDEF0123
    for with_c in (True, False):
        local = orc.sign_pack(orc.add_compensation(g_h, c_h if with_c else np.zeros_like(c_h)))
        want = orc.hop_merge(recv_h, local, word_begin, fold, hop_id, seed)
        if offset:
            g_d = unaligned_rows(1, n, offset)[0]
            g_d.copy_(dev(g_h))
            c_d = unaligned_rows(1, n, offset)[0]
            c_d.copy_(dev(c_h))
        else:
            g_d, c_d = dev(g_h), dev(c_h)
        out = dev(recv_h.copy())                       # in place over the received segment
        marsit.marsit_compress_hop_merge(out if fold > 1 else None, g_d, c_d if with_c else None, out,
                                         word_begin, fold, hop_id, seed)
        torch.cuda.synchronize()
        assert np.array_equal(host_bits(out), want), (n, fold, with_c)


def test_hop_merge_with_the_seed_in_device_memory():
    rng = np.random.default_rng(15)
    n = 3000
    recv = rng.integers(0, 2**64, size=n, dtype=np.uint64)
    local = rng.integers(0, 2**64, size=n, dtype=np.uint64)
    slot = torch.zeros(1, dtype=torch.int64, device="cuda")
    out = torch.zeros(n, dtype=torch.int64, device="cuda")
    for seed in (5, 0xFEDCBA9876543210):
        marsit.marsit_set_device_seed(slot, seed)
        marsit.marsit_hop_merge_device_seed(dev(recv), dev(local), out, 40, n, 4, 3, slot)
        torch.cuda.synchronize()
        assert np.array_equal(host_bits(out), orc.hop_merge(recv, local, 40, 4, 3, seed))


def test_device_seed_lets_a_captured_graph_be_replayed_with_new_seeds():
    """A caller's single-stream graph around hop merges whose seed lives in device memory: every
    replay uses the seed written just before it."""
    rng = np.random.default_rng(16)
    n = 20_000
    recv = rng.integers(0, 2**64, size=n, dtype=np.uint64)
    local = rng.integers(0, 2**64, size=n, dtype=np.uint64)
    r_d, l_d = dev(recv), dev(local)
    out = torch.zeros(n, dtype=torch.int64, device="cuda")
    slot = torch.zeros(1, dtype=torch.int64, device="cuda")
    marsit.marsit_set_device_seed(slot, 1)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        marsit.marsit_hop_merge_device_seed(r_d, l_d, out, 7, n, 3, 2, slot)      # warm-up
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        marsit.marsit_hop_merge_device_seed(r_d, l_d, out, 7, n, 3, 2, slot)
    for seed in (11, 0x123456789ABCDEF, 11):
        marsit.marsit_set_device_seed(slot, seed)
        graph.replay()
        torch.cuda.synchronize()
        assert np.array_equal(host_bits(out), orc.hop_merge(recv, local, 7, 3, 2, seed)), seed


def test_binding_rejects_short_or_strided_operands():
    """The kernels trust the sizes they are given, so the binding checks them on the host: nothing
    is launched for an operand that is too short or not contiguous."""
    M, d = 4, 1000
    g = torch.zeros((M, d), dtype=torch.float32, device="cuda")
    c = torch.zeros((M, d), dtype=torch.float32, device="cuda")
    u = torch.zeros(d, dtype=torch.float32, device="cuda")
    b = marsit.new_bitmap(d)
    with pytest.raises(ValueError):
        marsit.marsit_ring_step_sim(g, c, u[:d - 1], b, 1e-3, 1)
    with pytest.raises(ValueError):
        marsit.marsit_ring_step_sim(g, c, u, b[:-1], 1e-3, 1)
    with pytest.raises(ValueError):
        marsit.marsit_ring_step_sim(g, c, u, b, 1e-3, 1, d=d + 1)
    with pytest.raises(TypeError):
        marsit.marsit_ring_step_sim(g, c[:, ::2], u, b, 1e-3, 1)
    with pytest.raises(TypeError):
        marsit.marsit_compress(torch.zeros(2 * d, dtype=torch.float32, device="cuda")[::2], None, b)
    with pytest.raises(ValueError):
        marsit.marsit_compress(g[0], c[0], b[:3])
    with pytest.raises(ValueError):
        marsit.marsit_decode_compensate(b, g[0], c[0], 1e-3, u, c[0][:10])
    with pytest.raises(ValueError):
        marsit.marsit_hop_merge(b, b, b, 0, b.numel() + 1, 2, 1, 1)
    with pytest.raises(ValueError):
        marsit.marsit_step_apply(1, 2, g, c, u[:5], None, b, 1e-3, 1)
    with pytest.raises(ValueError):
        marsit.marsit_fold_segments(torch.zeros((3, 10), dtype=torch.int64, device="cuda"), 4, 0, b, 0, 10, 0, 1)
    with pytest.raises(TypeError):
        marsit.marsit_apply_update(u.double(), u)
    torch.cuda.synchronize()
    assert not u.any() and not c.any()


# ------------------------------------------------------------------------------------------------
# NaN inputs: outside the bit-for-bit contract at the NaN's own position, but they must not leak
# ------------------------------------------------------------------------------------------------

@pytest.mark.parametrize("M,grid_x,d", [(8, 0, 64 * 40 + 17), (16, 4, 64 * 33), (9, 0, 64 * 21 + 5), (7, 3, 64 * 19 + 63)])
def test_nan_elements_leave_their_neighbours_bit_exact(M, grid_x, d):
    """A NaN in one worker's element e can only change position e of the outputs (the sign of a NaN
    that an add produces is machine-dependent, so position e itself is outside the bit-for-bit
    contract).  Everything else -- the other 63 bits of the word, the other elements of every
    vector -- equals the oracle bit for bit, and position e still decodes to +-scale."""
    scale, seed = 2e-3, 4242
    rng = np.random.default_rng(d + M)
    g = rng.standard_normal((M, d)).astype(np.float32)
    c = (0.3 * rng.standard_normal((M, d))).astype(np.float32)
    planted = sorted(set(int(e) for e in rng.integers(0, d, size=12)) | {0, 63, 64, d - 1})
    for n, e in enumerate(planted):
        m = n % M
        if n % 3 == 0:
            g[m, e] = np.nan                                  # a NaN that is passed through
        elif n % 3 == 1:
            g[m, e], c[m, e] = np.inf, -np.inf                # a NaN that the add produces
        else:
            g[:, e] = np.nan                                  # NaN in every worker
    ragged = grid_x != 0 and M % grid_x != 0
    c_h = c.copy()
    with np.errstate(invalid="ignore"):
        if ragged:
            want_u, want_b = orc.ragged_torus_step(g, c_h, scale, seed, grid_x)
        else:
            want_u, want_b, _ = oracle_step(g, c_h, scale, seed, grid_x=grid_x)
    g_d, c_d = dev(g), dev(c)
    update = torch.empty(d, dtype=torch.float32, device="cuda")
    bits = marsit.new_bitmap(d)
    if ragged:
        marsit.marsit_ragged_torus_step_sim(g_d, c_d, update, bits, scale, seed, grid_x)
    else:
        marsit.marsit_ring_step_sim(g_d, c_d, update, bits, scale, seed, grid_x=grid_x)
    torch.cuda.synchronize()
    got_u, got_b, got_c = host_f32(update), host_bits(bits), host_f32(c_d)

    clean = np.ones(d, dtype=bool)
    clean[planted] = False
    assert np.array_equal(got_u.view(np.uint32)[clean], want_u.view(np.uint32)[clean])
    assert np.array_equal(got_c.view(np.uint32)[:, clean], c_h.view(np.uint32)[:, clean])
    mask = np.zeros(orc.n_words(d), dtype=np.uint64)                 # bit positions that are planted
    for e in planted:
        mask[e // 64] |= np.uint64(1) << np.uint64(e % 64)
    assert np.array_equal(got_b & ~mask, want_b & ~mask)
    # the planted positions: still a valid decode, consistent with the bitmap and the compensation
    with np.errstate(invalid="ignore"):
        s = g + c
    for e in planted:
        assert abs(got_u[e]) == np.float32(scale)
        bit = (int(got_b[e // 64]) >> (e % 64)) & 1
        assert (got_u[e] > 0) == bool(bit)
        for m in range(M):
            if np.isnan(s[m, e]):
                assert np.isnan(got_c[m, e])
            else:
                assert got_c[m, e] == np.float32(s[m, e] - got_u[e])

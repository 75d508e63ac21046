"""Pins for the CPU oracle: every check here compares the oracle with something that is NOT the
oracle -- the paper's stated properties, exact enumeration, closed forms, numpy routines, an
independently written second formulation, other people's Philox."""

import ctypes
import itertools
import os
import subprocess
import sys
from fractions import Fraction

import numpy as np
import pytest

from oracle import marsit_oracle as orc
import philox_ref

HERE = os.path.dirname(os.path.abspath(__file__))
MASK64 = (1 << 64) - 1


# ---------------------------------------------------------------------------------------------
# Philox: known answers, Python big-int transcription, PyTorch's host engine
# ---------------------------------------------------------------------------------------------

def _kat_rows():
    rows = []
    with open(os.path.join(HERE, "golden", "philox4x32_10_kat.txt")) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            v = [int(x, 16) for x in line.split()]
            rows.append((v[0:4], v[4:6], v[6:10]))
    return rows


def test_philox_known_answers():
    rows = _kat_rows()
    assert len(rows) == 3
    for ctr, key, want in rows:
        assert list(orc.philox4x32_10(ctr, key)) == want
        assert philox_ref.philox4x32_10(ctr, key) == want


def test_philox_matches_python_transcription():
    rng = np.random.default_rng(7)
    for _ in range(500):
        ctr = rng.integers(0, 2**32, size=4, dtype=np.uint64)
        key = rng.integers(0, 2**32, size=2, dtype=np.uint64)
        assert list(orc.philox4x32_10(ctr, key)) == philox_ref.philox4x32_10(ctr, key)


@pytest.fixture(scope="module")
def aten_philox(tmp_path_factory):
    import torch
    inc = os.path.join(os.path.dirname(torch.__file__), "include")
    src = os.path.join(HERE, "helpers", "aten_philox_probe.cpp")
    so = str(tmp_path_factory.mktemp("aten") / "aten_philox_probe.so")
    try:
        subprocess.run(["g++", "-O1", "-std=c++17", "-fPIC", "-shared", "-I" + inc, "-o", so, src],
                       check=True, capture_output=True)
    except (subprocess.CalledProcessError, FileNotFoundError) as exc:   # pragma: no cover
        pytest.skip(f"cannot compile the ATen Philox probe: {exc}")
    lib = ctypes.CDLL(so)
    lib.aten_philox4x32_10.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint64,
                                       ctypes.c_void_p]

    def call(seed, subsequence, offset):
        out = np.zeros(4, dtype=np.uint32)
        lib.aten_philox4x32_10(seed, subsequence, offset, out.ctypes.data_as(ctypes.c_void_p))
        return [int(x) for x in out]
    return call


def test_stream_matches_pytorch_engine(aten_philox):
    """stream (seed, hop, word)[j] == PyTorch's engine with subsequence = word index and
    offset = block | hop << 32 (its counter is (offset lo, offset hi, subseq lo, subseq hi))."""
    rng = np.random.default_rng(11)
    for _ in range(200):
        seed = int(rng.integers(0, 2**63)) * 2 + int(rng.integers(0, 2))
        hop = int(rng.integers(0, 2**20))
        word = int(rng.integers(0, 2**40))
        block = int(rng.integers(0, 16))
        want = aten_philox(seed, word, block | (hop << 32))
        got = [orc.stream_u32(seed, hop, word, 4 * block + k) for k in range(4)]
        assert got == want
        assert [philox_ref.stream_u32(seed, hop, word, 4 * block + k) for k in range(4)] == want


# ---------------------------------------------------------------------------------------------
# Eq. 2 and the operator: exact enumeration of the unbiasedness property (Section 4.1.1)
# ---------------------------------------------------------------------------------------------

def test_eq2_probabilities():
    """P(v=1) = 1/m where v*=1 and (m-1)/m where v*=0, when the keep-local draw has P = 1/m."""
    for m in range(1, 9):
        p_keep = Fraction(1, m)
        for l in (0, 1):
            p_v1 = Fraction(0)
            for t in (0, 1):
                w = p_keep if t else 1 - p_keep
                p_v1 += w * (orc.transient_from_keep(l, t) & 1)
            assert p_v1 == (Fraction(1, m) if l else Fraction(m - 1, m))


def test_odot_truth_table():
    """Same bit in both vectors: unchanged.  Different: the transient bit decides (Section 1)."""
    for r, l, v in itertools.product((0, 1), repeat=3):
        out = orc.odot(r, l, v) & 1
        assert out == (r if r == l else v)
    # word-wide: every bit position acts on its own
    rng = np.random.default_rng(3)
    for _ in range(50):
        r, l, v = (int(x) for x in rng.integers(0, 2**63, size=3, dtype=np.uint64) * 2 + 1)
        got = orc.odot(r, l, v)
        for j in range(64):
            rb, lb, vb = (r >> j) & 1, (l >> j) & 1, (v >> j) & 1
            assert (got >> j) & 1 == (rb if rb == lb else vb)


def _chain_prob_one(bits):
    """Exact P(final = 1) for a chain over workers with sign bits `bits`, fold count h+1 at hop h,
    enumerating every outcome of the keep-local draws with its rational weight."""
    M = len(bits)
    total = Fraction(0)
    for draws in itertools.product((0, 1), repeat=M - 1):
        weight = Fraction(1)
        r = bits[0]
        for h in range(1, M):
            m = h + 1
            t = draws[h - 1]
            weight *= Fraction(1, m) if t else Fraction(m - 1, m)
            v = orc.transient_from_keep(bits[h], t)
            r = orc.odot(r, bits[h], v) & 1
        total += weight * r
    return total


@pytest.mark.parametrize("M", [1, 2, 3, 4, 5, 6])
def test_exact_unbiasedness_ring(M):
    """Expected merged sign bit == mean of the workers' sign bits, for every sign pattern."""
    for bits in itertools.product((0, 1), repeat=M):
        assert _chain_prob_one(bits) == Fraction(sum(bits), M)


@pytest.mark.parametrize("X,Y", [(2, 2), (3, 2), (2, 3)])
def test_exact_unbiasedness_torus(X, Y):
    """Rows first (fold counts 2..X), then columns over the row results (fold counts 2..Y)."""
    M = X * Y
    n_draws = Y * (X - 1) + (Y - 1)
    for bits in itertools.product((0, 1), repeat=M):
        total = Fraction(0)
        for draws in itertools.product((0, 1), repeat=n_draws):
            it = iter(draws)
            weight = Fraction(1)
            rows = []
            for y in range(Y):
                r = bits[y * X]
                for h in range(1, X):
                    t = next(it)
                    weight *= Fraction(1, h + 1) if t else Fraction(h, h + 1)
                    l = bits[y * X + h]
                    r = orc.odot(r, l, orc.transient_from_keep(l, t)) & 1
                rows.append(r)
            r = rows[0]
            for k in range(1, Y):
                t = next(it)
                weight *= Fraction(1, k + 1) if t else Fraction(k, k + 1)
                r = orc.odot(r, rows[k], orc.transient_from_keep(rows[k], t)) & 1
            total += weight * r
        assert total == Fraction(sum(bits), M)


# ---------------------------------------------------------------------------------------------
# Empirical unbiasedness through the whole pass with the Philox stream (binomial bound)
# ---------------------------------------------------------------------------------------------

def _pattern_inputs(patterns, M, n_rep):
    """g[m, p*n_rep + r] has the sign given by bit m of patterns[p]."""
    d = len(patterns) * n_rep
    g = np.empty((M, d), dtype=np.float32)
    for p, pat in enumerate(patterns):
        for m in range(M):
            g[m, p * n_rep:(p + 1) * n_rep] = 1.0 if (pat >> m) & 1 else -1.0
    return g


@pytest.mark.parametrize("M,grid_x,patterns", [
    (2, 0, list(range(4))),
    (3, 0, list(range(8))),
    (5, 0, list(range(32))),
    (8, 0, [0x00, 0x01, 0x80, 0x03, 0x18, 0x0F, 0xF0, 0xAA, 0x55, 0x7F, 0xFE, 0xFF, 0x35]),
    (6, 3, [0, 1, 2, 4, 8, 16, 32, 7, 56, 21, 42, 63, 27]),
    (16, 4, [0x0001, 0x8000, 0x00FF, 0xFF00, 0x0F0F, 0x5555, 0x7FFF, 0x1248]),
])
def test_empirical_unbiasedness(M, grid_x, patterns):
    n_rep = 1 << 18
    g = _pattern_inputs(patterns, M, n_rep)
    c = np.zeros_like(g)
    update, bits, _ = orc.sync_step(g, c, scale=1.0, seed=0x1234_5678_9ABC_DEF0 + M, grid_x=grid_x,
                                    threads=8)
    plus = (update > 0).reshape(len(patterns), n_rep)
    for p, pat in enumerate(patterns):
        mean = bin(pat).count("1") / M
        bound = 5.0 * np.sqrt(max(mean * (1 - mean), 1e-12) / n_rep)
        assert abs(plus[p].mean() - mean) <= bound, (M, grid_x, hex(pat))


@pytest.mark.parametrize("fold", [1, 2, 3, 4, 5, 7, 8, 16])
def test_keep_mask_frequency_and_independence(fold):
    """P(t=1) = 1/m per bit position; neighbouring bits and neighbouring hops uncorrelated."""
    n_words = 4096
    seed = 99
    masks = np.array([orc.keep_mask(fold, 5, seed, w) for w in range(n_words)], dtype=np.uint64)
    bits = ((masks[:, None] >> np.arange(64, dtype=np.uint64)[None, :]) & np.uint64(1)).astype(np.float64)
    p = 1.0 / fold
    n = bits.size
    sigma = np.sqrt(p * (1 - p) / n) if fold > 1 else 0.0
    assert abs(bits.mean() - p) <= 5 * sigma + 1e-9
    if fold == 1:
        assert np.all(masks == np.uint64(MASK64))      # fold 1: always keep local
        return
    # per bit position
    per_pos = bits.mean(axis=0)
    assert np.all(np.abs(per_pos - p) <= 5 * np.sqrt(p * (1 - p) / n_words))
    # lag-1 correlation along the bit axis
    a, b = bits[:, :-1].ravel() - p, bits[:, 1:].ravel() - p
    corr = (a * b).mean() / (p * (1 - p))
    assert abs(corr) <= 5 / np.sqrt(a.size)
    # a different hop id gives an unrelated mask
    other = np.array([orc.keep_mask(fold, 6, seed, w) for w in range(n_words)], dtype=np.uint64)
    ob = ((other[:, None] >> np.arange(64, dtype=np.uint64)[None, :]) & np.uint64(1)).astype(np.float64)
    corr2 = ((bits - p) * (ob - p)).mean() / (p * (1 - p))
    assert abs(corr2) <= 5 / np.sqrt(n)


def test_keep_mask_threshold_definition():
    """t_j = (u_j < floor(2^32 / m)) with u_j from the independent Python Philox."""
    for fold, hop, seed, word in [(2, 1, 5, 0), (3, 2, 2**40 + 17, 123456789), (7, 0x10003, 1, 2**33 + 5)]:
        thr = (1 << 32) // fold
        want = 0
        for j in range(64):
            if philox_ref.stream_u32(seed, hop, word, j) < thr:
                want |= 1 << j
        assert orc.keep_mask(fold, hop, seed, word) == want


# ---------------------------------------------------------------------------------------------
# Identity / agreement cases
# ---------------------------------------------------------------------------------------------

def test_all_workers_equal_is_identity():
    rng = np.random.default_rng(5)
    d = 64 * 37 + 13
    row = rng.standard_normal(d).astype(np.float32)
    for M, gx in [(1, 0), (2, 0), (5, 0), (8, 0), (6, 2)]:
        g = np.tile(row, (M, 1))
        c = np.zeros_like(g)
        for seed in (0, 1, 2**63 + 5):
            update, bits, maps = orc.sync_step(g.copy(), c.copy(), 0.5, seed, grid_x=gx,
                                               want_sign_maps=True)
            assert np.array_equal(bits, maps[0])
            assert np.array_equal(update, np.where(np.signbit(row), np.float32(-0.5), np.float32(0.5)))


def test_fold_one_returns_local():
    rng = np.random.default_rng(6)
    recv = rng.integers(0, 2**63, size=33, dtype=np.uint64)
    local = rng.integers(0, 2**63, size=33, dtype=np.uint64)
    assert np.array_equal(orc.hop_merge(recv, local, 7, 1, 3, 42), local)


def test_two_workers_take_local_iff_top_bit_clear():
    """m = 2: threshold 2^31, so a differing bit takes the local sign iff u < 2^31."""
    seed, hop, word = 77, 1, 900
    recv, local = 0xAAAA_AAAA_5555_5555, 0x0F0F_0F0F_F0F0_F0F0
    got = orc.merge_word(recv, local, 2, hop, seed, word)
    for j in range(64):
        rb, lb = (recv >> j) & 1, (local >> j) & 1
        u = philox_ref.stream_u32(seed, hop, word, j)
        want = lb if (u >> 31) == 0 else rb
        assert (got >> j) & 1 == want


# ---------------------------------------------------------------------------------------------
# Second formulation (written independently): the final bit is the sign bit of the worker picked
# by the last successful keep-local draw of its chain ("reservoir" form)
# ---------------------------------------------------------------------------------------------

def _floor_bounds(begin, n, parts):
    return [begin + (i * n) // parts for i in range(parts + 1)]


def _part(w, bounds):
    for i in range(len(bounds) - 1):
        if bounds[i] <= w < bounds[i + 1]:
            return i
    raise AssertionError


def _reservoir_final_bits(signs, d, M, X, seed):
    """signs[m][e] in {0,1}.  Returns the final bit of every element, in pure Python."""
    Y = M // X
    W = (d + 63) // 64
    row_bounds = _floor_bounds(0, W, X)
    final = np.zeros(d, dtype=np.uint8)
    for e in range(d):
        w, j = divmod(e, 64)
        a = _part(w, row_bounds)
        picked_rows = []
        for y in range(Y):
            pick = 0
            for h in range(1, X):
                if philox_ref.stream_u32(seed, (0 << 16) | (y << 8) | h, w, j) < (1 << 32) // (h + 1):
                    pick = h
            picked_rows.append(signs[y * X + (a + pick) % X][e])
        col_bounds = _floor_bounds(row_bounds[a], row_bounds[a + 1] - row_bounds[a], Y)
        b = _part(w, col_bounds)
        pick = 0
        for k in range(1, Y):
            if philox_ref.stream_u32(seed, (1 << 16) | k, w, j) < (1 << 32) // (k + 1):
                pick = k
        final[e] = picked_rows[(b + pick) % Y]
    return final


@pytest.mark.parametrize("M,grid_x,d", [(3, 0, 64 * 10 + 5), (5, 0, 64 * 7), (8, 0, 64 * 9 + 63),
                                        (6, 3, 64 * 11 + 1), (4, 2, 64 * 5 + 17)])
def test_second_formulation(M, grid_x, d):
    rng = np.random.default_rng(100 + M)
    g = rng.standard_normal((M, d)).astype(np.float32)
    c = (0.3 * rng.standard_normal((M, d))).astype(np.float32)
    seed = 0xDEADBEEF00 + M
    s = g + c
    signs = (~np.signbit(s)).astype(np.uint8)
    want = _reservoir_final_bits(signs, d, M, grid_x or M, seed)
    update, bits, _ = orc.sync_step(g, c.copy(), 1.0, seed, grid_x=grid_x)
    got = ((bits[np.arange(d) // 64] >> (np.arange(d) % 64).astype(np.uint64)) & np.uint64(1)).astype(np.uint8)
    assert np.array_equal(got, want)
    assert np.array_equal(update > 0, want.astype(bool))


# ---------------------------------------------------------------------------------------------
# Packing, decode, compensation: numpy routines and closed forms
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("d", [1, 63, 64, 65, 64 * 20 + 7])
def test_sign_pack_matches_numpy_packbits(d):
    rng = np.random.default_rng(d)
    s = rng.standard_normal(d).astype(np.float32)
    s[rng.integers(0, d, size=max(1, d // 10))] = 0.0
    s[rng.integers(0, d, size=max(1, d // 10))] = -0.0
    bits = orc.sign_pack(s)
    padded = np.zeros(orc.n_words(d) * 64, dtype=np.uint8)
    padded[:d] = ~np.signbit(s)
    want = np.packbits(padded, bitorder="little").view("<u8")
    assert np.array_equal(bits, want)
    # round trip
    assert np.array_equal(orc.sign_unpack(bits, d), np.where(np.signbit(s), -1.0, 1.0).astype(np.float32))


def test_sign_special_values():
    s = np.array([0.0, -0.0, np.inf, -np.inf, 1e-45, -1e-45, 3.0, -3.0], dtype=np.float32)
    assert int(orc.sign_pack(s)[0]) == 0b01010101
    all_pos = np.full(130, 2.0, dtype=np.float32)
    b = orc.sign_pack(all_pos)
    assert [int(x) for x in b] == [MASK64, MASK64, 0b11]     # tail bits beyond d stay zero


def test_add_compensation_matches_numpy_float32():
    rng = np.random.default_rng(1)
    g = (rng.standard_normal(10_000) * 10.0 ** rng.integers(-30, 30, 10_000)).astype(np.float32)
    c = (rng.standard_normal(10_000) * 10.0 ** rng.integers(-30, 30, 10_000)).astype(np.float32)
    g[:4] = [1e-40, -1e-40, 1.0, -1.0]
    c[:4] = [1e-41, 1e-40, -1.0, 1.0]
    s = orc.add_compensation(g, c)
    assert np.array_equal(s.view(np.uint32), (g + c).view(np.uint32))     # bit for bit, denormals kept
    assert np.array_equal(orc.add_compensation(g, None).view(np.uint32), g.view(np.uint32))


def test_decode_closed_form():
    rng = np.random.default_rng(2)
    d = 64 * 13 + 29
    bits = rng.integers(0, 2**63, size=orc.n_words(d), dtype=np.uint64)
    scale = np.float32(3.25e-3)
    upd = orc.decode(bits, float(scale), d)
    assert set(np.unique(upd)) <= {scale, -scale}              # only {+eta_s, -eta_s}
    assert np.isclose(np.sum((upd / scale).astype(np.float64) ** 2), d)   # ||g_t / eta_s||^2 = D
    e = np.arange(d)
    bit = (bits[e // 64] >> (e % 64).astype(np.uint64)) & np.uint64(1)
    assert np.array_equal(upd > 0, bit.astype(bool))


def test_compensation_invariants_single_step():
    rng = np.random.default_rng(8)
    M, d = 5, 64 * 40 + 3
    g = rng.standard_normal((M, d)).astype(np.float32)
    c0 = (0.1 * rng.standard_normal((M, d))).astype(np.float32)
    c = c0.copy()
    update, _, _ = orc.sync_step(g, c, 1e-3, 4242)
    s = g + c0
    # compensation update: c_next = s - update, one fp32 rounding
    assert np.array_equal(c.view(np.uint32), (s - update[None, :]).view(np.uint32))
    # every worker subtracts the same global update
    assert np.allclose((c[0] - c[1]).astype(np.float64), (s[0].astype(np.float64) - s[1]), atol=2e-7 * 8)


def test_compensation_telescopes_over_steps():
    """Appendix B: mean_m c_T = sum_t (mean_m g_t - update_t) while no full-precision round occurs."""
    rng = np.random.default_rng(9)
    M, d, T = 4, 64 * 16, 12
    c = np.zeros((M, d), dtype=np.float32)
    acc = np.zeros(d, dtype=np.float64)
    for t in range(T):
        g = (0.01 * rng.standard_normal((M, d))).astype(np.float32)
        update, _, _ = orc.sync_step(g, c, 1e-3, 1000 + t)
        acc += g.astype(np.float64).mean(axis=0) - update.astype(np.float64)
    assert np.allclose(c.astype(np.float64).mean(axis=0), acc, atol=T * 4 * 2.0 ** -24 * 0.1)


def test_split_bounds_floor_rule():
    assert [int(x) for x in orc.split_bounds(0, 1024, 3)] == [0, 341, 682, 1024]
    assert [int(x) for x in orc.split_bounds(10, 7, 4)] == [10, 11, 13, 15, 17]
    b = orc.split_bounds(0, 2_156_250, 8)
    assert int(b[0]) == 0 and int(b[-1]) == 2_156_250
    assert all(int(b[i]) == (i * 2_156_250) // 8 for i in range(9))
    # fewer words than parts: some parts are empty, none is negative
    b = orc.split_bounds(0, 3, 8)
    assert int(b[-1]) == 3 and np.all(np.diff(b.astype(np.int64)) >= 0)


def test_padding_and_ld_are_ignored():
    rng = np.random.default_rng(10)
    M, d, ld = 3, 64 * 6 + 9, 64 * 7 + 4
    g = rng.standard_normal((M, ld)).astype(np.float32)
    c = rng.standard_normal((M, ld)).astype(np.float32)
    g2, c2 = np.ascontiguousarray(g[:, :d]), np.ascontiguousarray(c[:, :d])
    cpad = c.copy()
    u1, b1, _ = orc.sync_step(g, cpad, 0.01, 5, d=d)
    u2, b2, _ = orc.sync_step(g2, c2, 0.01, 5)
    assert np.array_equal(u1, u2) and np.array_equal(b1, b2)
    assert np.array_equal(cpad[:, :d], c2)
    assert np.array_equal(cpad[:, d:], c[:, d:])              # padding untouched
    assert int(b1[-1]) >> (d % 64) == 0                        # tail bits zero


def test_threads_do_not_change_results():
    rng = np.random.default_rng(12)
    g = rng.standard_normal((8, 64 * 50 + 1)).astype(np.float32)
    c1 = np.zeros_like(g)
    c2 = np.zeros_like(g)
    u1, b1, _ = orc.sync_step(g, c1, 1e-3, 31337, threads=1)
    u2, b2, _ = orc.sync_step(g, c2, 1e-3, 31337, threads=4)
    assert np.array_equal(u1, u2) and np.array_equal(b1, b2) and np.array_equal(c1, c2)


def test_hop_merge_composes_to_sync_step():
    """Chaining the single-hop routine along the ring schedule reproduces the whole pass."""
    rng = np.random.default_rng(13)
    M, d = 4, 64 * 23 + 40
    g = rng.standard_normal((M, d)).astype(np.float32)
    c = np.zeros_like(g)
    seed = 2024
    update, bits, maps = orc.sync_step(g, c, 1.0, seed, want_sign_maps=True)
    W = orc.n_words(d)
    bounds = [int(x) for x in orc.split_bounds(0, W, M)]
    final = np.zeros(W, dtype=np.uint64)
    for i in range(M):
        lo, hi = bounds[i], bounds[i + 1]
        r = maps[i, lo:hi].copy()
        for h in range(1, M):
            r = orc.hop_merge(r, np.ascontiguousarray(maps[(i + h) % M, lo:hi]), lo, h + 1, h, seed)
        final[lo:hi] = r
    assert np.array_equal(final, bits)


# ---------------------------------------------------------------------------------------------
# Full-precision round (Algorithm 1, branch mod(t,K) == 0) and model update (Algorithm 2)
# ---------------------------------------------------------------------------------------------

def test_full_sync_is_the_mean_and_resets_compensation():
    rng = np.random.default_rng(14)
    M, d = 8, 1000
    g = rng.standard_normal((M, d)).astype(np.float32)
    c = rng.standard_normal((M, d)).astype(np.float32)
    want = ((g + c).astype(np.float64).mean(axis=0)).astype(np.float32)
    upd = orc.full_sync(g, c)
    assert np.array_equal(upd, want)
    assert not c.any()


def test_average_bits_per_element_table():
    """Fig. 4(b): one full-precision round (32 bits) every K rounds, one bit otherwise."""
    printed = {50: 1.62, 100: 1.31, 200: 1.16}
    for K, bits in printed.items():
        assert round((K - 1 + 32) / K, 2) == bits


def test_apply_update():
    x = np.array([1.0, 2.0, -3.0], dtype=np.float32)
    u = np.array([0.5, -0.5, 0.25], dtype=np.float32)
    assert np.array_equal(orc.apply_update(x, u), np.array([0.5, 2.5, -3.25], dtype=np.float32))


def test_local_momentum_geometric_closed_form():
    """Constant gradient 1, beta = 1/2: buf_t = 2 - 2^(1-t) exactly (every value is a short binary
    fraction), g_t = eta_l * buf_t; a gradient of -3 in another worker scales the same series."""
    buf = np.zeros((2, 5), dtype=np.float32)
    grad = np.empty((2, 5), dtype=np.float32)
    grad[0] = 1.0
    grad[1] = -3.0
    grad[:, 4] = 777.0                      # column >= d: never read, never written
    for t in range(1, 20):
        g = orc.local_momentum(buf, grad, 0.5, 0.25, d=4)
        want = 2.0 - 2.0 ** (1 - t)
        assert np.all(buf[0, :4] == np.float32(want)) and np.all(buf[1, :4] == np.float32(-3.0 * want))
        assert np.all(g[0, :4] == np.float32(0.25 * want)) and np.all(g[1, :4] == np.float32(-0.75 * want))
        assert np.all(buf[:, 4] == 0.0) and np.all(g[:, 4] == 12345.0)


def test_local_momentum_special_cases():
    """beta = 0 is plain scaling of the gradient; beta = 1 with eta_l = 1 is a running sum."""
    rng = np.random.default_rng(77)
    grad = rng.standard_normal((3, 1000)).astype(np.float32)
    buf = rng.standard_normal((3, 1000)).astype(np.float32)
    g = orc.local_momentum(buf, grad, 0.0, 0.1)
    assert np.array_equal(buf, grad) and np.array_equal(g, np.float32(0.1) * grad)
    total = np.zeros_like(grad)
    acc = np.zeros_like(grad)
    for _ in range(5):
        step = rng.integers(-8, 9, size=grad.shape).astype(np.float32)      # integers: sums are exact
        total += step
        g = orc.local_momentum(acc, step, 1.0, 1.0)
        assert np.array_equal(acc, total) and np.array_equal(g, total)


def test_local_momentum_matches_torch_sgd_buffer():
    """The heavy-ball buffer is the one torch.optim.SGD keeps (dampening 0): with lr = eta_l the
    parameter moves by -g every step.  torch fuses nothing here on CPU, so agreement is to rounding."""
    import torch
    rng = np.random.default_rng(78)
    x0 = rng.standard_normal(500).astype(np.float32)
    p = torch.nn.Parameter(torch.from_numpy(x0.copy()))
    opt = torch.optim.SGD([p], lr=0.05, momentum=0.9)
    buf = np.zeros((1, 500), dtype=np.float32)
    x = x0.astype(np.float64)
    for t in range(6):
        grad = rng.standard_normal((1, 500)).astype(np.float32)
        p.grad = torch.from_numpy(grad[0].copy())
        opt.step()
        g = orc.local_momentum(buf, grad, 0.9, 0.05)
        x = x - g[0].astype(np.float64)
        assert np.allclose(p.detach().numpy(), x, rtol=0, atol=2e-6 * (t + 1))


def test_local_adam_sign_like_special_case():
    """beta1 = beta2 = 0, no bias left to correct, eps = 0: the moments are the gradient and its
    square, sqrt(a*a) = |a| exactly whenever a*a neither overflows nor goes denormal, a/|a| = +-1,
    so the step is exactly +-eta_l; a zero gradient gives 0/0 = NaN, which Adam's eps is there for."""
    rng = np.random.default_rng(90)
    grad = rng.standard_normal((2, 300)).astype(np.float32)
    grad[grad == 0] = 1.0
    p = rng.standard_normal((2, 300)).astype(np.float32)
    q = np.abs(rng.standard_normal((2, 300))).astype(np.float32)
    g = orc.local_adam(p, q, grad, 0.0, 0.0, 0.0, 0.125, 1.0, 1.0)
    assert np.array_equal(p, grad) and np.array_equal(q, grad * grad)
    assert np.array_equal(g, np.where(grad > 0, np.float32(0.125), np.float32(-0.125)))
    # eps is added to the root, not under it: a = 3, eps = 1 -> 3 / (3 + 1)
    one = np.full((1, 4), 3.0, dtype=np.float32)
    g = orc.local_adam(np.zeros_like(one), np.zeros_like(one), one, 0.0, 0.0, 1.0, 1.0, 1.0, 1.0)
    assert np.all(g == np.float32(0.75))


def test_local_adam_constant_gradient_closed_form():
    """Constant gradient a from zero moments: p_t = (1 - beta1^t) a and q_t = (1 - beta2^t) a^2, so the
    corrected moments are a and a^2 at every round and the step is eta_l * a / (|a| + eps) -- the
    property the bias correction exists for.  Columns >= d are neither read nor written."""
    b1, b2, eps, eta = 0.9, 0.999, 1e-8, 0.01
    a = np.array([[0.5, -2.0, 1e-3, -7.0, 777.0], [3.0, -0.25, 40.0, 1e-2, 777.0]], dtype=np.float32)
    p = np.zeros_like(a)
    q = np.zeros_like(a)
    for t in range(1, 40):
        g = orc.local_adam(p, q, a, b1, b2, eps, eta, 1.0 - b1 ** t, 1.0 - b2 ** t, d=4)
        want_p = (1.0 - b1 ** t) * a[:, :4].astype(np.float64)
        want_q = (1.0 - b2 ** t) * a[:, :4].astype(np.float64) ** 2
        assert np.allclose(p[:, :4], want_p, rtol=2e-5, atol=0) and np.allclose(q[:, :4], want_q, rtol=2e-5, atol=0)
        want = eta * a[:, :4] / (np.abs(a[:, :4]) + eps)
        assert np.allclose(g[:, :4], want, rtol=5e-5, atol=0), t
        assert np.all(p[:, 4] == 0.0) and np.all(q[:, 4] == 0.0) and np.all(g[:, 4] == 12345.0)


def test_local_adam_matches_torch_adam():
    """torch.optim.Adam (CPU, fp32, no weight decay, no amsgrad) moves the parameter by -g every step
    when lr = eta_l.  torch orders the arithmetic differently (lerp for the first moment, the bias
    correction folded into the step size), so agreement is to accumulated fp32 rounding."""
    import torch
    rng = np.random.default_rng(91)
    b1, b2, eps, eta = 0.9, 0.98, 1e-6, 0.02
    x0 = rng.standard_normal(400).astype(np.float32)
    par = torch.nn.Parameter(torch.from_numpy(x0.copy()))
    opt = torch.optim.Adam([par], lr=eta, betas=(b1, b2), eps=eps)
    p = np.zeros((1, 400), dtype=np.float32)
    q = np.zeros((1, 400), dtype=np.float32)
    x = x0.astype(np.float64)
    for t in range(1, 9):
        grad = (rng.standard_normal((1, 400)) * 10.0 ** rng.uniform(-3, 1)).astype(np.float32)
        par.grad = torch.from_numpy(grad[0].copy())
        opt.step()
        g = orc.local_adam(p, q, grad, b1, b2, eps, eta, 1.0 - b1 ** t, 1.0 - b2 ** t)
        x = x - g[0].astype(np.float64)
        assert np.allclose(par.detach().numpy(), x, rtol=0, atol=3e-6 * t), t
        state = opt.state[par]
        assert np.allclose(state["exp_avg"].numpy(), p[0], rtol=1e-5, atol=1e-6 * np.abs(p).max())
        assert np.allclose(state["exp_avg_sq"].numpy(), q[0], rtol=1e-5, atol=1e-6 * q.max())


def test_local_adam_single_roundings():
    """Each operation is rounded once in fp32, in the stated order: an element-by-element replay
    with numpy float32 scalars (which round after every operation) gives the same bits."""
    rng = np.random.default_rng(92)
    f = np.float32
    b1, b2, eps, eta, bias1, bias2 = f(0.9), f(0.999), f(1e-8), f(0.003), f(1 - 0.9 ** 3), f(1 - 0.999 ** 3)
    grad = rng.standard_normal((1, 64)).astype(np.float32)
    p = rng.standard_normal((1, 64)).astype(np.float32)
    q = np.abs(rng.standard_normal((1, 64))).astype(np.float32)
    p0, q0 = p.copy(), q.copy()
    g = orc.local_adam(p, q, grad, b1, b2, eps, eta, bias1, bias2)
    for i in range(64):
        a = grad[0, i]
        pp = b1 * p0[0, i] + (f(1) - b1) * a
        qq = b2 * q0[0, i] + (f(1) - b2) * (a * a)
        step = eta * ((pp / bias1) / (np.sqrt(qq / bias2) + eps))
        assert pp == p[0, i] and qq == q[0, i] and step == g[0, i], i


# ---------------------------------------------------------------------------------------------
# Matching-rate diagnostics (Section 3.2.2, Fig. 2b)
# ---------------------------------------------------------------------------------------------

def test_aggregate_sign_and_majority_vote_match_numpy():
    rng = np.random.default_rng(20)
    M, d = 7, 64 * 30 + 11
    g = rng.standard_normal((M, d)).astype(np.float32)
    c = (0.2 * rng.standard_normal((M, d))).astype(np.float32)
    s = g + c
    agg = ~np.signbit(s.astype(np.float64).sum(axis=0))
    maj = (2 * (~np.signbit(s)).sum(axis=0) >= M)

    def unpack(bits):
        e = np.arange(d)
        return ((bits[e // 64] >> (e % 64).astype(np.uint64)) & np.uint64(1)).astype(bool)
    assert np.array_equal(unpack(orc.aggregate_sign(g, c)), agg)
    assert np.array_equal(unpack(orc.majority_vote(g, c)), maj)
    a, b = orc.aggregate_sign(g, c), orc.majority_vote(g, c)
    assert orc.count_matching(a, b, d) == int((agg == maj).sum())
    assert orc.count_matching(a, a, d) == d
    assert int(a[-1]) >> (d % 64) == 0


@pytest.mark.parametrize("M", [2, 3, 8, 16])
def test_marsit_matching_rate_closed_form(M):
    """For i.i.d. zero-mean Gaussian workers the merged bit is the sign of a uniformly drawn worker,
    and P(sign(s_m) == sign(sum_k s_k)) = 1/2 + arcsin(1/sqrt(M)) / pi  (bivariate normal, correlation
    1/sqrt(M)).  The oracle's pass must reproduce that rate within a binomial bound."""
    rng = np.random.default_rng(30 + M)
    d = 1 << 19
    g = rng.standard_normal((M, d)).astype(np.float32)
    c = np.zeros_like(g)
    ref = orc.aggregate_sign(g, c)
    _, bits, _ = orc.sync_step(g, c.copy(), 1.0, 77 + M, threads=8)
    rate = orc.count_matching(bits, ref, d) / d
    want = 0.5 + np.arcsin(1.0 / np.sqrt(M)) / np.pi
    assert abs(rate - want) <= 5 * np.sqrt(want * (1 - want) / d)
    # the majority vote matches the aggregate more often (for M = 2 every disagreement is a tie)
    if M >= 3:
        assert orc.count_matching(orc.majority_vote(g, c), ref, d) / d > rate


# ---------------------------------------------------------------------------------------------
# Weighted merge and the reduction-tree schedule
# ---------------------------------------------------------------------------------------------

def test_weighted_threshold_generalises_eq2():
    for m in range(1, 17):
        assert orc.weighted_threshold(m - 1, 1) == (1 << 32) // m          # Eq. 2 itself
    assert orc.weighted_threshold(4, 4) == 1 << 31
    assert orc.weighted_threshold(2, 1) == (1 << 32) // 3
    assert orc.weighted_threshold(1, 2) == (2 << 32) // 3
    # same stream, same decision rule as the unweighted merge
    recv, local = 0x0123456789ABCDEF, 0xFEDCBA9876543210
    for m in (2, 3, 7):
        assert orc.merge_word_weighted(recv, local, m - 1, 1, 5, 99, 1234) == orc.merge_word(recv, local, m, 5, 99, 1234)


# ---------------------------------------------------------------------------------------------
# Torus whose last row is short (M not a multiple of the number of columns)
# ---------------------------------------------------------------------------------------------

def _ragged_rows(M, X):
    Y = -(-M // X)
    return [X] * (Y - 1) + [M - (Y - 1) * X]


@pytest.mark.parametrize("M,X", [(3, 2), (5, 2), (5, 3), (7, 3), (5, 4), (7, 2), (4, 3)])
def test_exact_unbiasedness_ragged_torus(M, X):
    """Rows with fold counts 2..X_y, then columns over the row results, each weighted by the number
    of workers it stands for: P(final = 1) = (+ workers) / M exactly, whatever the start row."""
    rows = _ragged_rows(M, X)
    Y = len(rows)
    n_draws = sum(r - 1 for r in rows) + (Y - 1)
    for b in range(Y):                                       # the column chain may start at any row
        for bits in itertools.product((0, 1), repeat=M):
            total = Fraction(0)
            for draws in itertools.product((0, 1), repeat=n_draws):
                it = iter(draws)
                weight = Fraction(1)
                results = []
                for y, Xy in enumerate(rows):
                    r = bits[y * X]
                    for h in range(1, Xy):
                        t = next(it)
                        weight *= Fraction(1, h + 1) if t else Fraction(h, h + 1)
                        l = bits[y * X + h]
                        r = orc.odot(r, l, orc.transient_from_keep(l, t)) & 1
                    results.append(r)
                r, gathered = results[b], rows[b]
                for k in range(1, Y):
                    y = (b + k) % Y
                    t = next(it)
                    p = Fraction(orc.weighted_threshold(gathered, rows[y]), 1 << 32)
                    assert abs(p - Fraction(rows[y], gathered + rows[y])) < Fraction(1, 1 << 32)
                    p = Fraction(rows[y], gathered + rows[y])
                    weight *= p if t else 1 - p
                    r = orc.odot(r, results[y], orc.transient_from_keep(results[y], t)) & 1
                    gathered += rows[y]
                total += weight * r
            assert total == Fraction(sum(bits), M)


@pytest.mark.parametrize("M,X,d", [(4, 2, 64 * 9 + 5), (6, 3, 64 * 7), (8, 8, 64 * 5 + 1), (16, 4, 64 * 6), (3, 1, 64 * 4 + 9)])
def test_ragged_torus_with_full_rows_is_the_torus(M, X, d):
    """With X dividing M every weight ratio is 1/(k+1): the same bits as the plain schedule."""
    rng = np.random.default_rng(300 + M)
    g = rng.standard_normal((M, d)).astype(np.float32)
    c = (0.3 * rng.standard_normal((M, d))).astype(np.float32)
    c1, c2 = c.copy(), c.copy()
    u1, b1 = orc.ragged_torus_step(g, c1, 1e-3, 77, X)
    u2, b2, _ = orc.sync_step(g, c2, 1e-3, 77, grid_x=X)
    assert np.array_equal(b1, b2) and np.array_equal(u1, u2) and np.array_equal(c1, c2)


def _ragged_reservoir_bits(signs, d, M, X, seed):
    """Second formulation, pure Python: per bit, the last successful draw of the column chain
    names a row, the last successful draw of that row's chain names a worker."""
    rows = _ragged_rows(M, X)
    Y = len(rows)
    W = (d + 63) // 64
    row_bounds = _floor_bounds(0, W, X)
    final = np.zeros(d, dtype=np.uint8)
    for e in range(d):
        w, j = divmod(e, 64)
        a = _part(w, row_bounds)
        col_bounds = _floor_bounds(row_bounds[a], row_bounds[a + 1] - row_bounds[a], Y)
        b = _part(w, col_bounds)
        pick, gathered = 0, rows[b]
        for k in range(1, Y):
            y = (b + k) % Y
            if philox_ref.stream_u32(seed, (1 << 16) | k, w, j) < (rows[y] << 32) // (gathered + rows[y]):
                pick = k
            gathered += rows[y]
        y = (b + pick) % Y
        start, col = a % rows[y], 0
        for h in range(1, rows[y]):
            if philox_ref.stream_u32(seed, (y << 8) | h, w, j) < (1 << 32) // (h + 1):
                col = h
        final[e] = signs[y * X + (start + col) % rows[y]][e]
    return final


@pytest.mark.parametrize("M,X,d", [(5, 2, 64 * 9 + 5), (7, 3, 64 * 8), (5, 4, 64 * 6 + 63), (11, 4, 64 * 7 + 1), (3, 2, 70)])
def test_ragged_torus_second_formulation(M, X, d):
    rng = np.random.default_rng(400 + M)
    g = rng.standard_normal((M, d)).astype(np.float32)
    c = (0.3 * rng.standard_normal((M, d))).astype(np.float32)
    seed = 0xFACE0000 + M
    signs = (~np.signbit(g + c)).astype(np.uint8)
    want = _ragged_reservoir_bits(signs, d, M, X, seed)
    c_after = c.copy()
    update, bits = orc.ragged_torus_step(g, c_after, 0.5, seed, X)
    got = ((bits[np.arange(d) // 64] >> (np.arange(d) % 64).astype(np.uint64)) & np.uint64(1)).astype(np.uint8)
    assert np.array_equal(got, want)
    assert np.array_equal(update, np.where(want == 1, np.float32(0.5), np.float32(-0.5)))
    assert np.array_equal(c_after, (g + c) - update)                 # compensation update, fp32


@pytest.mark.parametrize("M,X,patterns", [(5, 2, list(range(32))), (7, 3, [0, 1, 64, 3, 0x38, 0x55, 0x2A, 0x7F, 0x41, 0x0F]),
                                          (13, 4, [0x0001, 0x1000, 0x00FF, 0x1F00, 0x0F0F, 0x1555, 0x1FFF])])
def test_ragged_torus_empirical_unbiasedness(M, X, patterns):
    n_rep = 1 << 17
    g = _pattern_inputs(patterns, M, n_rep)
    c = np.zeros_like(g)
    update, bits = orc.ragged_torus_step(g, c, 1.0, 0xABCDEF + M, X, threads=8)
    plus = (update > 0).reshape(len(patterns), n_rep).mean(axis=1)
    for p, pat in enumerate(patterns):
        k = bin(pat).count("1")
        prob = k / M
        sigma = np.sqrt(max(prob * (1 - prob), 1e-12) / n_rep)
        assert abs(plus[p] - prob) <= 5 * sigma + 1e-9, (pat, plus[p], prob)


def _tree_merges(M):
    """(level, receiver, sender, w_local, w_recv) of the binary reduction tree, bottom level first."""
    out, stride, level = [], 1, 0
    while stride < M:
        for k in range(0, M - stride, 2 * stride):
            src = k + stride
            out.append((level, k, src, min(stride, M - k), min(stride, M - src)))
        stride *= 2
        level += 1
    return out


@pytest.mark.parametrize("M", [2, 3, 4, 5, 6, 7])
def test_exact_unbiasedness_tree(M):
    merges = _tree_merges(M)
    assert len(merges) == M - 1
    for bits in itertools.product((0, 1), repeat=M):
        total = Fraction(0)
        for draws in itertools.product((0, 1), repeat=len(merges)):
            val = list(bits)
            weight = Fraction(1)
            for (level, k, src, wl, wr), t in zip(merges, draws):
                p = Fraction(wl, wl + wr)
                weight *= p if t else 1 - p
                val[k] = orc.odot(val[src], val[k], orc.transient_from_keep(val[k], t)) & 1
            total += weight * val[0]
        assert total == Fraction(sum(bits), M)


def _tree_leaf(M, seed, w, j):
    """Second formulation: walk from the root towards the leaves; at every merge on the way the
    draw decides between the receiver's own subtree and the sender's."""
    top = 0
    while (1 << top) < M:
        top += 1
    k = 0
    for level in range(top - 1, -1, -1):
        stride = 1 << level
        src = k + stride
        if src >= M:
            continue
        wl, wr = min(stride, M - k), min(stride, M - src)
        u = philox_ref.stream_u32(seed, (2 << 16) | (level << 8) | k, w, j)
        if not u < (wl << 32) // (wl + wr):
            k = src
    return k


@pytest.mark.parametrize("M,d", [(2, 64 * 3 + 5), (3, 64 * 4), (5, 64 * 3 + 63), (8, 64 * 6 + 1), (11, 64 * 2 + 9)])
def test_tree_second_formulation(M, d):
    rng = np.random.default_rng(200 + M)
    g = rng.standard_normal((M, d)).astype(np.float32)
    c = (0.3 * rng.standard_normal((M, d))).astype(np.float32)
    seed = 0xFACE0000 + M
    s = g + c
    want = np.array([0 if np.signbit(s[_tree_leaf(M, seed, e // 64, e % 64), e]) else 1 for e in range(d)],
                    dtype=np.uint8)
    c_before = c.copy()
    update, bits = orc.tree_step(g, c, 0.25, seed)
    got = ((bits[np.arange(d) // 64] >> (np.arange(d) % 64).astype(np.uint64)) & np.uint64(1)).astype(np.uint8)
    assert np.array_equal(got, want)
    assert np.array_equal(update, np.where(want == 1, np.float32(0.25), np.float32(-0.25)))
    assert np.array_equal(c.view(np.uint32), ((g + c_before) - update[None, :]).view(np.uint32))


@pytest.mark.parametrize("M,patterns", [(3, list(range(8))), (6, [0, 1, 32, 7, 56, 21, 63, 44]), (8, [0x01, 0x80, 0x0F, 0xAA, 0x7F, 0xFF])])
def test_tree_empirical_unbiasedness(M, patterns):
    n_rep = 1 << 17
    g = _pattern_inputs(patterns, M, n_rep)
    update, _ = orc.tree_step(g, np.zeros_like(g), 1.0, 0xABCD + M)
    plus = (update > 0).reshape(len(patterns), n_rep)
    for p, pat in enumerate(patterns):
        mean = bin(pat).count("1") / M
        assert abs(plus[p].mean() - mean) <= 5.0 * np.sqrt(max(mean * (1 - mean), 1e-12) / n_rep)


# ---------------------------------------------------------------------------------------------
# The strawman of Section 3.2: SSDM's stochastic sign and cascading compression
# ---------------------------------------------------------------------------------------------

def test_l2_norm_matches_numpy():
    rng = np.random.default_rng(40)
    t = rng.standard_normal(10_001).astype(np.float32)
    want = np.sqrt(np.float32(np.sum(t.astype(np.float64) ** 2)))
    assert orc.l2_norm(t) == float(np.float32(want))
    assert orc.l2_norm(np.zeros(5, dtype=np.float32)) == 0.0


def test_ssdm_sign_probability_is_the_appendix_formula():
    """Count, over the whole stream definition, how often +1 comes out: for one element the decision
    is u < p * 2^32 with p = 1/2 + v/(2||v||) evaluated in fp32, so P(+1) = ceil(p * 2^32) / 2^32."""
    v = np.array([3.0, -4.0, 0.0, 12.0], dtype=np.float32)          # ||v|| = 13
    norm = orc.l2_norm(v)
    assert norm == 13.0
    # empirical frequency over many packed words (same 4 values replicated in the first bits)
    n_words = 1 << 15
    t = np.zeros(n_words * 64, dtype=np.float32)
    t.reshape(n_words, 64)[:, :4] = v
    bits = orc.ssdm_sign(t, norm, 0, orc.cascade_hop_id(0), 4242)
    for j, vj in enumerate(v):
        freq = float(((bits >> np.uint64(j)) & np.uint64(1)).mean())
        p = 0.5 + float(vj) / 26.0
        assert abs(freq - p) <= 5 * np.sqrt(p * (1 - p) / n_words), (j, freq, p)
    # zero entries are fair coins, and so is everything when the norm is zero
    freq0 = float(((bits >> np.uint64(10)) & np.uint64(1)).mean())
    assert abs(freq0 - 0.5) <= 5 * 0.5 / np.sqrt(n_words)
    z = orc.ssdm_sign(np.zeros(64 * 4096, dtype=np.float32), 0.0, 0, 1, 7)
    ones = sum(bin(int(x)).count("1") for x in z)
    assert abs(ones / (64 * 4096) - 0.5) <= 5 * 0.5 / np.sqrt(64 * 4096)


def test_ssdm_decision_rule_against_python():
    rng = np.random.default_rng(41)
    t = rng.standard_normal(64 * 3 + 7).astype(np.float32)
    norm = np.float32(orc.l2_norm(t))
    seed, hop, begin = 99, orc.cascade_hop_id(3), 1000
    bits = orc.ssdm_sign(t, float(norm), begin, hop, seed)
    for e in range(t.size):
        p = np.float32(0.5) + t[e] / (np.float32(2.0) * norm)
        u = philox_ref.stream_u32(seed, hop, begin + e // 64, e % 64)
        want = 1 if float(u) < float(p) * 4294967296.0 else 0
        assert (int(bits[e // 64]) >> (e % 64)) & 1 == want


def test_ssdm_is_unbiased():
    """Appendix A: E[ ||v|| * sign~(v) ] = v."""
    rng = np.random.default_rng(42)
    v = rng.standard_normal(64).astype(np.float32)
    norm = orc.l2_norm(v)
    n = 20_000
    acc = np.zeros(64)
    for s in range(n):
        b = int(orc.ssdm_sign(v, norm, 0, 1, 1000 + s)[0])
        acc += np.array([1.0 if (b >> j) & 1 else -1.0 for j in range(64)])
    est = norm * acc / n
    assert np.all(np.abs(est - v) <= 5 * norm / np.sqrt(n))


def test_cascading_compression_is_unbiased_for_the_sum():
    """Section 3.2: the expected result of cascading compression equals the sum of all gradients
    (update * M estimates sum_m s^(m)); checked on a tiny vector over many seeds."""
    rng = np.random.default_rng(43)
    M, d = 3, 64
    g = rng.standard_normal((M, d)).astype(np.float32)
    c = np.zeros_like(g)
    n = 6000
    acc = np.zeros(d)
    worst = 0.0
    for s in range(n):
        upd, bits, norms = orc.cascade_ring_step(g, c, 5000 + s)
        acc += upd.astype(np.float64) * M
        worst = max(worst, float(norms.max()))
    total = g.astype(np.float64).sum(axis=0)
    assert np.all(np.abs(acc / n - total) <= 5 * worst / np.sqrt(n))


@pytest.mark.parametrize("M,d", [(2, 8), (3, 8), (4, 5)])
def test_cascading_deviation_grows_like_the_appendix_says(M, d):
    """Appendix A compares the cascaded result s_3 with the plain mean s_1.  Because Q is unbiased
    with E||Q(v) - v||^2 = (D - 1) ||v||^2, the expected squared error of the chain obeys
    e_k = D e_(k-1) + (D - 1) ||S_k||^2 (S_k: sum of the first k workers of the chain), and
    E||s_3 - s_1||^2 = e_M / M^2 -- the geometric growth in M behind the (2D)^M bound."""
    rng = np.random.default_rng(60 + M)
    g = rng.standard_normal((M, d)).astype(np.float32)
    c = np.zeros_like(g)
    order = [(M - 1 + h) % M for h in range(M)]          # the only word falls in the last part
    e, run = 0.0, np.zeros(d)
    for m in order:
        run = run + g[m].astype(np.float64)
        e = d * e + (d - 1) * float(run @ run)
    expected = e / M ** 2
    mean = g.astype(np.float64).sum(axis=0) / M
    n = 8000
    dev = np.empty(n)
    for i in range(n):
        upd, _, _ = orc.cascade_ring_step(g, c, 9000 + i)
        diff = upd.astype(np.float64) - mean
        dev[i] = diff @ diff
    assert abs(dev.mean() - expected) <= 5 * dev.std() / np.sqrt(n)
    assert dev.mean() <= (2 * d) ** M * max(float(r @ r) for r in g.astype(np.float64)) / M     # the printed bound


def test_cascading_matching_rate_is_near_a_coin_flip_and_below_marsit():
    """Fig. 2(b)'s ordering on synthetic data: with a large part the l2 norm swamps every element,
    the stochastic sign is nearly a fair coin, and cascading compression matches the sign of the
    true aggregate far less often than Marsit's merged signs (and those less often than a majority
    vote)."""
    rng = np.random.default_rng(44)
    M, d = 3, 1 << 17
    g = rng.standard_normal((M, d)).astype(np.float32)
    c = np.zeros_like(g)
    ref = orc.aggregate_sign(g, c)
    _, cas_bits, _ = orc.cascade_ring_step(g, c, 11)
    _, mar_bits, _ = orc.sync_step(g, c.copy(), 1.0, 11, threads=4)
    r_cas = orc.count_matching(cas_bits, ref, d) / d
    r_mar = orc.count_matching(mar_bits, ref, d) / d
    r_maj = orc.count_matching(orc.majority_vote(g, c), ref, d) / d
    assert 0.5 - 0.01 < r_cas < 0.52
    assert r_cas + 0.1 < r_mar < r_maj


@pytest.mark.parametrize("M", [1, 2, 3, 5, 8])
def test_cascading_on_a_single_element_is_the_exact_mean(M):
    """With one element the l2 norm is |t|, the stochastic sign is certain (p is 0 or 1), and every
    hop recovers the running sum exactly: the result is the plain mean, whatever the seed."""
    rng = np.random.default_rng(50 + M)
    for trial in range(20):
        s = rng.standard_normal((M, 1)).astype(np.float32)
        upd, bits, norms = orc.cascade_ring_step(s, np.zeros_like(s), 1000 + trial)
        # the last part's chain starts at worker M-1 and goes round the ring
        order = [(M - 1 + h) % M for h in range(M)]
        run = np.float32(s[order[0], 0])
        for m in order[1:]:
            run = np.float32(run + s[m, 0])
        assert upd[0] == np.float32(run / np.float32(M))
        assert int(bits[0]) == (0 if np.signbit(run) else 1)
        assert norms[M - 1] == np.float32(abs(run))      # the only packed word falls in the last part


def test_majority_vote_ties_count_as_plus():
    g = np.array([[1.0, -1.0, 2.0, -2.0], [-1.0, 1.0, 2.0, -2.0]], dtype=np.float32)
    assert int(orc.majority_vote(g, np.zeros_like(g))[0]) == 0b0111
    g4 = np.array([[1.0], [1.0], [-1.0], [-1.0]], dtype=np.float32)
    assert int(orc.majority_vote(g4, np.zeros_like(g4))[0]) == 1
    g4[0, 0] = -1.0
    assert int(orc.majority_vote(g4, np.zeros_like(g4))[0]) == 0

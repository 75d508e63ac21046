"""ctypes front end of the CPU oracle (``marsit_oracle.c``).

TEST INFRASTRUCTURE ONLY: the tests, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this module; the product package never does.  The arithmetic lives in the
C file; this module only marshals numpy arrays.

The shared object is built with plain gcc (``build_oracle()``), with ``-ffp-contract=off`` and no
fast-math so that every fp32 operation of Algorithm 1 is a single IEEE-754 rounding.
"""

from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "marsit_oracle.c")
_SO = os.path.join(_HERE, "libmarsit_oracle.so")

MAX_WORKERS = 64

_lib = None


def build_oracle(force: bool = False) -> str:
    """Compile the C oracle into ``oracle/libmarsit_oracle.so`` and return its path."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-std=c11", "-O2", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
               "-fno-fast-math", "-Wall", "-Wextra", "-o", _SO, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _SO


def _load():
    global _lib
    if _lib is not None:
        return _lib
    lib = ctypes.CDLL(build_oracle())
    u32, u64, f32 = ctypes.c_uint32, ctypes.c_uint64, ctypes.c_float
    vp = ctypes.c_void_p
    lib.oracle_philox4x32_10.argtypes = [vp, vp, vp]
    lib.oracle_philox4x32_10.restype = None
    lib.oracle_stream_u32.argtypes = [u64, u32, u64, u32]
    lib.oracle_stream_u32.restype = u32
    lib.oracle_add_compensation.argtypes = [vp, vp, vp, u64]
    lib.oracle_add_compensation.restype = None
    lib.oracle_sign_pack.argtypes = [vp, vp, u64]
    lib.oracle_sign_pack.restype = None
    lib.oracle_sign_unpack.argtypes = [vp, vp, u64]
    lib.oracle_sign_unpack.restype = None
    lib.oracle_transient_from_keep.argtypes = [u64, u64]
    lib.oracle_transient_from_keep.restype = u64
    lib.oracle_keep_mask.argtypes = [u32, u32, u64, u64]
    lib.oracle_keep_mask.restype = u64
    lib.oracle_odot.argtypes = [u64, u64, u64]
    lib.oracle_odot.restype = u64
    lib.oracle_merge_word.argtypes = [u64, u64, u32, u32, u64, u64]
    lib.oracle_merge_word.restype = u64
    lib.oracle_hop_merge.argtypes = [vp, vp, vp, u64, u64, u32, u32, u64]
    lib.oracle_hop_merge.restype = ctypes.c_int
    lib.oracle_decode.argtypes = [vp, f32, vp, u64]
    lib.oracle_decode.restype = None
    lib.oracle_compensate.argtypes = [vp, vp, vp, u64]
    lib.oracle_compensate.restype = None
    lib.oracle_split_bounds.argtypes = [u64, u64, u32, vp]
    lib.oracle_split_bounds.restype = None
    lib.oracle_hop_id.argtypes = [u32, u32, u32]
    lib.oracle_hop_id.restype = u32
    lib.oracle_sync_step.argtypes = [vp, vp, vp, vp, vp, u32, u64, u64, f32, u64, u32, ctypes.c_int]
    lib.oracle_sync_step.restype = ctypes.c_int
    lib.oracle_ragged_torus_step.argtypes = [vp, vp, vp, vp, u32, u64, u64, f32, u64, u32, ctypes.c_int]
    lib.oracle_ragged_torus_step.restype = ctypes.c_int
    lib.oracle_full_sync.argtypes = [vp, vp, vp, u32, u64, u64]
    lib.oracle_full_sync.restype = ctypes.c_int
    lib.oracle_apply_update.argtypes = [vp, vp, u64]
    lib.oracle_apply_update.restype = None
    lib.oracle_local_momentum.argtypes = [vp, vp, vp, u32, u64, u64, f32, f32]
    lib.oracle_local_momentum.restype = ctypes.c_int
    lib.oracle_local_adam.argtypes = [vp, vp, vp, vp, u32, u64, u64, f32, f32, f32, f32, f32, f32]
    lib.oracle_local_adam.restype = ctypes.c_int
    lib.oracle_aggregate_sign.argtypes = [vp, vp, vp, u32, u64, u64]
    lib.oracle_aggregate_sign.restype = None
    lib.oracle_majority_vote.argtypes = [vp, vp, vp, u32, u64, u64]
    lib.oracle_majority_vote.restype = None
    lib.oracle_count_matching.argtypes = [vp, vp, u64]
    lib.oracle_count_matching.restype = u64
    lib.oracle_weighted_threshold.argtypes = [u32, u32]
    lib.oracle_weighted_threshold.restype = u64
    lib.oracle_merge_word_weighted.argtypes = [u64, u64, u32, u32, u32, u64, u64]
    lib.oracle_merge_word_weighted.restype = u64
    lib.oracle_hop_merge_weighted.argtypes = [vp, vp, vp, u64, u64, u32, u32, u32, u64]
    lib.oracle_hop_merge_weighted.restype = ctypes.c_int
    lib.oracle_tree_hop_id.argtypes = [u32, u32]
    lib.oracle_tree_hop_id.restype = u32
    lib.oracle_l2_norm.argtypes = [vp, u64]
    lib.oracle_l2_norm.restype = f32
    lib.oracle_ssdm_sign.argtypes = [vp, f32, vp, u64, u64, u32, u64]
    lib.oracle_ssdm_sign.restype = None
    lib.oracle_cascade_hop_id.argtypes = [u32]
    lib.oracle_cascade_hop_id.restype = u32
    lib.oracle_cascade_ring_step.argtypes = [vp, vp, vp, vp, vp, u32, u64, u64, u64]
    lib.oracle_cascade_ring_step.restype = ctypes.c_int
    lib.oracle_tree_step.argtypes = [vp, vp, vp, vp, u32, u64, u64, f32, u64]
    lib.oracle_tree_step.restype = ctypes.c_int
    _lib = lib
    return lib


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _f32(a, name):
    a = np.asarray(a)
    if a.dtype != np.float32 or not a.flags.c_contiguous:
        raise TypeError(f"{name}: need a C-contiguous float32 array")
    return a


def _u64(a, name):
    a = np.asarray(a)
    if a.dtype != np.uint64 or not a.flags.c_contiguous:
        raise TypeError(f"{name}: need a C-contiguous uint64 array")
    return a


def n_words(d: int) -> int:
    return (int(d) + 63) // 64


# --- random stream ---------------------------------------------------------------------------

def philox4x32_10(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32).copy()
    k = np.asarray(key, dtype=np.uint32).copy()
    assert c.shape == (4,) and k.shape == (2,)
    out = np.zeros(4, dtype=np.uint32)
    _load().oracle_philox4x32_10(_ptr(c), _ptr(k), _ptr(out))
    return out


def stream_u32(seed: int, hop_id: int, word_index: int, j: int) -> int:
    return int(_load().oracle_stream_u32(seed, hop_id, word_index, j))


def hop_id(phase: int, row: int, hop: int) -> int:
    return int(_load().oracle_hop_id(phase, row, hop))


# --- Algorithm 1, piece by piece -------------------------------------------------------------

def add_compensation(g, c):
    g = _f32(g, "g")
    c = None if c is None else _f32(c, "c")
    s = np.empty_like(g)
    _load().oracle_add_compensation(_ptr(g), _ptr(c), _ptr(s), g.size)
    return s


def sign_pack(s):
    s = _f32(s, "s")
    bits = np.zeros(n_words(s.size), dtype=np.uint64)
    _load().oracle_sign_pack(_ptr(s), _ptr(bits), s.size)
    return bits


def sign_unpack(bits, d: int):
    bits = _u64(bits, "bits")
    assert bits.size >= n_words(d)
    out = np.empty(d, dtype=np.float32)
    _load().oracle_sign_unpack(_ptr(bits), _ptr(out), d)
    return out


def transient_from_keep(local: int, keep: int) -> int:
    return int(_load().oracle_transient_from_keep(local, keep))


def keep_mask(fold: int, hop: int, seed: int, word_index: int) -> int:
    return int(_load().oracle_keep_mask(fold, hop, seed, word_index))


def odot(recv: int, local: int, v: int) -> int:
    return int(_load().oracle_odot(recv, local, v))


def merge_word(recv: int, local: int, fold: int, hop: int, seed: int, word_index: int) -> int:
    return int(_load().oracle_merge_word(recv, local, fold, hop, seed, word_index))


def hop_merge(recv, local, word_begin: int, fold: int, hop: int, seed: int):
    recv = _u64(recv, "recv")
    local = _u64(local, "local")
    assert recv.shape == local.shape
    out = np.empty_like(recv)
    rc = _load().oracle_hop_merge(_ptr(recv), _ptr(local), _ptr(out), word_begin, recv.size,
                                  fold, hop, seed)
    if rc != 0:
        raise ValueError(f"oracle_hop_merge: bad argument (rc={rc})")
    return out


def decode(bits, scale: float, d: int):
    bits = _u64(bits, "bits")
    assert bits.size >= n_words(d)
    upd = np.empty(d, dtype=np.float32)
    _load().oracle_decode(_ptr(bits), scale, _ptr(upd), d)
    return upd


def compensate(s, update):
    s = _f32(s, "s")
    update = _f32(update, "update")
    assert s.shape == update.shape
    out = np.empty_like(s)
    _load().oracle_compensate(_ptr(s), _ptr(update), _ptr(out), s.size)
    return out


def split_bounds(begin: int, n: int, parts: int):
    b = np.zeros(parts + 1, dtype=np.uint64)
    _load().oracle_split_bounds(begin, n, parts, _ptr(b))
    return b


# --- whole passes ----------------------------------------------------------------------------

def sync_step(g, c, scale: float, seed: int, grid_x: int = 0, d: int | None = None,
              threads: int = 1, want_sign_maps: bool = False):
    """One one-bit pass.  ``g`` and ``c`` are ``[M, ld]`` float32; ``c`` is updated in place.

    Returns ``(update[d], bits_final[W], sign_maps[M, W] or None)``.
    """
    g = _f32(g, "g")
    c = _f32(c, "c")
    assert g.ndim == 2 and g.shape == c.shape
    M, ld = g.shape
    d = ld if d is None else int(d)
    W = n_words(d)
    update = np.empty(d, dtype=np.float32)
    bits = np.zeros(W, dtype=np.uint64)
    maps = np.zeros((M, W), dtype=np.uint64) if want_sign_maps else None
    rc = _load().oracle_sync_step(_ptr(g), _ptr(c), _ptr(update), _ptr(bits), _ptr(maps),
                                  M, d, ld, scale, seed, grid_x, threads)
    if rc != 0:
        raise ValueError(f"oracle_sync_step failed (rc={rc})")
    return update, bits, maps


def ragged_torus_step(g, c, scale: float, seed: int, grid_x: int, d: int | None = None, threads: int = 1):
    """One one-bit pass over a torus of ``grid_x`` columns whose last row may be short (any
    ``1 <= grid_x <= M``); ``c`` is updated in place.  Returns ``(update[d], bits_final[W])``."""
    g = _f32(g, "g")
    c = _f32(c, "c")
    assert g.ndim == 2 and g.shape == c.shape
    M, ld = g.shape
    d = ld if d is None else int(d)
    update = np.zeros(d, dtype=np.float32)
    bits = np.zeros(n_words(d), dtype=np.uint64)
    rc = _load().oracle_ragged_torus_step(_ptr(g), _ptr(c), _ptr(update), _ptr(bits), M, d, ld, scale,
                                          seed & 0xFFFFFFFFFFFFFFFF, grid_x, threads)
    if rc != 0:
        raise ValueError(f"oracle_ragged_torus_step failed (rc={rc})")
    return update, bits


def full_sync(g, c, d: int | None = None):
    """Full-precision round: returns the mean update, zeroes ``c`` in place."""
    g = _f32(g, "g")
    c = _f32(c, "c")
    assert g.ndim == 2 and g.shape == c.shape
    M, ld = g.shape
    d = ld if d is None else int(d)
    update = np.empty(d, dtype=np.float32)
    rc = _load().oracle_full_sync(_ptr(g), _ptr(c), _ptr(update), M, d, ld)
    if rc != 0:
        raise ValueError(f"oracle_full_sync failed (rc={rc})")
    return update


def apply_update(x, update):
    x = _f32(x, "x")
    update = _f32(update, "update")
    assert x.shape == update.shape
    _load().oracle_apply_update(_ptr(x), _ptr(update), x.size)
    return x


def local_momentum(buf, grad, beta, eta_l, d=None):
    """buf <- beta*buf + grad (in place); returns g = eta_l * buf.  buf, grad: float32 [M, ld]."""
    buf = _f32(buf, "buf")
    grad = _f32(grad, "grad")
    assert buf.ndim == 2 and buf.shape == grad.shape
    M, ld = buf.shape
    d = ld if d is None else int(d)
    g = np.full_like(grad, 12345.0)
    rc = _load().oracle_local_momentum(_ptr(buf), _ptr(grad), _ptr(g), M, d, ld,
                                       beta, eta_l)
    assert rc == 0
    return g


def local_adam(mom1, mom2, grad, beta1, beta2, eps, eta_l, bias1, bias2, d=None):
    """Adam moments updated in place (float32 [M, ld]); returns g = eta_l * corrected step.
    bias1 = 1 - beta1**t, bias2 = 1 - beta2**t for the round t >= 1 being taken."""
    mom1 = _f32(mom1, "mom1")
    mom2 = _f32(mom2, "mom2")
    grad = _f32(grad, "grad")
    assert mom1.ndim == 2 and mom1.shape == grad.shape == mom2.shape
    M, ld = mom1.shape
    d = ld if d is None else int(d)
    g = np.full_like(grad, 12345.0)
    rc = _load().oracle_local_adam(_ptr(mom1), _ptr(mom2), _ptr(grad), _ptr(g), M, d, ld, beta1, beta2, eps, eta_l,
                                   bias1, bias2)
    assert rc == 0
    return g


# --- diagnostics (Section 3.2.2, Fig. 2b) ------------------------------------------------------

def _vote(fn, g, c, d):
    g = _f32(g, "g")
    c = _f32(c, "c")
    assert g.ndim == 2 and g.shape == c.shape
    M, ld = g.shape
    d = ld if d is None else int(d)
    bits = np.zeros(n_words(d), dtype=np.uint64)
    fn(_ptr(g), _ptr(c), _ptr(bits), M, d, ld)
    return bits


def aggregate_sign(g, c, d: int | None = None):
    """Packed sign of the non-compressed aggregate sum_m (g[m] + c[m])."""
    return _vote(_load().oracle_aggregate_sign, g, c, d)


def majority_vote(g, c, d: int | None = None):
    """Packed majority vote over the workers' signs (ties count as +)."""
    return _vote(_load().oracle_majority_vote, g, c, d)


def count_matching(a, b, d: int) -> int:
    a = _u64(a, "a")
    b = _u64(b, "b")
    assert a.size >= n_words(d) and b.size >= n_words(d)
    return int(_load().oracle_count_matching(_ptr(a), _ptr(b), d))


# --- other schedules: weighted merge, reduction tree -------------------------------------------

def weighted_threshold(w_recv: int, w_local: int) -> int:
    return int(_load().oracle_weighted_threshold(w_recv, w_local))


def merge_word_weighted(recv: int, local: int, w_recv: int, w_local: int, hop: int, seed: int,
                        word_index: int) -> int:
    return int(_load().oracle_merge_word_weighted(recv, local, w_recv, w_local, hop, seed, word_index))


def hop_merge_weighted(recv, local, word_begin: int, w_recv: int, w_local: int, hop: int, seed: int):
    recv = _u64(recv, "recv")
    local = _u64(local, "local")
    assert recv.shape == local.shape
    out = np.empty_like(recv)
    rc = _load().oracle_hop_merge_weighted(_ptr(recv), _ptr(local), _ptr(out), word_begin, recv.size,
                                           w_recv, w_local, hop, seed)
    if rc != 0:
        raise ValueError(f"oracle_hop_merge_weighted: bad argument (rc={rc})")
    return out


def tree_hop_id(level: int, receiver: int) -> int:
    return int(_load().oracle_tree_hop_id(level, receiver))


def tree_step(g, c, scale: float, seed: int, d: int | None = None):
    """One one-bit pass over a binary reduction tree; ``c`` is updated in place.
    Returns ``(update[d], bits_final[W])``."""
    g = _f32(g, "g")
    c = _f32(c, "c")
    assert g.ndim == 2 and g.shape == c.shape
    M, ld = g.shape
    d = ld if d is None else int(d)
    update = np.empty(d, dtype=np.float32)
    bits = np.zeros(n_words(d), dtype=np.uint64)
    rc = _load().oracle_tree_step(_ptr(g), _ptr(c), _ptr(update), _ptr(bits), M, d, ld, scale, seed)
    if rc != 0:
        raise ValueError(f"oracle_tree_step failed (rc={rc})")
    return update, bits


# --- the strawman of Section 3.2: SSDM stochastic sign, cascading compression -----------------

def l2_norm(t) -> float:
    t = _f32(t, "t")
    return float(_load().oracle_l2_norm(_ptr(t), t.size))


def ssdm_sign(t, norm: float, word_begin: int, hop: int, seed: int):
    t = _f32(t, "t")
    bits = np.zeros(n_words(t.size), dtype=np.uint64)
    _load().oracle_ssdm_sign(_ptr(t), norm, _ptr(bits), t.size, word_begin, hop, seed)
    return bits


def cascade_hop_id(hop: int) -> int:
    return int(_load().oracle_cascade_hop_id(hop))


def cascade_ring_step(g, c, seed: int, d: int | None = None):
    """Cascading compression with SSDM over the ring.  Returns ``(update[d], bits[W], norms[M])``."""
    g = _f32(g, "g")
    c = _f32(c, "c")
    assert g.ndim == 2 and g.shape == c.shape
    M, ld = g.shape
    d = ld if d is None else int(d)
    update = np.zeros(d, dtype=np.float32)
    bits = np.zeros(n_words(d), dtype=np.uint64)
    norms = np.zeros(M, dtype=np.float32)
    rc = _load().oracle_cascade_ring_step(_ptr(g), _ptr(c), _ptr(update), _ptr(bits), _ptr(norms),
                                          M, d, ld, seed)
    if rc != 0:
        raise ValueError(f"oracle_cascade_ring_step failed (rc={rc})")
    return update, bits, norms

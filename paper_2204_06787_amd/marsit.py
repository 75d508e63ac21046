"""Python binding over the C ABI of ``libmarsit.so`` (see ``include/marsit.h``).

Argument marshalling only: every step of the path runs in the HIP kernels.  PyTorch supplies device
memory (``tensor.data_ptr()``) and the current stream, nothing else.  There is no fallback: if the
library is missing, loading raises.
"""

from __future__ import annotations

import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libmarsit.so")

MAX_WORKERS = 64
MAX_ELEMENTS = (1 << 34) - 1024
OK, EINVAL, EALIGN, EHIP, ESCRATCH = 0, -1, -2, -3, -4
STATIC_SCRATCH_WORDS = 4194304

# every symbol include/marsit.h declares
EXPORTS = (
    "marsit_version", "marsit_last_hip_error", "marsit_status_string", "marsit_philox4x32_10",
    "marsit_split_bounds", "marsit_compress", "marsit_hop_merge", "marsit_decode_compensate",
    "marsit_ring_step_sim", "marsit_chain_step_sim", "marsit_chain_workspace_words",
    "marsit_full_sync", "marsit_step", "marsit_step_apply", "marsit_apply_update", "marsit_local_momentum",
    "marsit_local_adam",
    "marsit_pipeline_create", "marsit_pipeline_destroy", "marsit_pipeline_workspace_words",
    "marsit_compress_hop_merge", "marsit_decode_compensate_apply", "marsit_fold_segments",
    "marsit_exchange_step_sim", "marsit_pipeline_step", "marsit_pipeline_ring_step", "marsit_pipeline_last_hip_error",
    "marsit_aggregate_sign", "marsit_majority_vote", "marsit_count_matching",
    "marsit_hop_merge_weighted", "marsit_tree_step_sim", "marsit_tree_step_apply",
    "marsit_ragged_torus_step_sim", "marsit_ragged_torus_step_apply",
    "marsit_ssdm_cascade_hop", "marsit_cascade_ring_step_sim",
    "marsit_hop_merge_device_seed", "marsit_set_device_seed",
    "marsit_exchange_step_sim_static", "marsit_grid_work_items", "marsit_round", "marsit_set_fused_waves_per_cu",
)

_lib = None


class MarsitError(RuntimeError):
    def __init__(self, fn: str, status: int):
        self.status = status
        lib = _lib
        text = lib.marsit_status_string(status).decode() if lib is not None else "?"
        extra = f", hipError_t={lib.marsit_last_hip_error()}" if (lib is not None and status == EHIP) else ""
        super().__init__(f"{fn} failed: {text} (status {status}{extra})")


def load_library(path: str | None = None):
    """Load the HIP library; raises if it has not been built (``python -m paper_2204_06787_amd.build``)."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or os.environ.get("MARSIT_LIBRARY") or LIB_PATH     # MARSIT_LIBRARY: another build of the library
    if not os.path.exists(path):
        raise RuntimeError(
            f"{path} is missing: build the HIP library first (python -m paper_2204_06787_amd.build). "
            "There is no CPU fallback.")
    lib = ctypes.CDLL(path)
    u32, u64, f32, vp, ci = ctypes.c_uint32, ctypes.c_uint64, ctypes.c_float, ctypes.c_void_p, ctypes.c_int
    lib.marsit_version.argtypes = []
    lib.marsit_version.restype = ci
    lib.marsit_last_hip_error.argtypes = []
    lib.marsit_last_hip_error.restype = ci
    lib.marsit_status_string.argtypes = [ci]
    lib.marsit_status_string.restype = ctypes.c_char_p
    lib.marsit_grid_work_items.argtypes = [u64]
    lib.marsit_grid_work_items.restype = u64
    lib.marsit_philox4x32_10.argtypes = [vp, vp, vp]
    lib.marsit_philox4x32_10.restype = None
    lib.marsit_split_bounds.argtypes = [u64, u32, u32, vp]
    lib.marsit_split_bounds.restype = ci
    lib.marsit_compress.argtypes = [vp, vp, vp, u64, vp]
    lib.marsit_compress.restype = ci
    lib.marsit_hop_merge.argtypes = [vp, vp, vp, u64, u64, u32, u32, u64, vp]
    lib.marsit_hop_merge.restype = ci
    lib.marsit_decode_compensate.argtypes = [vp, vp, vp, f32, vp, vp, u64, vp]
    lib.marsit_decode_compensate.restype = ci
    lib.marsit_ring_step_sim.argtypes = [vp, vp, vp, vp, u32, u64, u64, f32, u64, u32, vp]
    lib.marsit_ring_step_sim.restype = ci
    lib.marsit_chain_step_sim.argtypes = [vp, vp, vp, vp, vp, u32, u64, u64, f32, u64, u32, vp]
    lib.marsit_chain_step_sim.restype = ci
    lib.marsit_chain_workspace_words.argtypes = [u32, u64, u32]
    lib.marsit_chain_workspace_words.restype = u64
    lib.marsit_pipeline_create.argtypes = [ctypes.POINTER(vp), u32]
    lib.marsit_pipeline_create.restype = ci
    lib.marsit_pipeline_destroy.argtypes = [vp]
    lib.marsit_pipeline_destroy.restype = ci
    lib.marsit_pipeline_workspace_words.argtypes = [u32, u64, u32]
    lib.marsit_pipeline_workspace_words.restype = u64
    lib.marsit_pipeline_ring_step.argtypes = [vp, vp, vp, vp, vp, vp, u64, u64, f32, u64, vp]
    lib.marsit_pipeline_step.argtypes = [vp, vp, vp, vp, vp, vp, u64, u64, f32, u64, u32, vp]
    lib.marsit_pipeline_step.restype = ci
    lib.marsit_pipeline_ring_step.restype = ci
    lib.marsit_compress_hop_merge.argtypes = [vp, vp, vp, vp, u64, u64, u32, u32, u64, vp]
    lib.marsit_compress_hop_merge.restype = ci
    lib.marsit_hop_merge_device_seed.argtypes = [vp, vp, vp, u64, u64, u32, u32, vp, vp]
    lib.marsit_hop_merge_device_seed.restype = ci
    lib.marsit_set_device_seed.argtypes = [vp, u64, vp]
    lib.marsit_set_device_seed.restype = ci
    lib.marsit_pipeline_last_hip_error.argtypes = []
    lib.marsit_pipeline_last_hip_error.restype = ci
    lib.marsit_hop_merge_weighted.argtypes = [vp, vp, vp, u64, u64, u32, u32, u32, u64, vp]
    lib.marsit_hop_merge_weighted.restype = ci
    lib.marsit_tree_step_sim.argtypes = [vp, vp, vp, vp, u32, u64, u64, f32, u64, vp]
    lib.marsit_tree_step_sim.restype = ci
    lib.marsit_ssdm_cascade_hop.argtypes = [vp, vp, vp, vp, vp, vp, vp, u64, u64, u32, u64, vp]
    lib.marsit_ssdm_cascade_hop.restype = ci
    lib.marsit_cascade_ring_step_sim.argtypes = [vp, vp, vp, vp, vp, vp, u32, u64, u64, u64, vp]
    lib.marsit_cascade_ring_step_sim.restype = ci
    lib.marsit_aggregate_sign.argtypes = [vp, vp, vp, u32, u64, u64, vp]
    lib.marsit_aggregate_sign.restype = ci
    lib.marsit_majority_vote.argtypes = [vp, vp, vp, u32, u64, u64, vp]
    lib.marsit_majority_vote.restype = ci
    lib.marsit_count_matching.argtypes = [vp, vp, u64, vp, vp]
    lib.marsit_count_matching.restype = ci
    lib.marsit_full_sync.argtypes = [vp, vp, vp, u32, u64, u64, vp]
    lib.marsit_full_sync.restype = ci
    lib.marsit_step.argtypes = [u64, u64, vp, vp, vp, vp, u32, u64, u64, f32, u64, u32, vp]
    lib.marsit_step.restype = ci
    lib.marsit_decode_compensate_apply.argtypes = [vp, vp, vp, f32, vp, vp, vp, u64, vp]
    lib.marsit_decode_compensate_apply.restype = ci
    lib.marsit_fold_segments.argtypes = [vp, u64, u32, u32, vp, u64, u64, u32, u64, vp]
    lib.marsit_fold_segments.restype = ci
    lib.marsit_exchange_step_sim.argtypes = [vp, vp, vp, vp, vp, u32, u64, u64, f32, u64, u32, vp]
    lib.marsit_exchange_step_sim.restype = ci
    lib.marsit_exchange_step_sim_static.argtypes = [vp, vp, vp, vp, u32, u64, u64, f32, u64, u32, vp]
    lib.marsit_exchange_step_sim_static.restype = ci
    lib.marsit_tree_step_apply.argtypes = [vp, vp, vp, vp, vp, u32, u64, u64, f32, u64, vp]
    lib.marsit_tree_step_apply.restype = ci
    lib.marsit_ragged_torus_step_sim.argtypes = [vp, vp, vp, vp, u32, u64, u64, f32, u64, u32, vp]
    lib.marsit_ragged_torus_step_sim.restype = ci
    lib.marsit_ragged_torus_step_apply.argtypes = [vp, vp, vp, vp, vp, u32, u64, u64, f32, u64, u32, vp]
    lib.marsit_ragged_torus_step_apply.restype = ci
    lib.marsit_step_apply.argtypes = [u64, u64, vp, vp, vp, vp, vp, u32, u64, u64, f32, u64, u32, vp]
    lib.marsit_step_apply.restype = ci
    lib.marsit_set_fused_waves_per_cu.argtypes = [u32]
    lib.marsit_set_fused_waves_per_cu.restype = ci
    lib.marsit_round.argtypes = [u64, u64, ci, u32, vp, vp, vp, vp, vp, u32, u64, u64, f32, u64, vp]
    lib.marsit_round.restype = ci
    lib.marsit_apply_update.argtypes = [vp, vp, u64, vp]
    lib.marsit_apply_update.restype = ci
    lib.marsit_local_momentum.argtypes = [vp, vp, vp, u32, u64, u64, f32, f32, vp]
    lib.marsit_local_momentum.restype = ci
    lib.marsit_local_adam.argtypes = [vp, vp, vp, vp, u32, u64, u64, f32, f32, f32, f32, f32, f32, vp]
    lib.marsit_local_adam.restype = ci
    if path == (os.environ.get("MARSIT_LIBRARY") or LIB_PATH):
        _lib = lib
    return lib


def n_words(d: int) -> int:
    return (int(d) + 63) // 64


def _check(fn: str, status: int):
    if status != OK:
        raise MarsitError(fn, status)


def _stream(stream) -> int:
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, torch.cuda.Stream):
        return stream.cuda_stream
    return int(stream)


def _f32_ptr(t, name, allow_none=False, need=0):
    """Device pointer of a float32 tensor.  A vector (the [M, ld] operands go through ``_rows``
    first) must be contiguous and hold at least ``need`` elements: the kernels trust these sizes."""
    if t is None:
        if allow_none:
            return None
        raise TypeError(f"{name} is required")
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == torch.float32):
        raise TypeError(f"{name}: need a float32 tensor in device memory")
    if t.dim() <= 1:
        if t.dim() == 1 and t.numel() > 1 and t.stride(0) != 1:
            raise TypeError(f"{name}: need a contiguous vector")
        if t.numel() < need:
            raise ValueError(f"{name}: {t.numel()} elements, need at least {need}")
    return t.data_ptr()


def _bits_ptr(t, name, allow_none=False, need=0):
    if t is None:
        if allow_none:
            return None
        raise TypeError(f"{name} is required")
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype in (torch.int64, torch.uint64)
            and t.is_contiguous()):
        raise TypeError(f"{name}: need a contiguous 64-bit integer tensor in device memory")
    if t.numel() < need:
        raise ValueError(f"{name}: {t.numel()} words, need at least {need}")
    return t.data_ptr()


def _rows(t, name, d=None):
    """[M, >=d] tensor with unit inner stride -> (M, row stride in elements)."""
    if not isinstance(t, torch.Tensor) or t.dim() != 2 or t.stride(1) != 1:
        raise TypeError(f"{name}: need a 2-D tensor whose rows are contiguous")
    if d is not None and t.shape[1] < d:
        raise ValueError(f"{name}: rows of {t.shape[1]} elements, need at least {d}")
    return t.shape[0], (t.stride(0) if t.shape[0] > 1 else max(t.stride(0), t.shape[1]))


def _matrix_args(g, c, d, names=("g", "c")):
    """Checks the [M, ld] operand pair and returns (M, ld, d)."""
    M, ld = _rows(g, names[0])
    if _rows(c, names[1]) != (M, ld):
        raise TypeError(f"{names[0]} and {names[1]} must have the same shape and row stride")
    d = g.shape[1] if d is None else int(d)
    if d < 0 or g.shape[1] < d or c.shape[1] < d:
        raise ValueError(f"d = {d} exceeds the rows of {names[0]} / {names[1]}")
    return M, ld, d


def new_bitmap(d: int, device="cuda") -> torch.Tensor:
    """Device buffer for a packed sign bitmap of d elements (int64 storage, 64 signs per word)."""
    return torch.empty(n_words(d), dtype=torch.int64, device=device)


# --- host-side helpers -------------------------------------------------------------------------

def marsit_version() -> int:
    return load_library().marsit_version()


def marsit_philox4x32_10(ctr, key):
    c = (ctypes.c_uint32 * 4)(*[int(x) & 0xFFFFFFFF for x in ctr])
    k = (ctypes.c_uint32 * 2)(*[int(x) & 0xFFFFFFFF for x in key])
    out = (ctypes.c_uint32 * 4)()
    load_library().marsit_philox4x32_10(c, k, out)
    return [int(x) for x in out]


def marsit_split_bounds(n_words_: int, M: int, grid_x: int = 0):
    out = (ctypes.c_uint64 * (MAX_WORKERS + 1))()
    _check("marsit_split_bounds", load_library().marsit_split_bounds(n_words_, M, grid_x, out))
    return [int(out[i]) for i in range(M + 1)]


# --- device entry points -----------------------------------------------------------------------

def marsit_compress(g, c, bits_out, d: int | None = None, stream=None):
    d = g.numel() if d is None else int(d)
    _check("marsit_compress", load_library().marsit_compress(
        _f32_ptr(g, "g", need=d), _f32_ptr(c, "c", True, need=d), _bits_ptr(bits_out, "bits_out", need=n_words(d)),
        d, _stream(stream)))
    return bits_out


def marsit_hop_merge(recv, local, out, word_begin: int, n_words_: int, fold: int, hop_id: int,
                     seed: int, stream=None):
    _check("marsit_hop_merge", load_library().marsit_hop_merge(
        _bits_ptr(recv, "recv", need=n_words_), _bits_ptr(local, "local", need=n_words_),
        _bits_ptr(out, "out", need=n_words_), word_begin,
        n_words_, fold, hop_id, seed & 0xFFFFFFFFFFFFFFFF, _stream(stream)))
    return out


def marsit_compress_hop_merge(recv, g, c, out, word_begin: int, fold: int, hop_id: int, seed: int,
                              n: int | None = None, stream=None):
    """``g``/``c``: the worker's vectors from the first element of the part (1-D views)."""
    n = g.numel() if n is None else int(n)
    _check("marsit_compress_hop_merge", load_library().marsit_compress_hop_merge(
        _bits_ptr(recv, "recv", True, need=n_words(n)), _f32_ptr(g, "g", need=n), _f32_ptr(c, "c", True, need=n),
        _bits_ptr(out, "out", need=n_words(n)),
        word_begin, n, fold, hop_id, seed & 0xFFFFFFFFFFFFFFFF, _stream(stream)))
    return out


def marsit_hop_merge_device_seed(recv, local, out, word_begin: int, n_words_: int, fold: int, hop_id: int,
                                 seed_device, stream=None):
    """``seed_device``: one-element int64 tensor in device memory holding the seed."""
    _check("marsit_hop_merge_device_seed", load_library().marsit_hop_merge_device_seed(
        _bits_ptr(recv, "recv", need=n_words_), _bits_ptr(local, "local", need=n_words_),
        _bits_ptr(out, "out", need=n_words_), word_begin,
        n_words_, fold, hop_id, _bits_ptr(seed_device, "seed_device", need=1), _stream(stream)))
    return out


def marsit_set_device_seed(seed_device, seed: int, stream=None):
    _check("marsit_set_device_seed", load_library().marsit_set_device_seed(
        _bits_ptr(seed_device, "seed_device", need=1), seed & 0xFFFFFFFFFFFFFFFF, _stream(stream)))
    return seed_device


def marsit_decode_compensate(bits, g, c, scale: float, update_out, c_out, d: int | None = None,
                             stream=None):
    d = g.numel() if d is None else int(d)
    _check("marsit_decode_compensate", load_library().marsit_decode_compensate(
        _bits_ptr(bits, "bits", need=n_words(d)), _f32_ptr(g, "g", need=d), _f32_ptr(c, "c", True, need=d), scale,
        _f32_ptr(update_out, "update_out", True, need=d), _f32_ptr(c_out, "c_out", need=d), d, _stream(stream)))
    return update_out, c_out


def marsit_decode_compensate_apply(bits, g, c, scale: float, x, update_out, c_out, d: int | None = None,
                                   stream=None):
    """``marsit_decode_compensate`` with the model update ``x -= update`` in the same pass."""
    d = g.numel() if d is None else int(d)
    _check("marsit_decode_compensate_apply", load_library().marsit_decode_compensate_apply(
        _bits_ptr(bits, "bits", need=n_words(d)), _f32_ptr(g, "g", need=d), _f32_ptr(c, "c", True, need=d), scale,
        _f32_ptr(x, "x", need=d), _f32_ptr(update_out, "update_out", True, need=d),
        _f32_ptr(c_out, "c_out", need=d), d, _stream(stream)))
    return x, c_out


def marsit_ring_step_sim(g, c, update_out, bits_out, scale: float, seed: int, grid_x: int = 0,
                         d: int | None = None, stream=None):
    """``g``, ``c``: ``[M, ld]`` float32 (rows contiguous); ``c`` is updated in place."""
    M, ld, d = _matrix_args(g, c, d)
    _check("marsit_ring_step_sim", load_library().marsit_ring_step_sim(
        _f32_ptr(g, "g"), _f32_ptr(c, "c"), _f32_ptr(update_out, "update_out", need=d),
        _bits_ptr(bits_out, "bits_out", True, need=n_words(d)), M, d, ld, scale, seed & 0xFFFFFFFFFFFFFFFF, grid_x,
        _stream(stream)))
    return update_out, bits_out


def marsit_set_fused_waves_per_cu(waves: int):
    """Tuning hook: wavefronts per CU of the compiled fused kernels (0: built-in choice)."""
    _check("marsit_set_fused_waves_per_cu", load_library().marsit_set_fused_waves_per_cu(waves))


def marsit_chain_workspace_words(M: int, d: int, grid_x: int = 0) -> int:
    return int(load_library().marsit_chain_workspace_words(M, d, grid_x))


def marsit_chain_step_sim(g, c, update_out, bits_out, workspace, scale: float, seed: int,
                          grid_x: int = 0, d: int | None = None, stream=None):
    """The pass hop by hop (un-fused).  ``workspace``: int64 tensor of ``marsit_chain_workspace_words``."""
    M, ld, d = _matrix_args(g, c, d)
    if workspace.numel() < marsit_chain_workspace_words(M, d, grid_x):
        raise ValueError("workspace too small")
    _check("marsit_chain_step_sim", load_library().marsit_chain_step_sim(
        _f32_ptr(g, "g"), _f32_ptr(c, "c"), _f32_ptr(update_out, "update_out", need=d),
        _bits_ptr(bits_out, "bits_out", need=n_words(d)), _bits_ptr(workspace, "workspace"), M, d, ld, scale,
        seed & 0xFFFFFFFFFFFFFFFF, grid_x, _stream(stream)))
    return update_out, bits_out


def marsit_fold_segments(maps, K: int, first: int, out, word_begin: int, n_words_: int, hop_base: int,
                         seed: int, stride_words: int | None = None, stream=None):
    """``maps``: ``[K, stride_words]`` 64-bit tensor (or a flat one with ``stride_words`` given)
    whose row k holds operand k's segment in its first ``n_words_`` words."""
    if stride_words is None:
        if maps.dim() != 2 or maps.stride(1) != 1:
            raise TypeError("maps: need [K, words] with contiguous rows, or pass stride_words")
        stride_words = maps.stride(0)
    if not (isinstance(maps, torch.Tensor) and maps.is_cuda and maps.dtype in (torch.int64, torch.uint64)):
        raise TypeError("maps: need a 64-bit integer tensor in device memory")
    if K < 1 or (maps.dim() == 2 and maps.shape[0] < K) or n_words_ < 0:
        raise ValueError("maps holds fewer than K operands")
    reach = (K - 1) * stride_words + n_words_          # words from maps' first element to the last one read
    have = (maps.shape[0] - 1) * maps.stride(0) + maps.shape[1] if maps.dim() == 2 else maps.numel()
    if reach > have:
        raise ValueError(f"maps: the K operands reach {reach} words, the tensor holds {have}")
    _check("marsit_fold_segments", load_library().marsit_fold_segments(
        maps.data_ptr(), stride_words, K, first, _bits_ptr(out, "out", need=n_words_), word_begin, n_words_, hop_base,
        seed & 0xFFFFFFFFFFFFFFFF, _stream(stream)))
    return out


def marsit_exchange_step_sim(g, c, update_out, bits_out, workspace, scale: float, seed: int,
                             grid_x: int = 0, d: int | None = None, stream=None):
    """The pass as one exchange step: signs, one fold per part, decode.  Workspace as for the chain."""
    M, ld, d = _matrix_args(g, c, d)
    if workspace.numel() < marsit_chain_workspace_words(M, d, grid_x):
        raise ValueError("workspace too small")
    _check("marsit_exchange_step_sim", load_library().marsit_exchange_step_sim(
        _f32_ptr(g, "g"), _f32_ptr(c, "c"), _f32_ptr(update_out, "update_out", need=d),
        _bits_ptr(bits_out, "bits_out", need=n_words(d)), _bits_ptr(workspace, "workspace"), M, d, ld, scale,
        seed & 0xFFFFFFFFFFFFFFFF, grid_x, _stream(stream)))
    return update_out, bits_out


def marsit_exchange_step_sim_static(g, c, update_out, bits_out, scale: float, seed: int, grid_x: int = 0,
                                    d: int | None = None, stream=None):
    """``marsit_exchange_step_sim`` on the library's own static workspace: the call allocates nothing."""
    M, ld, d = _matrix_args(g, c, d)
    _check("marsit_exchange_step_sim_static", load_library().marsit_exchange_step_sim_static(
        _f32_ptr(g, "g"), _f32_ptr(c, "c"), _f32_ptr(update_out, "update_out", need=d),
        _bits_ptr(bits_out, "bits_out", need=n_words(d)), M, d, ld, scale,
        seed & 0xFFFFFFFFFFFFFFFF, grid_x, _stream(stream)))
    return update_out, bits_out


class RingPipeline:
    """Handle of ``marsit_pipeline_*``: M workers, one HIP stream each, on a ring or a torus."""

    def __init__(self, M: int):
        self._h = ctypes.c_void_p()
        self.M = int(M)
        _check("marsit_pipeline_create", load_library().marsit_pipeline_create(ctypes.byref(self._h), M))

    def workspace_words(self, d: int, grid_x: int = 0) -> int:
        return int(load_library().marsit_pipeline_workspace_words(self.M, d, grid_x))

    def step(self, g, c, update_out, bits_out, workspace, scale: float, seed: int, grid_x: int = 0,
             d: int | None = None, stream=None):
        M, ld, d = _matrix_args(g, c, d)
        if M != self.M:
            raise TypeError("g and c must be [M, ld] with the pipeline's M")
        need = self.workspace_words(d, grid_x)
        if need == 0 and d > 0:
            raise ValueError("grid_x must be 0 or divide M")
        if workspace.numel() < need:
            raise ValueError("workspace too small")
        _check("marsit_pipeline_step", load_library().marsit_pipeline_step(
            self._h, _f32_ptr(g, "g"), _f32_ptr(c, "c"), _f32_ptr(update_out, "update_out", need=d),
            _bits_ptr(bits_out, "bits_out", need=n_words(d)), _bits_ptr(workspace, "workspace"), d, ld, scale,
            seed & 0xFFFFFFFFFFFFFFFF, grid_x, _stream(stream)))
        return update_out, bits_out

    def ring_step(self, g, c, update_out, bits_out, workspace, scale: float, seed: int,
                  d: int | None = None, stream=None):
        M, ld, d = _matrix_args(g, c, d)
        if M != self.M:
            raise TypeError("g and c must be [M, ld] with the pipeline's M")
        if workspace.numel() < self.workspace_words(d):
            raise ValueError("workspace too small")
        _check("marsit_pipeline_ring_step", load_library().marsit_pipeline_ring_step(
            self._h, _f32_ptr(g, "g"), _f32_ptr(c, "c"), _f32_ptr(update_out, "update_out", need=d),
            _bits_ptr(bits_out, "bits_out", need=n_words(d)), _bits_ptr(workspace, "workspace"), d, ld, scale,
            seed & 0xFFFFFFFFFFFFFFFF, _stream(stream)))
        return update_out, bits_out

    def close(self):
        if self._h:
            _check("marsit_pipeline_destroy", load_library().marsit_pipeline_destroy(self._h))
            self._h = ctypes.c_void_p()

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()


def marsit_full_sync(g, c, update_out, d: int | None = None, stream=None):
    M, ld, d = _matrix_args(g, c, d)
    _check("marsit_full_sync", load_library().marsit_full_sync(
        _f32_ptr(g, "g"), _f32_ptr(c, "c"), _f32_ptr(update_out, "update_out", need=d), M, d, ld,
        _stream(stream)))
    return update_out


def marsit_step(t: int, K: int, g, c, update_out, bits_out, scale: float, seed: int,
                grid_x: int = 0, d: int | None = None, stream=None):
    M, ld, d = _matrix_args(g, c, d)
    _check("marsit_step", load_library().marsit_step(
        t, K, _f32_ptr(g, "g"), _f32_ptr(c, "c"), _f32_ptr(update_out, "update_out", need=d),
        _bits_ptr(bits_out, "bits_out", True, need=n_words(d)), M, d, ld, scale, seed & 0xFFFFFFFFFFFFFFFF, grid_x,
        _stream(stream)))
    return update_out, bits_out


def marsit_step_apply(t: int, K: int, g, c, x, update_out, bits_out, scale: float, seed: int,
                      grid_x: int = 0, d: int | None = None, stream=None):
    """``marsit_step`` with the model update ``x -= g_t`` in the same pass; ``update_out`` may be None."""
    M, ld, d = _matrix_args(g, c, d)
    _check("marsit_step_apply", load_library().marsit_step_apply(
        t, K, _f32_ptr(g, "g"), _f32_ptr(c, "c"), _f32_ptr(x, "x", need=d),
        _f32_ptr(update_out, "update_out", True, need=d),
        _bits_ptr(bits_out, "bits_out", True, need=n_words(d)), M, d, ld, scale, seed & 0xFFFFFFFFFFFFFFFF, grid_x,
        _stream(stream)))
    return x


SCHEDULE_RING, SCHEDULE_TORUS, SCHEDULE_TREE = 0, 1, 2


def marsit_round(t: int, K: int, schedule: int, grid_x: int, g, c, x, update_out, bits_out, scale: float,
                 seed: int, d: int | None = None, stream=None):
    """One round of Algorithm 1 (and of Algorithm 2 when ``x`` is given) over the named schedule."""
    M, ld, d = _matrix_args(g, c, d)
    _check("marsit_round", load_library().marsit_round(
        t, K, schedule, grid_x, _f32_ptr(g, "g"), _f32_ptr(c, "c"), _f32_ptr(x, "x", True, need=d),
        _f32_ptr(update_out, "update_out", True, need=d),
        _bits_ptr(bits_out, "bits_out", True, need=n_words(d)), M, d, ld, scale, seed & 0xFFFFFFFFFFFFFFFF,
        _stream(stream)))
    return update_out


def marsit_apply_update(x, update, d: int | None = None, stream=None):
    d = x.numel() if d is None else int(d)
    _check("marsit_apply_update", load_library().marsit_apply_update(
        _f32_ptr(x, "x", need=d), _f32_ptr(update, "update", need=d), d, _stream(stream)))
    return x


def marsit_local_momentum(buf, grad, g_out, beta: float, eta_l: float, d: int | None = None, stream=None):
    M, ld, d = _matrix_args(buf, grad, d, names=("buf", "grad"))
    if _rows(g_out, "g_out", d) != (M, ld):
        raise TypeError("buf, grad and g_out must have the same shape and row stride")
    _check("marsit_local_momentum", load_library().marsit_local_momentum(
        _f32_ptr(buf, "buf"), _f32_ptr(grad, "grad"), _f32_ptr(g_out, "g_out"), M, d, ld, beta, eta_l,
        _stream(stream)))
    return g_out


def marsit_local_adam(mom1, mom2, grad, g_out, beta1: float, beta2: float, eps: float, eta_l: float,
                      bias1: float, bias2: float, d: int | None = None, stream=None):
    """Local Adam of the M workers; ``bias1 = 1 - beta1**t``, ``bias2 = 1 - beta2**t`` for round t >= 1."""
    M, ld, d = _matrix_args(mom1, grad, d, names=("mom1", "grad"))
    if _rows(mom2, "mom2", d) != (M, ld) or _rows(g_out, "g_out", d) != (M, ld):
        raise TypeError("mom1, mom2, grad and g_out must have the same shape and row stride")
    _check("marsit_local_adam", load_library().marsit_local_adam(
        _f32_ptr(mom1, "mom1"), _f32_ptr(mom2, "mom2"), _f32_ptr(grad, "grad"), _f32_ptr(g_out, "g_out"), M, d, ld,
        beta1, beta2, eps, eta_l, bias1, bias2, _stream(stream)))
    return g_out


# --- diagnostics (Section 3.2.2, Fig. 2b) --------------------------------------------------------

def _vote(name, g, c, bits_out, d, stream):
    M, ld, d = _matrix_args(g, c, d)
    _check(name, getattr(load_library(), name)(
        _f32_ptr(g, "g"), _f32_ptr(c, "c"), _bits_ptr(bits_out, "bits_out", need=n_words(d)), M, d, ld,
        _stream(stream)))
    return bits_out


def marsit_aggregate_sign(g, c, bits_out, d: int | None = None, stream=None):
    return _vote("marsit_aggregate_sign", g, c, bits_out, d, stream)


def marsit_majority_vote(g, c, bits_out, d: int | None = None, stream=None):
    return _vote("marsit_majority_vote", g, c, bits_out, d, stream)


def marsit_count_matching(bits_a, bits_b, d: int, count_out, stream=None):
    """``count_out``: one-element int64 tensor in device memory (overwritten)."""
    _check("marsit_count_matching", load_library().marsit_count_matching(
        _bits_ptr(bits_a, "bits_a", need=n_words(d)), _bits_ptr(bits_b, "bits_b", need=n_words(d)), d,
        _bits_ptr(count_out, "count_out", need=1),
        _stream(stream)))
    return count_out


# --- other schedules -----------------------------------------------------------------------------

def marsit_hop_merge_weighted(recv, local, out, word_begin: int, n_words_: int, w_recv: int,
                              w_local: int, hop_id: int, seed: int, stream=None):
    _check("marsit_hop_merge_weighted", load_library().marsit_hop_merge_weighted(
        _bits_ptr(recv, "recv", need=n_words_), _bits_ptr(local, "local", need=n_words_),
        _bits_ptr(out, "out", need=n_words_), word_begin,
        n_words_, w_recv, w_local, hop_id, seed & 0xFFFFFFFFFFFFFFFF, _stream(stream)))
    return out


def marsit_tree_step_sim(g, c, update_out, bits_out, scale: float, seed: int, d: int | None = None,
                         stream=None):
    """The one-bit pass over a binary reduction tree; ``c`` is updated in place."""
    M, ld, d = _matrix_args(g, c, d)
    _check("marsit_tree_step_sim", load_library().marsit_tree_step_sim(
        _f32_ptr(g, "g"), _f32_ptr(c, "c"), _f32_ptr(update_out, "update_out", need=d),
        _bits_ptr(bits_out, "bits_out", True, need=n_words(d)), M, d, ld, scale, seed & 0xFFFFFFFFFFFFFFFF,
        _stream(stream)))
    return update_out, bits_out


def marsit_tree_step_apply(g, c, x, update_out, bits_out, scale: float, seed: int, d: int | None = None,
                           stream=None):
    """``marsit_tree_step_sim`` with the model update ``x -= g_t`` in the same pass."""
    M, ld, d = _matrix_args(g, c, d)
    _check("marsit_tree_step_apply", load_library().marsit_tree_step_apply(
        _f32_ptr(g, "g"), _f32_ptr(c, "c"), _f32_ptr(x, "x", need=d),
        _f32_ptr(update_out, "update_out", True, need=d),
        _bits_ptr(bits_out, "bits_out", True, need=n_words(d)), M, d, ld, scale, seed & 0xFFFFFFFFFFFFFFFF,
        _stream(stream)))
    return x


def marsit_ragged_torus_step_sim(g, c, update_out, bits_out, scale: float, seed: int, grid_x: int,
                                 d: int | None = None, stream=None):
    """The one-bit pass over a torus of ``grid_x`` columns whose last row may be short."""
    M, ld, d = _matrix_args(g, c, d)
    _check("marsit_ragged_torus_step_sim", load_library().marsit_ragged_torus_step_sim(
        _f32_ptr(g, "g"), _f32_ptr(c, "c"), _f32_ptr(update_out, "update_out", need=d),
        _bits_ptr(bits_out, "bits_out", True, need=n_words(d)), M, d, ld, scale, seed & 0xFFFFFFFFFFFFFFFF,
        grid_x, _stream(stream)))
    return update_out, bits_out


def marsit_ragged_torus_step_apply(g, c, x, update_out, bits_out, scale: float, seed: int, grid_x: int,
                                   d: int | None = None, stream=None):
    M, ld, d = _matrix_args(g, c, d)
    _check("marsit_ragged_torus_step_apply", load_library().marsit_ragged_torus_step_apply(
        _f32_ptr(g, "g"), _f32_ptr(c, "c"), _f32_ptr(x, "x", need=d),
        _f32_ptr(update_out, "update_out", True, need=d),
        _bits_ptr(bits_out, "bits_out", True, need=n_words(d)), M, d, ld, scale, seed & 0xFFFFFFFFFFFFFFFF,
        grid_x, _stream(stream)))
    return x


# --- the strawman of Section 3.2 (comparison point) ------------------------------------------------

CASCADE_WORKSPACE_BYTES = 8256


def new_cascade_workspace(device="cuda") -> torch.Tensor:
    return torch.empty(CASCADE_WORKSPACE_BYTES // 8, dtype=torch.int64, device=device)


def marsit_ssdm_cascade_hop(recv_bits, recv_norm, g, c, bits_out, norm_out, workspace, word_begin: int,
                            n: int, hop_id: int, seed: int, stream=None):
    """``recv_norm``/``norm_out``: one-element float32 tensors in device memory."""
    _check("marsit_ssdm_cascade_hop", load_library().marsit_ssdm_cascade_hop(
        _bits_ptr(recv_bits, "recv_bits", True, need=n_words(n)), _f32_ptr(recv_norm, "recv_norm", True, need=1),
        _f32_ptr(g, "g", need=n), _f32_ptr(c, "c", need=n), _bits_ptr(bits_out, "bits_out", need=n_words(n)),
        _f32_ptr(norm_out, "norm_out", need=1),
        _bits_ptr(workspace, "workspace", need=CASCADE_WORKSPACE_BYTES // 8), word_begin, n, hop_id, seed & 0xFFFFFFFFFFFFFFFF,
        _stream(stream)))
    return bits_out, norm_out


def marsit_cascade_ring_step_sim(g, c, update_out, bits_out, norms_out, workspace, seed: int,
                                 d: int | None = None, stream=None):
    M, ld, d = _matrix_args(g, c, d)
    _check("marsit_cascade_ring_step_sim", load_library().marsit_cascade_ring_step_sim(
        _f32_ptr(g, "g"), _f32_ptr(c, "c"), _f32_ptr(update_out, "update_out", need=d),
        _bits_ptr(bits_out, "bits_out", need=n_words(d)), _f32_ptr(norms_out, "norms_out", need=M),
        _bits_ptr(workspace, "workspace", need=CASCADE_WORKSPACE_BYTES // 8), M, d, ld, seed & 0xFFFFFFFFFFFFFFFF, _stream(stream)))
    return update_out, bits_out, norms_out

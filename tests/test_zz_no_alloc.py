"""The entry point that allocates nothing: marsit_exchange_step_sim_static against
marsit_exchange_step_sim (the same kernels on a caller's workspace), through the C ABI.

Two calls in a row on the same GPU, the second with a smaller input, so that whatever the first
call left in the library's static workspace would show if a word of it were read before being
written.  Bar: merged bitmap and update bit-exact, compensation bit for bit (same kernels, same
operands).  The collection order puts this file last on purpose.
"""

import numpy as np
import pytest
import torch

from paper_2204_06787_amd import marsit
from gpu_util import dev, host_bits, host_f32

pytestmark = pytest.mark.gpu


def _inputs(M, d, ld, seed):
    rng = np.random.default_rng(seed)
    g = rng.standard_normal((M, ld)).astype(np.float32)
    c = (0.3 * rng.standard_normal((M, ld))).astype(np.float32)
    return g, c


def _both(M, d, ld, grid_x, seed, steps=2):
    """Runs `steps` carried steps through both entry points; returns nothing, asserts equality."""
    g_h, c_h = _inputs(M, d, ld, seed)
    g = dev(g_h)
    c_ref, c_new = dev(c_h), dev(c_h)
    ws = torch.empty(max(1, marsit.marsit_chain_workspace_words(M, d, grid_x)), dtype=torch.int64, device="cuda")
    for t in range(steps):
        upd_ref = torch.full((d,), 5.0, dtype=torch.float32, device="cuda")
        upd_new = torch.full((d,), 6.0, dtype=torch.float32, device="cuda")
        bits_ref, bits_new = marsit.new_bitmap(d), marsit.new_bitmap(d)
        bits_ref.fill_(-1)
        bits_new.fill_(0x55)
        marsit.marsit_exchange_step_sim(g, c_ref, upd_ref, bits_ref, ws, 1e-3, seed + t, grid_x=grid_x, d=d)
        marsit.marsit_exchange_step_sim_static(g, c_new, upd_new, bits_new, 1e-3, seed + t, grid_x=grid_x, d=d)
        torch.cuda.synchronize()
        what = f"M={M} d={d} ld={ld} grid_x={grid_x} step {t}"
        assert np.array_equal(host_bits(bits_new), host_bits(bits_ref)), f"bitmap, {what}"
        assert np.array_equal(host_f32(upd_new).view(np.uint32), host_f32(upd_ref).view(np.uint32)), f"update, {what}"
        assert np.array_equal(host_f32(c_new).view(np.uint32), host_f32(c_ref).view(np.uint32)), f"compensation, {what}"


def test_static_workspace_matches_caller_workspace_twice_in_a_row():
    print("no-alloc entry point: ring M=8 d=1000003, then ring M=3 d=70001, then torus 2x2 d=4099", flush=True)
    _both(8, 1_000_003, 1_000_003, 0, seed=11)        # 125 008 workspace words
    _both(3, 70_001, 70_004, 0, seed=12)              # smaller: 3 282 words, the rest keeps the first call's bits
    _both(4, 4_099, 4_100, 2, seed=13)                # torus: per-worker bitmaps and row results
    _both(5, 63, 64, 0, seed=14)                      # one ragged word per worker


def test_static_workspace_size_limit_and_argument_errors():
    M = 8
    d_fit = (marsit.STATIC_SCRATCH_WORDS // M) * 64               # exactly fills the array
    assert marsit.marsit_chain_workspace_words(M, d_fit, 0) == marsit.STATIC_SCRATCH_WORDS
    lib = marsit.load_library()
    one = torch.zeros(64, dtype=torch.float32, device="cuda")
    bits = marsit.new_bitmap(64)
    p, b = one.data_ptr(), bits.data_ptr()
    # too large: rejected before any launch (the pointers are never dereferenced)
    assert lib.marsit_exchange_step_sim_static(p, p, p, b, M, d_fit + 1, d_fit + 1, 1e-3, 1, 0, None) == marsit.ESCRATCH
    assert lib.marsit_exchange_step_sim_static(p, p, p, b, 16, 25_600_000, 25_600_000, 1e-3, 1, 4, None) == marsit.ESCRATCH
    # the argument errors of marsit_exchange_step_sim
    assert lib.marsit_exchange_step_sim_static(None, p, p, b, 1, 64, 64, 1e-3, 1, 0, None) == marsit.EINVAL
    assert lib.marsit_exchange_step_sim_static(p, p, p, None, 1, 64, 64, 1e-3, 1, 0, None) == marsit.EINVAL
    assert lib.marsit_exchange_step_sim_static(p, p, p, b, 0, 64, 64, 1e-3, 1, 0, None) == marsit.EINVAL
    assert lib.marsit_exchange_step_sim_static(p, p, p, b, 6, 64, 64, 1e-3, 1, 4, None) == marsit.EINVAL
    assert lib.marsit_exchange_step_sim_static(p, p, p, b, 1, 64, 32, 1e-3, 1, 0, None) == marsit.EINVAL
    assert lib.marsit_exchange_step_sim_static(p, p, p, b, 1, 64, 64, float("inf"), 1, 0, None) == marsit.EINVAL
    assert lib.marsit_exchange_step_sim_static(p, p, p, b, 1, 0, 0, 1e-3, 1, 0, None) == marsit.OK       # d == 0
    assert b"static scratch" in lib.marsit_status_string(marsit.ESCRATCH)


def test_static_workspace_at_the_headline_size():
    """M = 8, d = 25.6 M fits the static array (3.2 M of 4 Mi words)."""
    M, d = 8, 25_600_000
    assert marsit.marsit_chain_workspace_words(M, d, 0) <= marsit.STATIC_SCRATCH_WORDS
    gen = torch.Generator(device="cuda").manual_seed(99)
    g = torch.randn((M, d), generator=gen, dtype=torch.float32, device="cuda")
    c_ref = torch.zeros((M, d), dtype=torch.float32, device="cuda")
    c_new = torch.zeros((M, d), dtype=torch.float32, device="cuda")
    ws = torch.empty(marsit.marsit_chain_workspace_words(M, d, 0), dtype=torch.int64, device="cuda")
    upd_ref = torch.empty(d, dtype=torch.float32, device="cuda")
    upd_new = torch.empty(d, dtype=torch.float32, device="cuda")
    bits_ref, bits_new = marsit.new_bitmap(d), marsit.new_bitmap(d)
    for t in range(2):
        marsit.marsit_exchange_step_sim(g, c_ref, upd_ref, bits_ref, ws, 1e-3, 400 + t)
        marsit.marsit_exchange_step_sim_static(g, c_new, upd_new, bits_new, 1e-3, 400 + t)
        torch.cuda.synchronize()
        assert torch.equal(bits_new, bits_ref)
        assert torch.equal(upd_new.view(torch.int32), upd_ref.view(torch.int32))
        assert torch.equal(c_new.view(torch.int32), c_ref.view(torch.int32))

"""Algorithm 1 as a whole (one-bit rounds and the full-precision round every K) and the model update
of Algorithm 2, HIP path against the oracle."""

import numpy as np
import pytest
import torch

from oracle import marsit_oracle as orc
from paper_2204_06787_amd import marsit, workloads
from gpu_util import assert_f32_parity, dev, host_bits, host_f32, unaligned_rows

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("M,d,ld,aligned", [(1, 100, 100, True), (3, 4099, 4100, True), (8, 100_000, 100_000, True),
                                             (16, 33_333, 33_336, True), (8, 5001, 5003, False), (64, 777, 780, True)])
def test_full_sync(M, d, ld, aligned):
    rng = np.random.default_rng(M + d)
    g_h = rng.standard_normal((M, ld)).astype(np.float32)
    c_h = rng.standard_normal((M, ld)).astype(np.float32)
    if aligned:
        g_d, c_d = dev(g_h), dev(c_h)
    else:
        g_d, c_d = unaligned_rows(M, ld), unaligned_rows(M, ld)
        g_d.copy_(dev(g_h))
        c_d.copy_(dev(c_h))
    pad_before = c_h[:, d:].copy()
    want = orc.full_sync(g_h, c_h, d=d)
    u = torch.empty(d, dtype=torch.float32, device="cuda")
    marsit.marsit_full_sync(g_d, c_d, u, d=d)
    torch.cuda.synchronize()
    got = host_f32(u)
    # both sides add the fp32 terms in double in worker order, divide in double and round once
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    got_c = host_f32(c_d)
    assert not got_c[:, :d].any()                                # c <- 0
    assert np.array_equal(got_c[:, d:], pad_before)              # padding untouched
    assert np.array_equal(c_h[:, :d], got_c[:, :d])


def test_full_sync_single_worker_is_exact():
    rng = np.random.default_rng(3)
    g_h = rng.standard_normal((1, 1000)).astype(np.float32)
    c_h = rng.standard_normal((1, 1000)).astype(np.float32)
    want = orc.full_sync(g_h.copy(), c_h.copy())
    u = torch.empty(1000, dtype=torch.float32, device="cuda")
    marsit.marsit_full_sync(dev(g_h), dev(c_h), u)
    torch.cuda.synchronize()
    assert np.array_equal(host_f32(u), want)


@pytest.mark.parametrize("d", [1, 5, 4096, 100_003])
def test_apply_update(d):
    rng = np.random.default_rng(d)
    x_h = rng.standard_normal(d).astype(np.float32)
    u_h = (1e-3 * np.sign(rng.standard_normal(d))).astype(np.float32)
    x_d = dev(x_h)
    marsit.marsit_apply_update(x_d, dev(u_h))
    torch.cuda.synchronize()
    assert_f32_parity(host_f32(x_d), orc.apply_update(x_h.copy(), u_h), "x")


@pytest.mark.parametrize("M,d,ld,offset", [(1, 1, 1, 0), (3, 5, 7, 0), (8, 4096, 4096, 0), (4, 100_003, 100_003, 0),
                                           (5, 1000, 1004, 0), (2, 777, 780, 1), (64, 130, 132, 0)])
def test_local_momentum(M, d, ld, offset):
    """Three steps of the workers' heavy-ball buffers, in place over the gradient (g_out = grad)
    and into a separate output, from unaligned bases and padded rows too."""
    rng = np.random.default_rng(M * 1000 + d)
    buf_h = rng.standard_normal((M, ld)).astype(np.float32)
    if offset:
        buf_d = unaligned_rows(M, ld, offset)
        buf_d.copy_(dev(buf_h))
    else:
        buf_d = dev(buf_h)
    for t in range(3):
        grad_h = rng.standard_normal((M, ld)).astype(np.float32)
        want_g = orc.local_momentum(buf_h, grad_h, 0.9, 0.05, d=d)
        grad_d = dev(grad_h)
        if t % 2 == 0:
            out_d = torch.full((M, ld), 12345.0, dtype=torch.float32, device="cuda")
            marsit.marsit_local_momentum(buf_d, grad_d, out_d, 0.9, 0.05, d=d)
        else:
            out_d = marsit.marsit_local_momentum(buf_d, grad_d, grad_d, 0.9, 0.05, d=d)
            want_g[:, d:] = grad_h[:, d:]                      # in place: the padding keeps the gradient's values
        torch.cuda.synchronize()
        assert_f32_parity(host_f32(buf_d), buf_h, f"momentum buffer, step {t}")
        assert_f32_parity(host_f32(out_d), want_g, f"scaled gradient, step {t}")


@pytest.mark.parametrize("M,d,ld,offset", [(1, 1, 1, 0), (3, 5, 7, 0), (8, 4096, 4096, 0), (4, 100_003, 100_003, 0),
                                           (5, 1000, 1004, 0), (2, 777, 780, 1), (64, 130, 132, 0)])
def test_local_adam(M, d, ld, offset):
    """Four rounds of the workers' Adam moments (bias corrections of rounds 1..4), in place over the
    gradient and into a separate output, from unaligned bases and padded rows, gradients over
    fourteen orders of magnitude with exact zeros among them.  Quotients and the square root are
    correctly rounded on both sides, so the comparison is bit for bit."""
    rng = np.random.default_rng(M * 1000 + d + 5)
    b1, b2, eps, eta = 0.9, 0.999, 1e-8, 0.003
    p_h = (0.1 * rng.standard_normal((M, ld))).astype(np.float32)
    q_h = (0.01 * rng.standard_normal((M, ld)) ** 2).astype(np.float32)
    if offset:
        p_d, q_d = unaligned_rows(M, ld, offset), unaligned_rows(M, ld, offset)
        p_d.copy_(dev(p_h))
        q_d.copy_(dev(q_h))
    else:
        p_d, q_d = dev(p_h), dev(q_h)
    for t in range(1, 5):
        grad_h = (rng.standard_normal((M, ld)) * 10.0 ** rng.uniform(-10, 4, size=(M, ld))).astype(np.float32)
        grad_h[rng.random((M, ld)) < 0.05] = 0.0
        bias1, bias2 = 1.0 - b1 ** t, 1.0 - b2 ** t
        want_g = orc.local_adam(p_h, q_h, grad_h, b1, b2, eps, eta, bias1, bias2, d=d)
        grad_d = dev(grad_h)
        if t % 2 == 0:
            out_d = torch.full((M, ld), 12345.0, dtype=torch.float32, device="cuda")
            marsit.marsit_local_adam(p_d, q_d, grad_d, out_d, b1, b2, eps, eta, bias1, bias2, d=d)
        else:
            out_d = marsit.marsit_local_adam(p_d, q_d, grad_d, grad_d, b1, b2, eps, eta, bias1, bias2, d=d)
            want_g[:, d:] = grad_h[:, d:]                      # in place: the padding keeps the gradient's values
        torch.cuda.synchronize()
        assert_f32_parity(host_f32(p_d), p_h, f"first moment, round {t}")
        assert_f32_parity(host_f32(q_d), q_h, f"second moment, round {t}")
        assert_f32_parity(host_f32(out_d), want_g, f"scaled step, round {t}")


def test_local_adam_extreme_values():
    """Denormal and huge second moments, eps = 0 with a zero moment (0/0 = NaN on both sides), beta = 0."""
    f = np.float32
    grad_h = np.array([[0.0, 1e-30, -1e-25, 3e18, -1e19, 1e-45, 5.0, -0.0]], dtype=np.float32)
    for b1, b2, eps in ((0.9, 0.999, 1e-8), (0.0, 0.0, 0.0), (0.5, 0.25, 1.0)):
        p_h = np.zeros_like(grad_h)
        q_h = np.zeros_like(grad_h)
        p_d, q_d = dev(p_h), dev(q_h)
        for t in range(1, 4):
            bias1 = 1.0 - b1 ** t
            bias2 = 1.0 - b2 ** t
            want = orc.local_adam(p_h, q_h, grad_h, b1, b2, eps, 0.01, bias1, bias2)
            out_d = torch.empty_like(p_d)
            marsit.marsit_local_adam(p_d, q_d, dev(grad_h), out_d, b1, b2, eps, 0.01, bias1, bias2)
            torch.cuda.synchronize()
            got = host_f32(out_d)
            assert np.array_equal(np.isnan(got), np.isnan(want)), (b1, b2, eps, t)
            ok = ~np.isnan(want)
            assert np.array_equal(got[ok].view(np.uint32), want[ok].view(np.uint32)), (b1, b2, eps, t, got, want)
            assert np.array_equal(host_f32(p_d).view(np.uint32), p_h.view(np.uint32))
            assert np.array_equal(host_f32(q_d).view(np.uint32), q_h.view(np.uint32))


def test_sgd_driver_with_local_adam():
    """MarsitSGD with optimizer="adam" against the oracle's Adam + synchronisation + update."""
    from paper_2204_06787_amd.sgd import MarsitSGD
    M, d, K = 4, 50_001, 4
    rng = np.random.default_rng(98)
    x_h = rng.standard_normal(d).astype(np.float32)
    c_h = np.zeros((M, d), dtype=np.float32)
    p_h = np.zeros((M, d), dtype=np.float32)
    q_h = np.zeros((M, d), dtype=np.float32)
    opt = MarsitSGD(dev(x_h), M=M, K=K, eta_s=2e-3, seed=41, optimizer="adam", betas=(0.9, 0.98), eps=1e-6)
    for t in range(6):
        grad_h = rng.standard_normal((M, d)).astype(np.float32)
        opt.step_from_raw_gradients(dev(grad_h), eta_l=0.01)
        g_h = orc.local_adam(p_h, q_h, grad_h, 0.9, 0.98, 1e-6, 0.01, 1.0 - 0.9 ** (t + 1), 1.0 - 0.98 ** (t + 1))
        if t % K == 0:
            u_h = orc.full_sync(g_h, c_h)
        else:
            u_h, _, _ = orc.sync_step(g_h, c_h, 2e-3, 41 + t)
        x_h = orc.apply_update(x_h, u_h)
        torch.cuda.synchronize()
        assert_f32_parity(host_f32(opt.buf), p_h, f"first moments, round {t}")
        assert_f32_parity(host_f32(opt.buf2), q_h, f"second moments, round {t}")
        assert_f32_parity(host_f32(opt.c), c_h, f"compensation, round {t}")
        assert_f32_parity(host_f32(opt.update), u_h, f"update, round {t}")
        assert_f32_parity(host_f32(opt.x), x_h, f"model, round {t}")


def test_sgd_driver_with_local_momentum():
    """MarsitSGD.step_from_raw_gradients against the oracle's momentum + synchronisation + update."""
    from paper_2204_06787_amd.sgd import MarsitSGD
    M, d, K = 4, 70_001, 3
    rng = np.random.default_rng(99)
    x_h = rng.standard_normal(d).astype(np.float32)
    c_h = np.zeros((M, d), dtype=np.float32)
    buf_h = np.zeros((M, d), dtype=np.float32)
    opt = MarsitSGD(dev(x_h), M=M, K=K, eta_s=2e-3, seed=31, momentum=0.9)
    for t in range(5):
        grad_h = rng.standard_normal((M, d)).astype(np.float32)
        opt.step_from_raw_gradients(dev(grad_h), eta_l=0.01)
        g_h = orc.local_momentum(buf_h, grad_h, 0.9, 0.01)
        if t % K == 0:
            u_h = orc.full_sync(g_h, c_h)
        else:
            u_h, _, _ = orc.sync_step(g_h, c_h, 2e-3, 31 + t)
        x_h = orc.apply_update(x_h, u_h)
        torch.cuda.synchronize()
        assert_f32_parity(host_f32(opt.buf), buf_h, f"momentum buffers, round {t}")
        assert_f32_parity(host_f32(opt.c), c_h, f"compensation, round {t}")
        assert_f32_parity(host_f32(opt.update), u_h, f"update, round {t}")
        assert_f32_parity(host_f32(opt.x), x_h, f"model, round {t}")


@pytest.mark.parametrize("M,grid_x,d,ld,offset", [
    (8, 0, 70_001, 70_004, 0), (16, 4, 33_000, 33_000, 0), (3, 0, 64 * 5, 64 * 5, 0), (9, 0, 4099, 4100, 0),
    (6, 3, 1000, 1000, 0), (5, 0, 2000, 2001, 0), (8, 0, 777, 780, 1), (1, 0, 130, 132, 0), (48, 0, 300, 300, 0)])
@pytest.mark.parametrize("keep_update", [True, False])
def test_step_apply(M, grid_x, d, ld, offset, keep_update):
    """A round with the model update in the same pass: compiled and generic schedules, ragged
    tails, padded and misaligned rows, one-bit and full-precision rounds (K = 3, t = 0..4)."""
    K, scale, seed0 = 3, 2e-3, 77
    rng = np.random.default_rng(M * 100 + d)
    x_h = rng.standard_normal(d).astype(np.float32)
    c_h = np.zeros((M, ld), dtype=np.float32)
    if offset:
        c_d = unaligned_rows(M, ld, offset)
        x_d = torch.zeros(d + 8, dtype=torch.float32, device="cuda")[offset:offset + d]
        x_d.copy_(dev(x_h))
    else:
        c_d = torch.zeros((M, ld), dtype=torch.float32, device="cuda")
        x_d = dev(x_h)
    u_d = torch.full((d,), 7.0, dtype=torch.float32, device="cuda") if keep_update else None
    bits = marsit.new_bitmap(d)
    for t in range(5):
        g_h = (0.01 * rng.standard_normal((M, ld))).astype(np.float32)
        if offset:
            g_d = unaligned_rows(M, ld, offset)
            g_d.copy_(dev(g_h))
        else:
            g_d = dev(g_h)
        marsit.marsit_step_apply(t, K, g_d, c_d, x_d, u_d, bits, scale, seed0 + t, grid_x=grid_x, d=d)
        torch.cuda.synchronize()
        if t % K == 0:
            want_u = orc.full_sync(g_h, c_h, d=d)
        else:
            want_u, want_b, _ = orc.sync_step(g_h, c_h, scale, seed0 + t, grid_x=grid_x, d=d)
            assert np.array_equal(host_bits(bits), want_b), t
        if keep_update:
            assert_f32_parity(host_f32(u_d), want_u, f"update, round {t}")
        x_h = orc.apply_update(x_h, want_u)
        assert_f32_parity(host_f32(x_d), x_h, f"model, round {t}")
        assert_f32_parity(host_f32(c_d)[:, :d], c_h[:, :d], f"compensation, round {t}")
        assert np.array_equal(host_f32(c_d)[:, d:], c_h[:, d:])                     # padding untouched


@pytest.mark.parametrize("schedule,M,grid_x,d,ld", [
    ("ring", 8, 0, 70_001, 70_004), ("ring", 11, 0, 5_003, 5_003), ("torus", 16, 4, 33_000, 33_000),
    ("torus", 7, 3, 9_999, 10_000), ("torus", 13, 4, 4_099, 4_100), ("tree", 8, 0, 20_000, 20_000),
    ("tree", 11, 0, 3_001, 3_004), ("torus", 5, 5, 777, 780), ("torus", 6, 1, 640, 640)])
@pytest.mark.parametrize("with_model", [True, False])
def test_round_with_schedule_selector(schedule, M, grid_x, d, ld, with_model):
    """marsit_round: branch of Algorithm 1 and schedule chosen inside the library, against the
    oracle's routine for that schedule, K = 3, rounds 0..4, with and without the model update."""
    K, scale, seed0 = 3, 2e-3, 123
    sid = {"ring": marsit.SCHEDULE_RING, "torus": marsit.SCHEDULE_TORUS, "tree": marsit.SCHEDULE_TREE}[schedule]
    rng = np.random.default_rng(M * 1000 + d)
    x_h = rng.standard_normal(d).astype(np.float32)
    c_h = np.zeros((M, ld), dtype=np.float32)
    c_d = torch.zeros((M, ld), dtype=torch.float32, device="cuda")
    x_d = dev(x_h) if with_model else None
    u_d = torch.full((d,), 7.0, dtype=torch.float32, device="cuda")
    bits = marsit.new_bitmap(d)
    for t in range(5):
        g_h = (0.01 * rng.standard_normal((M, ld))).astype(np.float32)
        marsit.marsit_round(t, K, sid, grid_x, dev(g_h), c_d, x_d, u_d, bits, scale, seed0 + t, d=d)
        torch.cuda.synchronize()
        if t % K == 0:
            want_u = orc.full_sync(g_h, c_h, d=d)
        else:
            if schedule == "tree":
                want_u, want_b = orc.tree_step(g_h, c_h, scale, seed0 + t, d=d)
            elif schedule == "torus":
                want_u, want_b = orc.ragged_torus_step(g_h, c_h, scale, seed0 + t, grid_x, d=d)
            else:
                want_u, want_b, _ = orc.sync_step(g_h, c_h, scale, seed0 + t, d=d)
            assert np.array_equal(host_bits(bits), want_b), t
        assert_f32_parity(host_f32(u_d), want_u, f"update, round {t}")
        if with_model:
            x_h = orc.apply_update(x_h, want_u)
            assert_f32_parity(host_f32(x_d), x_h, f"model, round {t}")
        assert_f32_parity(host_f32(c_d)[:, :d], c_h[:, :d], f"compensation, round {t}")
        assert np.array_equal(host_f32(c_d)[:, d:], c_h[:, d:])


def test_round_argument_validation():
    lib = marsit.load_library()
    buf = torch.zeros(256, dtype=torch.float32, device="cuda")
    bits = marsit.new_bitmap(64)
    p, b = buf.data_ptr(), bits.data_ptr()

    def call(t=1, K=2, schedule=0, grid_x=0, x=p + 1024 // 2, u=p, M=2, d=64, ld=64, scale=1e-3):
        return lib.marsit_round(t, K, schedule, grid_x, p, p, x, u, b, M, d, ld, scale, 1, None)
    assert call(K=0) == marsit.EINVAL
    assert call(schedule=3) == marsit.EINVAL and call(schedule=-1) == marsit.EINVAL
    assert call(schedule=marsit.SCHEDULE_RING, grid_x=1) == marsit.EINVAL         # a ring has no grid
    assert call(schedule=marsit.SCHEDULE_TORUS, grid_x=0) == marsit.EINVAL
    assert call(schedule=marsit.SCHEDULE_TORUS, grid_x=3) == marsit.EINVAL        # more columns than workers
    assert call(schedule=marsit.SCHEDULE_TREE, grid_x=2) == marsit.EINVAL
    assert call(x=None, u=None) == marsit.EINVAL
    assert call(x=p, u=p) == marsit.EINVAL
    assert call(scale=float("nan")) == marsit.EINVAL
    assert call(M=0) == marsit.EINVAL and call(M=65) == marsit.EINVAL
    assert call(d=0, ld=0) == marsit.OK
    torch.cuda.synchronize()


def test_step_apply_equals_step_then_apply_update_bit_for_bit():
    """Against the two-call form on the device (both HIP): identical model, compensation, bitmap."""
    M, d, K = 8, 300_000 + 37, 4
    rng = np.random.default_rng(8)
    x0 = dev(rng.standard_normal(d).astype(np.float32))
    xa, xb = x0.clone(), x0.clone()
    ca = torch.zeros((M, d), dtype=torch.float32, device="cuda")
    cb = torch.zeros_like(ca)
    ua = torch.empty(d, dtype=torch.float32, device="cuda")
    ba, bb = marsit.new_bitmap(d).zero_(), marsit.new_bitmap(d).zero_()     # a full-precision round leaves them alone
    for t in range(6):
        g = dev((0.02 * rng.standard_normal((M, d))).astype(np.float32))
        marsit.marsit_step(t, K, g, ca, ua, ba, 1e-3, 900 + t)
        marsit.marsit_apply_update(xa, ua)
        marsit.marsit_step_apply(t, K, g, cb, xb, None, bb, 1e-3, 900 + t)
        torch.cuda.synchronize()
        assert torch.equal(xa, xb) and torch.equal(ca, cb) and torch.equal(ba, bb), t


@pytest.mark.parametrize("M,grid_x,K", [(8, 0, 4), (16, 4, 3), (3, 0, 1), (5, 0, 100)])
def test_marsit_driven_sgd_loop(M, grid_x, K):
    """Algorithm 2 with Algorithm 1 inside: T rounds, a full-precision round whenever t mod K == 0,
    x <- x - g_t after every round.  Every round must match the oracle bit for bit."""
    d, T, scale, seed0 = 20_000 + 7, 9, 1e-3, 31
    wl = workloads.Workload("loop", M=M, d=d, grid_x=grid_x, steps=T, scale=scale, dist="normal", std=0.01)
    x_d = torch.zeros(d, dtype=torch.float32, device="cuda")
    x_h = np.zeros(d, dtype=np.float32)
    c_d = workloads.zero_compensation(wl, device="cuda")
    c_h = np.zeros((M, d), dtype=np.float32)
    u_d = torch.empty(d, dtype=torch.float32, device="cuda")
    bits = marsit.new_bitmap(d)
    for t in range(T):
        g_d = workloads.make_gradients(wl, t, seed=seed0, device="cuda")
        g_h = host_f32(g_d).copy()
        sd = workloads.step_seed(seed0, t)
        marsit.marsit_step(t, K, g_d, c_d, u_d, bits, scale, sd, grid_x=grid_x)
        marsit.marsit_apply_update(x_d, u_d)
        torch.cuda.synchronize()
        if t % K != 0:
            want_u, want_b, _ = orc.sync_step(g_h, c_h, scale, sd, grid_x=grid_x)
            assert np.array_equal(host_bits(bits), want_b), t
            assert np.array_equal(host_f32(u_d), want_u), t
            assert_f32_parity(host_f32(c_d), c_h, f"c, round {t}")
        else:
            want_u = orc.full_sync(g_h, c_h)
            assert_f32_parity(host_f32(u_d), want_u, f"mean update, round {t}")
            assert not host_f32(c_d).any()
        x_h = orc.apply_update(x_h, want_u)
        assert_f32_parity(host_f32(x_d), x_h, f"model, round {t}")


def test_step_can_be_captured_in_a_hip_graph():
    """The library launches kernels only (no memset, no allocation, no synchronisation), so a step
    can be captured and replayed; every replay must reproduce the eager result, with eager work
    and synchronisations between the replays."""
    M, d, scale, seed = 8, 300_000 + 5, 1e-3, 2718
    rng = np.random.default_rng(5)
    g_h = rng.standard_normal((M, d)).astype(np.float32)
    g_d = dev(g_h)
    c_static = torch.zeros((M, d), dtype=torch.float32, device="cuda")
    u_static = torch.empty(d, dtype=torch.float32, device="cuda")
    b_static = marsit.new_bitmap(d)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # warm-up outside the capture
        marsit.marsit_step(3, 100, g_d, c_static, u_static, b_static, scale, seed)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    c_static.zero_()
    torch.cuda.synchronize()
    with torch.cuda.graph(graph):
        marsit.marsit_step(3, 100, g_d, c_static, u_static, b_static, scale, seed)
        marsit.marsit_step(4, 100, g_d, c_static, u_static, b_static, scale, seed + 1)

    c_h = np.zeros((M, d), dtype=np.float32)
    for replay in range(3):
        graph.replay()
        torch.cuda.synchronize()
        orc.sync_step(g_h, c_h, scale, seed)
        want_u, want_b, _ = orc.sync_step(g_h, c_h, scale, seed + 1)
        assert np.array_equal(host_bits(b_static), want_b), replay
        assert np.array_equal(host_f32(u_static), want_u), replay
        assert_f32_parity(host_f32(c_static), c_h, f"c after replay {replay}")
        # eager work between replays
        scratch = torch.randn(1000, device="cuda").sum().item()
        assert np.isfinite(scratch)


def test_resume_from_saved_compensation_reproduces_the_run():
    """The only state carried between rounds is the compensation (and the caller's seed schedule):
    restarting from a saved c at round k reproduces rounds k.. bit for bit, and launching the same
    round twice gives the same result (no hidden state, no run-to-run nondeterminism)."""
    M, d, T, k = 8, 123_457, 6, 3
    wl = workloads.Workload("resume", M=M, d=d, grid_x=0, steps=T, scale=1e-3, dist="normal", std=0.05)
    grads = [workloads.make_gradients(wl, t, seed=77, device="cuda") for t in range(T)]
    c = workloads.zero_compensation(wl, device="cuda")
    u = torch.empty(d, dtype=torch.float32, device="cuda")
    b = marsit.new_bitmap(d)
    history = []
    saved_c = None
    for t in range(T):
        if t == k:
            saved_c = c.clone()
        marsit.marsit_ring_step_sim(grads[t], c, u, b, wl.scale, workloads.step_seed(500, t))
        torch.cuda.synchronize()
        history.append((u.clone(), b.clone(), c.clone()))
    c2 = saved_c.clone()
    for t in range(k, T):
        marsit.marsit_ring_step_sim(grads[t], c2, u, b, wl.scale, workloads.step_seed(500, t))
        torch.cuda.synchronize()
        assert torch.equal(u, history[t][0]) and torch.equal(b, history[t][1]) and torch.equal(c2, history[t][2])
    # a different seed at round k changes the merged signs (the seed really is the only randomness)
    c3 = saved_c.clone()
    marsit.marsit_ring_step_sim(grads[k], c3, u, b, wl.scale, workloads.step_seed(501, k))
    torch.cuda.synchronize()
    assert not torch.equal(b, history[k][1])


@pytest.mark.parametrize("schedule,M,grid_x,K", [("ring", 8, 0, 10), ("torus", 16, 4, 7), ("tree", 8, 0, 1000), ("torus", 7, 3, 6),
                                                ("ring", 3, 0, 1)])
def test_marsit_sgd_follows_the_auxiliary_sequence(schedule, M, grid_x, K):
    """Appendix B: y_t = x_t - mean_m c_t^(m) moves exactly like plain SGD with the mean gradient,
    y_{t+1} = y_t - mean_m g_t^(m), whichever branch of Algorithm 1 a round takes.  Checked on a noisy
    quadratic, where the loss must also go down."""
    from paper_2204_06787_amd.sgd import MarsitSGD
    d, T, eta_l, eta_s = 200_003, 40, 0.05, 5e-3
    gen = torch.Generator(device="cuda").manual_seed(123)
    target = torch.randn(d, generator=gen, device="cuda")
    x = torch.zeros(d, dtype=torch.float32, device="cuda")
    opt = MarsitSGD(x, M=M, K=K, eta_s=eta_s, seed=99, schedule=schedule, grid_x=grid_x)
    y = x.double().clone()                                   # y_0 = x_0 - 0
    loss0 = float(((x - target) ** 2).mean())
    for t in range(T):
        noise = torch.randn((M, d), generator=gen, device="cuda") * 0.5
        grads = ((x - target).unsqueeze(0) + noise) * eta_l     # eta_l * grad f_m(x_t; xi)
        grads = grads.float().contiguous()
        opt.step(grads)
        y -= grads.double().mean(dim=0)
    torch.cuda.synchronize()
    got = x.double() - opt.c.double().mean(dim=0)
    assert float((got - y).abs().max()) <= 1e-4               # fp32 rounding of T rounds, values of order 1
    assert bool((opt.update.abs() == np.float32(eta_s)).all()) or (T - 1) % K == 0
    assert float(((x - target) ** 2).mean()) < 0.9 * loss0
    assert opt.t == T


@pytest.mark.parametrize("K,printed", [(50, 1.62), (100, 1.31), (200, 1.16)])
def test_rounds_taken_by_the_library_give_the_printed_average_bits(K, printed):
    """Fig. 4(b): 1.62 / 1.31 / 1.16 bits per element for K = 50 / 100 / 200.  The branch of
    Algorithm 1 is chosen inside the library (marsit_round); a full-precision round is recognised
    here by what it does -- it leaves the bitmap untouched and zeroes the compensation -- and costs
    32 bits per element, a one-bit round 1."""
    M, d = 2, 192
    g = torch.full((M, d), 0.25, dtype=torch.float32, device="cuda")
    c = torch.zeros((M, d), dtype=torch.float32, device="cuda")
    x = torch.zeros(d, dtype=torch.float32, device="cuda")
    bits = marsit.new_bitmap(d)
    full = 0
    for t in range(K):
        bits.fill_(0x5A5A)
        marsit.marsit_round(t, K, marsit.SCHEDULE_RING, 0, g, c, x, None, bits, 1e-3, 7 + t)
        torch.cuda.synchronize()
        untouched = bool((bits == 0x5A5A).all())
        assert untouched == (not bool(c.any()))
        full += int(untouched)
    assert full == 1
    assert round((32 * full + (K - full)) / K, 2) == printed

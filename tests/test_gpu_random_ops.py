"""Seeded random sizes, offsets and parameters through the per-worker entry points against the
oracle (the whole-pass entry points have their own file)."""

import numpy as np
import pytest
import torch

from oracle import marsit_oracle as orc
from paper_2204_06787_amd import marsit

pytestmark = pytest.mark.gpu

OPS = ["compress", "hop_merge", "weighted", "compress_hop_merge", "fold", "decode", "decode_apply", "momentum",
       "adam", "votes", "cascade_ring"]


def _vec(a: np.ndarray, off: int) -> torch.Tensor:
    base = torch.zeros(a.size + 8, dtype=torch.float32, device="cuda")
    v = base[off:off + a.size]
    v.copy_(torch.from_numpy(a).cuda())
    return v


def _bits(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(a.view(np.int64).copy()).cuda()


def _host_bits(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint64)


def _size(rng) -> int:
    return int(rng.choice([rng.integers(1, 130), rng.integers(130, 5000), 64 * int(rng.integers(1, 300)),
                           rng.integers(5000, 200_000)]))


@pytest.mark.parametrize("chunk", range(8))
def test_random_ops(chunk):
    rng = np.random.default_rng(314_159 + chunk)
    for it in range(50):
        op = str(rng.choice(OPS))
        n = _size(rng)
        W = orc.n_words(n)
        off = int(rng.choice([0, 0, 1, 3]))
        seed = int(rng.integers(0, 2**63))
        word_begin = int(rng.choice([0, 17, 2**31 - W - 1 if W < 2**20 else 0]))
        hop = int(rng.integers(0, 1 << 18))
        case = f"chunk={chunk} it={it} op={op} n={n} off={off} seed={seed} word_begin={word_begin} hop={hop}"
        print(case, flush=True)
        g_h = rng.standard_normal(n).astype(np.float32)
        c_h = (0.4 * rng.standard_normal(n)).astype(np.float32)
        recv_h = rng.integers(0, 2**64, size=W, dtype=np.uint64)
        local_h = rng.integers(0, 2**64, size=W, dtype=np.uint64)
        tail = np.uint64((1 << (n % 64)) - 1) if n % 64 else np.uint64(0xFFFFFFFFFFFFFFFF)

        if op == "compress":
            out = marsit.new_bitmap(n).fill_(-1)
            marsit.marsit_compress(_vec(g_h, off), _vec(c_h, off), out, d=n)
            torch.cuda.synchronize()
            assert np.array_equal(_host_bits(out), orc.sign_pack(orc.add_compensation(g_h, c_h))), case
        elif op == "hop_merge":
            fold = int(rng.integers(1, 65))
            out = marsit.marsit_hop_merge(_bits(recv_h), _bits(local_h), marsit.new_bitmap(n), word_begin, W, fold,
                                          hop, seed)
            torch.cuda.synchronize()
            assert np.array_equal(_host_bits(out), orc.hop_merge(recv_h, local_h, word_begin, fold, hop, seed)), case
        elif op == "weighted":
            w_recv, w_local = int(rng.integers(0, 64)), int(rng.integers(1, 64))
            out = marsit.marsit_hop_merge_weighted(_bits(recv_h), _bits(local_h), marsit.new_bitmap(n), word_begin, W,
                                                   w_recv, w_local, hop, seed)
            torch.cuda.synchronize()
            want = orc.hop_merge_weighted(recv_h, local_h, word_begin, w_recv, w_local, hop, seed)
            assert np.array_equal(_host_bits(out), want), case
        elif op == "compress_hop_merge":
            fold = int(rng.integers(1, 65))
            recv_h[-1] &= tail
            want = orc.hop_merge(recv_h, orc.sign_pack(orc.add_compensation(g_h, c_h)), word_begin, fold, hop, seed)
            out = _bits(recv_h)
            marsit.marsit_compress_hop_merge(out, _vec(g_h, off), _vec(c_h, off), out, word_begin, fold, hop, seed, n=n)
            torch.cuda.synchronize()
            assert np.array_equal(_host_bits(out), want), case
        elif op == "fold":
            K = int(rng.integers(1, 20))
            first = int(rng.integers(0, K))
            base = hop & ~0xFF
            maps_h = rng.integers(0, 2**64, size=(K, W + 3), dtype=np.uint64)
            want = maps_h[first, :W].copy()
            for h in range(1, K):
                want = orc.hop_merge(want, np.ascontiguousarray(maps_h[(first + h) % K, :W]), word_begin, h + 1,
                                     base | h, seed)
            out = marsit.marsit_fold_segments(_bits(maps_h.reshape(-1)).view(K, W + 3), K, first, marsit.new_bitmap(n),
                                              word_begin, W, base, seed)
            torch.cuda.synchronize()
            assert np.array_equal(_host_bits(out), want), case
        elif op in ("decode", "decode_apply"):
            scale = float(rng.choice([1e-3, 0.25, -1.5]))
            want_u = orc.decode(local_h, scale, n)
            want_c = orc.compensate(orc.add_compensation(g_h, c_h), want_u)
            c_d, u_d = _vec(c_h, off), _vec(np.zeros(n, dtype=np.float32), off)
            if op == "decode":
                marsit.marsit_decode_compensate(_bits(local_h), _vec(g_h, off), c_d, scale, u_d, c_d, d=n)
            else:
                x_h = rng.standard_normal(n).astype(np.float32)
                x_d = _vec(x_h, off)
                marsit.marsit_decode_compensate_apply(_bits(local_h), _vec(g_h, off), c_d, scale, x_d, u_d, c_d, d=n)
                torch.cuda.synchronize()
                want_x = orc.apply_update(x_h.copy(), want_u)
                assert np.array_equal(x_d.cpu().numpy().view(np.uint32), want_x.view(np.uint32)), case
            torch.cuda.synchronize()
            assert np.array_equal(u_d.cpu().numpy().view(np.uint32), want_u.view(np.uint32)), case
            assert np.array_equal(c_d.cpu().numpy().view(np.uint32), want_c.view(np.uint32)), case
        elif op == "momentum":
            M = int(rng.integers(1, 9))
            d = max(1, n // M)
            ld = d + int(rng.choice([0, 1, 4]))
            buf_h = rng.standard_normal((M, ld)).astype(np.float32)
            grad_h = rng.standard_normal((M, ld)).astype(np.float32)
            beta, eta = float(rng.choice([0.0, 0.5, 0.9, 0.99])), float(rng.choice([1.0, 0.1, 3e-4]))
            buf_d = torch.from_numpy(buf_h).cuda()
            grad_d = torch.from_numpy(grad_h).cuda()
            want_g = orc.local_momentum(buf_h, grad_h, beta, eta, d=d)
            marsit.marsit_local_momentum(buf_d, grad_d, grad_d, beta, eta, d=d)
            torch.cuda.synchronize()
            assert np.array_equal(buf_d.cpu().numpy().view(np.uint32), buf_h.view(np.uint32)), case
            assert np.array_equal(grad_d.cpu().numpy()[:, :d].view(np.uint32), want_g[:, :d].view(np.uint32)), case
            assert np.array_equal(grad_d.cpu().numpy()[:, d:], grad_h[:, d:]), case
        elif op == "adam":
            M = int(rng.integers(1, 9))
            d = max(1, n // M)
            ld = d + int(rng.choice([0, 1, 4]))
            p_h = (0.1 * rng.standard_normal((M, ld))).astype(np.float32)
            q_h = (0.01 * rng.standard_normal((M, ld)) ** 2).astype(np.float32)
            grad_h = (rng.standard_normal((M, ld)) * 10.0 ** rng.uniform(-6, 3, size=(M, ld))).astype(np.float32)
            b1, b2 = float(rng.choice([0.0, 0.5, 0.9])), float(rng.choice([0.0, 0.9, 0.999]))
            eps, eta = float(rng.choice([1e-8, 1e-3, 1.0])), float(rng.choice([1.0, 0.1, 3e-4]))
            t = int(rng.integers(1, 2000))
            bias1, bias2 = 1.0 - b1 ** t, 1.0 - b2 ** t
            p_d, q_d, grad_d = torch.from_numpy(p_h).cuda(), torch.from_numpy(q_h).cuda(), torch.from_numpy(grad_h).cuda()
            want_g = orc.local_adam(p_h, q_h, grad_h, b1, b2, eps, eta, bias1, bias2, d=d)
            marsit.marsit_local_adam(p_d, q_d, grad_d, grad_d, b1, b2, eps, eta, bias1, bias2, d=d)
            torch.cuda.synchronize()
            assert np.array_equal(p_d.cpu().numpy().view(np.uint32), p_h.view(np.uint32)), case
            assert np.array_equal(q_d.cpu().numpy().view(np.uint32), q_h.view(np.uint32)), case
            assert np.array_equal(grad_d.cpu().numpy()[:, :d].view(np.uint32), want_g[:, :d].view(np.uint32)), case
            assert np.array_equal(grad_d.cpu().numpy()[:, d:], grad_h[:, d:]), case
        elif op == "votes":
            M = int(rng.integers(1, 17))
            d = max(1, n // M)
            g2 = rng.standard_normal((M, d)).astype(np.float32)
            c2 = (0.2 * rng.standard_normal((M, d))).astype(np.float32)
            gd, cd = torch.from_numpy(g2).cuda(), torch.from_numpy(c2).cuda()
            agg = marsit.marsit_aggregate_sign(gd, cd, marsit.new_bitmap(d))
            maj = marsit.marsit_majority_vote(gd, cd, marsit.new_bitmap(d))
            count = torch.zeros(1, dtype=torch.int64, device="cuda")
            marsit.marsit_count_matching(agg, maj, d, count)
            torch.cuda.synchronize()
            want_agg, want_maj = orc.aggregate_sign(g2, c2), orc.majority_vote(g2, c2)
            assert np.array_equal(_host_bits(agg), want_agg) and np.array_equal(_host_bits(maj), want_maj), case
            assert int(count.item()) == orc.count_matching(want_agg, want_maj, d), case
        elif op == "cascade_ring":
            M = int(rng.integers(1, 9))
            d = max(1, n // M)
            g2 = rng.standard_normal((M, d)).astype(np.float32)
            c2 = (0.2 * rng.standard_normal((M, d))).astype(np.float32)
            want_u, want_b, want_n = orc.cascade_ring_step(g2, c2, seed)
            u = torch.empty(d, dtype=torch.float32, device="cuda")
            b = marsit.new_bitmap(d).fill_(-1)
            norms = torch.zeros(M, dtype=torch.float32, device="cuda")
            marsit.marsit_cascade_ring_step_sim(torch.from_numpy(g2).cuda(), torch.from_numpy(c2).cuda(), u, b, norms,
                                                marsit.new_cascade_workspace(), seed)
            torch.cuda.synchronize()
            assert np.array_equal(norms.cpu().numpy(), want_n), case
            assert np.array_equal(_host_bits(b), want_b), case
            assert np.array_equal(u.cpu().numpy().view(np.uint32), want_u.view(np.uint32)), case
        else:
            raise AssertionError(op)

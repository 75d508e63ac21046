"""Single-stream entry points under HIP graph capture.

Every entry point only launches kernels on the stream it is given (no allocation, no memset, no
synchronisation), so a caller can record a round into a graph and replay it.  Each case records one
call, replays the graph three times with eager library calls and synchronisations in between, and
checks every replay bit for bit against the same call made eagerly on copies of the same operands
(which the parity tests tie to the oracle).  The seed and the round counter are call arguments and
are therefore fixed in a recorded graph: every replay repeats the recorded round.
"""

import numpy as np
import pytest
import torch

from paper_2204_06787_amd import marsit
from gpu_util import dev, host_bits, host_f32

pytestmark = pytest.mark.gpu

SCALE = 1e-3


def _operands(M, d, seed):
    rng = np.random.default_rng(seed)
    g = rng.standard_normal((M, d)).astype(np.float32)
    c = (0.3 * rng.standard_normal((M, d))).astype(np.float32)
    x = rng.standard_normal(d).astype(np.float32)
    return dev(g), dev(c), dev(x)


def _state(c0, x0, d):
    return {"c": c0.clone(), "x": x0.clone(),
            "update": torch.full((d,), 3.0, dtype=torch.float32, device="cuda"),
            "bits": marsit.new_bitmap(d).fill_(0x33)}


def _same(a, b, what):
    assert np.array_equal(host_bits(a["bits"]), host_bits(b["bits"])), f"bitmap, {what}"
    for k in ("update", "c", "x"):
        assert np.array_equal(host_f32(a[k]).view(np.uint32), host_f32(b[k]).view(np.uint32)), f"{k}, {what}"


def _record_and_replay(label, M, d, call, seed):
    """call(g, state, stream): one library call on the given stream."""
    print(f"graph capture: {label} M={M} d={d}", flush=True)
    g, c0, x0 = _operands(M, d, seed)
    want = _state(c0, x0, d)
    call(g, want, None)                                    # eager, also the first use of this shape
    torch.cuda.synchronize()

    st = _state(c0, x0, d)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        call(g, st, torch.cuda.current_stream())
    torch.cuda.synchronize()

    other = _state(c0, x0, d)
    for replay in range(3):
        for k, src in (("c", c0), ("x", x0)):
            st[k].copy_(src)
        st["update"].fill_(3.0)
        st["bits"].fill_(0x33)
        call(g, other, None)                               # the program's own eager work between replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        _same(st, want, f"{label}, replay {replay}")


def test_fused_pass_replays():
    def ring(g, s, stream):
        marsit.marsit_ring_step_sim(g, s["c"], s["update"], s["bits"], SCALE, 77, stream=stream)
    _record_and_replay("ring, compiled schedule", 8, 70_016, ring, seed=1)
    _record_and_replay("ring, staged kernel and ragged tail", 20, 9_001, ring, seed=2)

    def torus(g, s, stream):
        marsit.marsit_ring_step_sim(g, s["c"], s["update"], s["bits"], SCALE, 78, grid_x=4, stream=stream)
    _record_and_replay("4x4 torus", 16, 33_000, torus, seed=3)

    def tree(g, s, stream):
        marsit.marsit_tree_step_sim(g, s["c"], s["update"], s["bits"], SCALE, 79, stream=stream)
    _record_and_replay("tree", 9, 12_345, tree, seed=4)


def test_round_replays():
    def one_bit(g, s, stream):
        marsit.marsit_round(3, 4, marsit.SCHEDULE_RING, 0, g, s["c"], s["x"], s["update"], s["bits"], SCALE, 80,
                            stream=stream)
    _record_and_replay("round of Algorithm 2, one-bit branch", 8, 50_000, one_bit, seed=5)

    def full(g, s, stream):
        marsit.marsit_round(4, 4, marsit.SCHEDULE_RING, 0, g, s["c"], s["x"], s["update"], s["bits"], SCALE, 81,
                            stream=stream)
    _record_and_replay("round of Algorithm 2, full-precision branch", 8, 50_000, full, seed=6)


def test_multi_kernel_entry_points_replay():
    def exchange_static(g, s, stream):
        marsit.marsit_exchange_step_sim_static(g, s["c"], s["update"], s["bits"], SCALE, 82, stream=stream)
    _record_and_replay("one exchange step on the static workspace (24 launches)", 8, 40_003, exchange_static,
                       seed=7)

    M, d = 4, 20_000
    ws = torch.empty(marsit.marsit_chain_workspace_words(M, d, 0), dtype=torch.int64, device="cuda")

    def chain(g, s, stream):
        marsit.marsit_chain_step_sim(g, s["c"], s["update"], s["bits"], ws, SCALE, 83, stream=stream)
    _record_and_replay("hop-by-hop chain (24 launches)", M, d, chain, seed=8)

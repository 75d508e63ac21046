"""Marsit-driven SGD (Algorithm 2 of the paper) for M workers simulated on one GPU.

A thin driver: it owns the state Algorithm 2 carries between rounds (the model ``x``, the
compensation vectors ``c``, the round counter) and makes one library call per round
(``marsit_round``: Algorithm 1 over the chosen schedule -- the one-bit pass, or the full-precision
round every ``K`` rounds, decided inside the library -- with the model update in the same pass).
All arithmetic and every decision of the method run in the library.
"""

from __future__ import annotations

import torch

from . import marsit


class MarsitSGD:
    def __init__(self, x: torch.Tensor, M: int, K: int, eta_s: float, seed: int,
                 schedule: str = "ring", grid_x: int = 0, momentum: float = 0.0):
        """``x``: the model, float32 ``[d]`` in device memory, updated in place.
        ``K``: a full-precision round whenever ``t mod K == 0`` (``t`` starts at 0).
        ``schedule``: ``"ring"`` (``grid_x`` = 0), ``"torus"`` (``grid_x`` columns; if they do not divide
        ``M`` the last row is short) or ``"tree"``.
        ``momentum``: heavy-ball coefficient of the workers' local optimizer (Section 5 of the paper
        trains the image models with Momentum); used by :meth:`step_from_raw_gradients`."""
        if schedule not in ("ring", "torus", "tree"):
            raise ValueError("schedule must be ring, torus or tree")
        if not (x.is_cuda and x.dtype == torch.float32 and x.dim() == 1 and x.is_contiguous()):
            raise TypeError("x: need a contiguous 1-D float32 tensor in device memory")
        if K < 1:
            raise ValueError("K must be at least 1")
        self.x, self.M, self.K, self.eta_s, self.seed = x, int(M), int(K), float(eta_s), int(seed)
        self.schedule = schedule
        self._schedule_id = {"ring": marsit.SCHEDULE_RING, "torus": marsit.SCHEDULE_TORUS,
                             "tree": marsit.SCHEDULE_TREE}[schedule]
        self.grid_x = int(grid_x) if schedule == "torus" else 0
        if schedule == "torus" and not 1 <= self.grid_x <= self.M:
            raise ValueError("torus: grid_x must be in 1..M")
        d = x.numel()
        self.c = torch.zeros((self.M, d), dtype=torch.float32, device=x.device)     # c_0 = 0
        self.update = torch.empty(d, dtype=torch.float32, device=x.device)
        self.bits = marsit.new_bitmap(d, device=x.device)
        self.momentum = float(momentum)
        self.buf = None                                     # [M, d] momentum buffers, made on first use
        self.t = 0

    def step_from_raw_gradients(self, grads: torch.Tensor, eta_l: float, stream=None) -> torch.Tensor:
        """One round from the workers' unscaled stochastic gradients ``[M, d]``: the local momentum
        buffers are advanced and ``eta_l`` times the buffers goes into the synchronisation.
        ``grads`` is overwritten with that scaled input."""
        if self.buf is None:
            self.buf = torch.zeros_like(self.c)
        marsit.marsit_local_momentum(self.buf, grads, grads, self.momentum, eta_l, stream=stream)
        return self.step(grads, stream=stream)

    def step(self, scaled_grads: torch.Tensor, stream=None) -> torch.Tensor:
        """One round.  ``scaled_grads``: ``[M, d]`` float32, worker m's stochastic gradient already
        multiplied by the local step size.  Returns the global update that was applied to ``x``."""
        seed = (self.seed + self.t) & 0xFFFFFFFFFFFFFFFF
        marsit.marsit_round(self.t, self.K, self._schedule_id, self.grid_x, scaled_grads, self.c, self.x,
                            self.update, self.bits, self.eta_s, seed, stream=stream)
        self.t += 1
        return self.update

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
                 schedule: str = "ring", grid_x: int = 0, momentum: float = 0.0,
                 optimizer: str = "momentum", betas=(0.9, 0.999), eps: float = 1e-8):
        """``x``: the model, float32 ``[d]`` in device memory, updated in place.
        ``K``: a full-precision round whenever ``t mod K == 0`` (``t`` starts at 0).
        ``schedule``: ``"ring"`` (``grid_x`` = 0), ``"torus"`` (``grid_x`` columns; if they do not divide
        ``M`` the last row is short) or ``"tree"``.
        ``optimizer``: the workers' local optimizer behind :meth:`step_from_raw_gradients`, as
        Section 5 of the paper names them: ``"momentum"`` (heavy ball with coefficient ``momentum``,
        the image models) or ``"adam"`` (``betas``, ``eps``; the sentiment-analysis model)."""
        if schedule not in ("ring", "torus", "tree"):
            raise ValueError("schedule must be ring, torus or tree")
        if not (x.is_cuda and x.dtype == torch.float32 and x.dim() == 1 and x.is_contiguous()):
            raise TypeError("x: need a contiguous 1-D float32 tensor in device memory")
        if K < 1:
            raise ValueError("K must be at least 1")
        if optimizer not in ("momentum", "adam"):
            raise ValueError("optimizer must be momentum or adam")
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
        self.optimizer, self.betas, self.eps = optimizer, (float(betas[0]), float(betas[1])), float(eps)
        self.buf = None                 # [M, d] momentum buffers / Adam first moments, made on first use
        self.buf2 = None                # [M, d] Adam second moments
        self.t = 0

    def step_from_raw_gradients(self, grads: torch.Tensor, eta_l: float, stream=None) -> torch.Tensor:
        """One round from the workers' unscaled stochastic gradients ``[M, d]``: the local optimizer's
        state is advanced and its step, scaled by ``eta_l``, goes into the synchronisation.
        ``grads`` is overwritten with that scaled input."""
        if self.buf is None:
            self.buf = torch.zeros_like(self.c)
        if self.optimizer == "adam":
            if self.buf2 is None:
                self.buf2 = torch.zeros_like(self.c)
            b1, b2 = self.betas
            rounds = self.t + 1         # the bias corrections depend on the round only
            marsit.marsit_local_adam(self.buf, self.buf2, grads, grads, b1, b2, self.eps, eta_l,
                                     1.0 - b1 ** rounds, 1.0 - b2 ** rounds, stream=stream)
        else:
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

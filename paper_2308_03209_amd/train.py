"""Algorithm 1 as a loop: the partitions this process holds are trained back to back in every
iteration, their gradients summed in place (Eq. 2's sum over i; the way the paper simulates
many partitions, Appendix C), then one update of the shared parameters is taken.

Only call sequencing and buffer plumbing: every arithmetic step is a kernel behind `binding`.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Optional, Sequence

import torch

from . import binding as B
from .model import Model, PartitionRunner


@dataclass
class PartitionData:
    run: PartitionRunner
    X: torch.Tensor          # features of the partition's nodes, on the device, in the runner's dtype
    y: torch.Tensor          # labels (int32) / targets, on the device
    mask_seed: int = 0       # seed of the per-iteration DropEdge-K choice
    custom_w: Optional[torch.Tensor] = None


class Trainer:
    def __init__(self, model: Model, parts: Sequence[PartitionData], scale_c: float, optimizer: str = "sgd",
                 lr: float = 0.01, weight_kind: int = B.W_DAR, b1: float = 0.9, b2: float = 0.999, eps: float = 1e-8):
        if optimizer not in ("sgd", "adam"):
            raise ValueError(optimizer)
        self.model, self.parts, self.c = model, list(parts), float(scale_c)
        self.opt = B.ADAM if optimizer == "adam" else B.SGD
        self.lr, self.b1, self.b2, self.eps = lr, b1, b2, eps
        self.weight_kind = weight_kind
        self.iteration = 0
        self._loss_log: List[torch.Tensor] = []

    def step(self, record_loss: bool = False) -> None:
        """One iteration of Algorithm 1 (lines 7-11) over all partitions; enqueues only."""
        t = self.iteration
        for i, p in enumerate(self.parts):
            p.run.iteration(p.X, p.y, t, p.mask_seed, self.weight_kind, self.c, accumulate=i > 0, custom_w=p.custom_w)
            if record_loss:
                self._loss_log.append(p.run.loss.clone())      # device copy; read back in losses()
        self.model.step(self.opt, self.lr, self.b1, self.b2, self.eps)
        self.iteration += 1

    def fit(self, n_iters: int, record_loss: bool = True) -> List[List[float]]:
        for _ in range(n_iters):
            self.step(record_loss)
        return self.losses()

    def losses(self) -> List[List[float]]:
        """Per recorded iteration, the per-partition losses (synchronises)."""
        if not self._loss_log:
            return []
        flat = torch.cat(self._loss_log).cpu().tolist()
        n = len(self.parts)
        return [flat[i:i + n] for i in range(0, len(flat), n)]

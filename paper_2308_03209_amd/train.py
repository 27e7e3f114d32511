"""Algorithm 1 as a loop: the partitions this process holds are trained back to back in every
iteration, their gradients summed in place (Eq. 2's sum over i; the way the paper simulates
many partitions, Appendix C), then one update of the shared parameters is taken.

Only call sequencing and buffer plumbing: every arithmetic step is a kernel behind `binding`.

`graphs=True` replays an iteration as one HIP graph: small workloads are bound by the forty-odd kernel
launches of a step, not by the kernels.  The library's calls only enqueue kernels on the current stream (no
allocation, no memset, no synchronisation), so a step can be captured as it is.  What a captured step bakes
in are the scalar arguments of its launches, hence the conditions: SGD (Adam's step count is such a scalar)
and no dropout (the iteration number is the dropout counter); the per-iteration DropEdge-K choice selects
among graphs, one per combination of mask indices seen.
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
                 lr: float = 0.01, weight_kind: int = B.W_DAR, b1: float = 0.9, b2: float = 0.999, eps: float = 1e-8,
                 graphs: bool = False):
        if optimizer not in ("sgd", "adam"):
            raise ValueError(optimizer)
        if graphs and (optimizer != "sgd" or any(p.run.q > 0.0 for p in parts)):
            raise ValueError("graphs=True needs SGD and no dropout (their per-iteration scalars would be baked in)")
        self.model, self.parts, self.c = model, list(parts), float(scale_c)
        self.opt = B.ADAM if optimizer == "adam" else B.SGD
        self.lr, self.b1, self.b2, self.eps = lr, b1, b2, eps
        self.weight_kind = weight_kind
        self.iteration = 0
        self._loss_log: List[torch.Tensor] = []
        self.graphs = bool(graphs)
        self._graphs = {}   # mask indices of the partitions -> captured step
        self._seen = set()  # combinations that have run eagerly once (first-use set-up done outside capture)

    def _mask_ids(self, t: int):
        return tuple(B.dropedge_pick(p.mask_seed, t, p.run.masks.count) if p.run.masks is not None else 0
                     for p in self.parts)

    def step(self, record_loss: bool = False) -> None:
        """One iteration of Algorithm 1 (lines 7-11) over all partitions; enqueues only."""
        t = self.iteration
        if self.graphs and not record_loss:
            key = self._mask_ids(t)
            g = self._graphs.get(key)
            if g is None and key in self._seen:
                g = torch.cuda.CUDAGraph()
                t_model = self.model.t
                with torch.cuda.graph(g):    # records the launches, runs nothing
                    self._enqueue(t, False)
                self.model.t = t_model
                self._graphs[key] = g
            if g is not None:
                g.replay()
                self.model.t += 1
                self.iteration += 1
                return
            self._seen.add(key)
        self._enqueue(t, record_loss)
        self.iteration += 1

    def _enqueue(self, t: int, record_loss: bool) -> None:
        for i, p in enumerate(self.parts):
            p.run.iteration(p.X, p.y, t, p.mask_seed, self.weight_kind, self.c, accumulate=i > 0, custom_w=p.custom_w)
            if record_loss:
                self._loss_log.append(p.run.loss.clone())      # device copy; read back in losses()
        self.model.step(self.opt, self.lr, self.b1, self.b2, self.eps)

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

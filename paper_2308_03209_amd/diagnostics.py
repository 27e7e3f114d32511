"""Diagnostics around the cut: how far the sum of the partitions' gradients is from the gradient on the
uncut graph (the objective of Eq. 2, evaluated for a given reweighting), and the replication factor (Eq. 1).

Call sequencing only; the gradients, their difference and the norms are computed by the library's kernels.
"""
from __future__ import annotations

from typing import Callable, Dict, List, Sequence, Tuple

import numpy as np
import torch

from . import binding as B
from .model import Model, PartitionRunner


def replication_factor(n_nodes: int, partitions: Sequence[B.Partition]) -> float:
    """Eq. 1: (1/|V|) * sum_i |V[i]| (cofree_replication_factor)."""
    return B.replication_factor(n_nodes, partitions)


def gradient_gap(kind: str, dims, layers: List[Dict[str, np.ndarray]], n_nodes: int, src: np.ndarray,
                 dst: np.ndarray, n_parts: int, seed_cut: int, weight_kind: int,
                 features: Callable[[np.ndarray, int], np.ndarray], labels: Callable[[np.ndarray, int], np.ndarray],
                 cut_flags: int = 0, scale_c: float = 1.0, loss: str = "softmax_ce") -> Tuple[float, float, float]:
    """Returns (||g_full - sum_i g_i||_F, ||g_full||_F, replication factor) for one parameter setting.

    g_full: gradient of the loss on the uncut graph (one partition holding every edge, unit weights);
    g_i: gradient of partition i's reweighted loss.  No DropEdge, no dropout: the gap of the cut alone.
    features(global_ids, d) / labels(global_ids, C) supply the inputs of a node set.
    """
    d_in, n_cls = dims[0][0], dims[-1][2]

    def run_part(model: Model, part: B.Partition, wk: int, accumulate: bool) -> None:
        ids = part.host_array(B.ARR_LOCAL2GLOBAL)
        X = torch.from_numpy(features(ids, d_in)).cuda()
        y = torch.from_numpy(labels(ids, n_cls)).cuda()
        run = PartitionRunner(part, model, None, loss=loss)
        run.forward(X, 0, 0)
        run.loss_backward(y, wk, scale_c, 0, 0, accumulate)

    full_model, sum_model = Model(kind, dims), Model(kind, dims)
    full_model.load(layers)
    sum_model.load(layers)
    full = B.build_partition(n_nodes, src, dst, 1, 0, seed_cut)
    run_part(full_model, full, B.W_NONE, False)
    parts = []
    for i in range(n_parts):
        part = B.build_partition(n_nodes, src, dst, n_parts, i, seed_cut, flags=cut_flags | B.WITH_RF)
        run_part(sum_model, part, weight_kind, i > 0)
        parts.append(part)
    out = torch.zeros(2, dtype=torch.float32, device="cuda")
    ws = torch.empty(B.loss_workspace_bytes(), dtype=torch.uint8, device="cuda")
    B.grad_gap(full_model.grad, sum_model.grad, out, ws)
    gap, ref = out.cpu().tolist()
    return gap, ref, replication_factor(n_nodes, parts)

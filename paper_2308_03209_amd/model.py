"""Buffers and call sequence of one training iteration on one partition (Algorithm 1 lines 6-12).

This module only allocates device memory with torch and issues the library's calls in
order: layer_fwd x L, loss_weighted, layer_bwd x L, step.  All arithmetic runs in the HIP
kernels behind `binding`.
"""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np
import torch

from . import binding as B

_KIND = {"gcn": B.GCN, "sage": B.SAGE_MEAN, "sage_conv": B.SAGE_CONV}
_DTYPE = {"f32": (B.F32, torch.float32), "bf16": (B.BF16, torch.bfloat16)}
_NAMES = {"gcn": ("W", "bW"), "sage": ("W", "bW", "U", "bU"), "sage_conv": ("W", "bW")}


def param_shapes(kind: str, dims: Sequence[Tuple[int, int, int]]) -> List[Dict[str, Tuple[int, ...]]]:
    out = []
    for (d_in, d_msg, d_out) in dims:
        if kind == "sage":
            out.append({"W": (d_msg, d_in), "bW": (d_msg,), "U": (d_out, d_msg + d_in), "bU": (d_out,)})
        elif kind == "sage_conv":
            out.append({"W": (d_out, 2 * d_in), "bW": (d_out,)})
        else:
            out.append({"W": (d_out, d_in), "bW": (d_out,)})
    return out


class Model:
    """Parameters, gradients and Adam state as single flat float32 device buffers with per-tensor views."""

    def __init__(self, kind: str, dims: Sequence[Tuple[int, int, int]], device="cuda"):
        self.kind = kind
        self.dims = list(dims)
        self.shapes = param_shapes(kind, dims)
        total = 0
        self.slices = []
        for layer in self.shapes:
            sl = {}
            for name in _NAMES[kind]:
                n = int(np.prod(layer[name]))
                n_pad = (n + 63) // 64 * 64          # keep every tensor 256-byte aligned
                sl[name] = (total, n, layer[name])
                total += n_pad
            self.slices.append(sl)
        self.theta = torch.zeros(total, dtype=torch.float32, device=device)
        self.grad = torch.zeros(total, dtype=torch.float32, device=device)
        self.m = None
        self.v = None
        self.t = 0

    def _views(self, flat) -> List[Dict[str, torch.Tensor]]:
        return [{k: flat[o:o + n].view(shape) for k, (o, n, shape) in sl.items()} for sl in self.slices]

    @property
    def params(self):
        return self._views(self.theta)

    @property
    def grads(self):
        return self._views(self.grad)

    def load(self, layers: Sequence[Dict[str, np.ndarray]]) -> None:
        for views, src in zip(self.params, layers):
            for k, v in views.items():
                v.copy_(torch.from_numpy(np.ascontiguousarray(src[k], dtype=np.float32)))

    def step(self, kind: int = B.SGD, lr: float = 0.01, b1=0.9, b2=0.999, eps=1e-8) -> None:
        if kind == B.ADAM and self.m is None:
            self.m = torch.zeros_like(self.theta)
            self.v = torch.zeros_like(self.theta)
        self.t += 1
        B.step(kind, self.theta, self.grad, self.m, self.v, lr, b1, b2, eps, self.t)


class BufferPool:
    """Device buffers shared by the runners of several partitions that are trained one after the other:
    every request is served from one allocation per (tag, columns, dtype), sized for the largest partition."""

    def __init__(self, max_rows: int, device="cuda"):
        self.max_rows, self.device, self.bufs = int(max_rows), device, {}

    def rows(self, tag, n: int, cols: int, dtype) -> torch.Tensor:
        key = (tag, cols, dtype)
        if key not in self.bufs:
            self.bufs[key] = torch.empty((self.max_rows, cols), dtype=dtype, device=self.device)
        return self.bufs[key][:n]

    def raw(self, tag, nbytes: int) -> torch.Tensor:
        key = (tag, "raw")
        if key not in self.bufs or self.bufs[key].numel() < nbytes:
            self.bufs[key] = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        return self.bufs[key]


class PartitionRunner:
    """Activation / scratch buffers of one partition and the forward-loss-backward call sequence."""

    def __init__(self, part: B.Partition, model: Model, masks: Optional[B.Masks] = None, dropout_q: float = 0.0,
                 dropout_seed: int = 0, device="cuda", dtype: str = "f32", pool: Optional[BufferPool] = None,
                 loss: str = "softmax_ce", fuse_gates: bool = True):
        """loss: "softmax_ce" (labels int32 [n]) or "sigmoid_bce" (multi-label targets uint8 [n, C]).
        fuse_gates: between two layers that end in ReLU, the upper layer's backward writes its input
        gradient already gated and scaled by the lower layer's ReLU and dropout (one elementwise pass
        less per layer).
        dtype: storage of features / activations / activation gradients ("f32" or "bf16");
        parameters, their gradients and the loss are always float32.  pool: share buffers with the runners
        of other partitions (which then must not run concurrently)."""
        self.part, self.model, self.masks = part, model, masks
        if loss not in ("softmax_ce", "sigmoid_bce"):
            raise ValueError(loss)
        self.loss_kind = loss
        self.fuse_gates = bool(fuse_gates)
        self.q, self.dseed = float(dropout_q), int(dropout_seed)
        self.dtype_code, self.torch_dtype = _DTYPE[dtype]
        n = part.num_nodes
        self.n = n
        L = len(model.dims)
        td = self.torch_dtype

        def buf(tag, cols):
            if pool is not None:
                return pool.rows(tag, n, cols, td)
            return torch.empty((n, cols), dtype=td, device=device)

        self.H = [None] + [buf(("H", l), d_out) for l, (_, _, d_out) in enumerate(model.dims)]
        self.saved = []
        for l, (d_in, d_msg, d_out) in enumerate(model.dims):
            if model.kind == "sage":
                self.saved.append({"Z": buf(("Z", l), d_msg), "A": buf(("A", l), d_msg)})
            elif d_in <= d_out:
                self.saved.append({"A": buf(("A", l), d_in)})
            else:
                self.saved.append({})
        # gradient w.r.t. each layer's input (none for the first layer: features need no gradient);
        # a layer's input gradient is dead once the layer below has consumed it, so two buffers alternate
        self.dH = [None] + [buf(("dH", l % 2), d_in) for l, (d_in, _, _) in enumerate(model.dims[1:], start=1)]
        self.dlogits = buf(("dlogits", 0), model.dims[-1][2])
        self.loss = torch.zeros(1, dtype=torch.float32, device=device)
        ws = B.loss_workspace_bytes()
        for l in range(L):
            d = self.desc(l, 0)
            ws = max(ws, B.layer_workspace_bytes(d, n, False), B.layer_workspace_bytes(d, n, True))
        self.workspace = pool.raw("workspace", ws) if pool is not None else torch.empty(ws, dtype=torch.uint8,
                                                                                        device=device)

    def desc(self, l: int, epoch: int) -> B.LayerDesc:
        d_in, d_msg, d_out = self.model.dims[l]
        last = l == len(self.model.dims) - 1
        act = 1 if (self.model.kind in ("gcn", "sage_conv") and not last) else 0
        q = 0.0 if last else self.q
        flags, q_below = 0, 0.0
        if self.fuse_gates and self.model.kind in ("gcn", "sage_conv"):
            if l > 0:
                flags |= B.GRAD_IN_GATED    # layer l-1 ends in ReLU and dropout with rate self.q
                q_below = self.q
            if not last:
                flags |= B.GRAD_OUT_GATED   # layer l+1 gates and scales what it hands down
        return B.layer_desc(_KIND[self.model.kind], d_in, d_msg, d_out, act, q, l, self.dseed, epoch, self.dtype_code,
                            flags, q_below)

    def forward(self, X: torch.Tensor, mask_id: int = 0, epoch: int = 0) -> torch.Tensor:
        if X.dtype != self.torch_dtype:
            raise ValueError(f"features must be {self.torch_dtype}")
        self.H[0] = X
        prm = self.model.params
        for l in range(len(self.model.dims)):
            B.layer_fwd(self.part, self.masks, mask_id, self.desc(l, epoch), self.H[l], prm[l], self.H[l + 1],
                        self.saved[l], self.workspace)
        return self.H[-1]

    def loss_backward(self, labels: torch.Tensor, weight_kind: int = B.W_DAR, scale_c: float = 1.0,
                      mask_id: int = 0, epoch: int = 0, accumulate: bool = False, custom_w=None,
                      train_mask=None) -> None:
        C = self.model.dims[-1][2]
        loss_fn = B.loss_weighted if self.loss_kind == "softmax_ce" else B.loss_bce_weighted
        loss_fn(self.part, weight_kind, custom_w, self.H[-1], labels, train_mask, C, scale_c, self.loss,
                self.dlogits, self.workspace, self.dtype_code)
        prm, grd = self.model.params, self.model.grads
        d_out = self.dlogits
        for l in range(len(self.model.dims) - 1, -1, -1):
            d_in = self.dH[l] if l > 0 else None
            B.layer_bwd(self.part, self.masks, mask_id, self.desc(l, epoch), self.H[l], self.H[l + 1], prm[l],
                        self.saved[l], d_out, d_in, grd[l], accumulate, self.workspace)
            d_out = d_in

    def iteration(self, X, labels, epoch: int, mask_seed: int = 0, weight_kind: int = B.W_DAR,
                  scale_c: float = 1.0, accumulate: bool = False, custom_w=None) -> int:
        """Pick the iteration's mask, forward, loss, backward.  Returns the mask index used."""
        k = B.dropedge_pick(mask_seed, epoch, self.masks.count) if self.masks is not None else 0
        self.forward(X, k, epoch)
        self.loss_backward(labels, weight_kind, scale_c, k, epoch, accumulate, custom_w)
        return k

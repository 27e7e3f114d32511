"""ctypes binding of libcofree.so: argument marshalling only.

Every function here has the name of the C entry point it calls (without the `cofree_`
prefix where that reads better as a method) and does no arithmetic of its own: torch is
used for device memory and for the current HIP stream.  If the library has not been built
the import of this module fails loudly - there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

import numpy as np
import torch  # imported before the library on purpose: libcofree.so must bind to the HIP runtime torch loaded

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libcofree.so")

OK, EINVAL, ENOMEM, EHIP, ESTATE = 0, 1, 2, 3, 4
F32, BF16 = 0, 1
GCN, SAGE_MEAN, SAGE_CONV = 0, 1, 2
W_DAR, W_NONE, W_CUSTOM, W_INV_RF = 0, 1, 2, 3
SGD, ADAM = 0, 1
GRAD_IN_GATED, GRAD_OUT_GATED = 1, 2
DEDUP, HOST_ONLY, WITH_RF, CUT_DBH = 1, 2, 4, 8
AGG_MEAN, AGG_MEAN_T, AGG_GCN = 0, 1, 2
(ARR_LOCAL2GLOBAL, ARR_ROWPTR, ARR_COL, ARR_EID, ARR_DEG_LOCAL, ARR_DEG_GLOBAL, ARR_DAR_WEIGHT,
 ARR_EDGE_LO, ARR_EDGE_HI, ARR_RF) = range(10)
_ARR_DTYPE = {ARR_LOCAL2GLOBAL: np.int64, ARR_ROWPTR: np.int64, ARR_COL: np.int32, ARR_EID: np.int32,
              ARR_DEG_LOCAL: np.int32, ARR_DEG_GLOBAL: np.int32, ARR_DAR_WEIGHT: np.float32,
              ARR_EDGE_LO: np.int32, ARR_EDGE_HI: np.int32, ARR_RF: np.int32}

# every symbol include/cofree.h declares
EXPORTS = [
    "cofree_last_error", "cofree_device_count", "cofree_layer_desc_size",
    "cofree_build_partition", "cofree_partition_free", "cofree_partition_num_nodes",
    "cofree_partition_num_edges", "cofree_partition_num_nnz", "cofree_partition_host_array",
    "cofree_partition_device_array",
    "cofree_partition_builder_begin", "cofree_partition_builder_add_edges", "cofree_partition_builder_finish",
    "cofree_partition_builder_free", "cofree_replication_factor",
    "cofree_dropedge_k", "cofree_masks_free", "cofree_masks_count", "cofree_masks_host_bits",
    "cofree_masks_host_graph", "cofree_dropedge_pick",
    "cofree_aggregate",
    "cofree_layer_workspace_bytes", "cofree_layer_fwd", "cofree_layer_bwd",
    "cofree_loss_workspace_bytes", "cofree_loss_weighted", "cofree_loss_weighted_static", "cofree_loss_bce_weighted",
    "cofree_grad_gap", "cofree_step", "cofree_dense_nt_f32",
    "cofree_profile_enable", "cofree_profile_read",
]


class CofreeError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"cofree error {code}: {msg}")
        self.code = code


class LayerDesc(C.Structure):
    _fields_ = [("kind", C.c_int32), ("dtype", C.c_int32), ("d_in", C.c_int32), ("d_msg", C.c_int32),
                ("d_out", C.c_int32), ("act", C.c_int32), ("dropout_q", C.c_float), ("layer_id", C.c_int32),
                ("seed", C.c_uint64), ("epoch", C.c_uint64), ("grad_flags", C.c_uint32), ("dropout_q_below", C.c_float)]


class KernelStat(C.Structure):
    _fields_ = [("name", C.c_char * 96), ("launches", C.c_int64), ("ms_total", C.c_double),
                ("alg_bytes", C.c_double), ("alg_flops", C.c_double)]


class LayerParams(C.Structure):
    _fields_ = [("W", C.c_void_p), ("bW", C.c_void_p), ("U", C.c_void_p), ("bU", C.c_void_p)]


class LayerGrads(C.Structure):
    _fields_ = [("W", C.c_void_p), ("bW", C.c_void_p), ("U", C.c_void_p), ("bU", C.c_void_p)]


class LayerSaved(C.Structure):
    _fields_ = [("Z", C.c_void_p), ("A", C.c_void_p)]


def _load() -> C.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2308_03209_amd.build` first "
                          "(there is no fallback for the HIP library)")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64, u32, u64, f32, f64, sz = (C.c_void_p, C.c_int32, C.c_int64, C.c_uint32, C.c_uint64, C.c_float,
                                            C.c_double, C.c_size_t)
    P = C.POINTER
    sig = {
        "cofree_last_error": (C.c_char_p, []),
        "cofree_device_count": (i32, []),
        "cofree_layer_desc_size": (sz, []),
        "cofree_build_partition": (i32, [i64, i64, vp, vp, i32, i32, u64, vp, u32, P(vp)]),
        "cofree_partition_free": (None, [vp]),
        "cofree_partition_builder_begin": (i32, [i64, i32, i32, u64, u32, P(vp)]),
        "cofree_partition_builder_add_edges": (i32, [vp, i64, vp, vp]),
        "cofree_partition_builder_finish": (i32, [vp, P(vp)]),
        "cofree_partition_builder_free": (None, [vp]),
        "cofree_replication_factor": (i32, [i64, P(vp), i32, P(f64)]),
        "cofree_partition_num_nodes": (i64, [vp]),
        "cofree_partition_num_edges": (i64, [vp]),
        "cofree_partition_num_nnz": (i64, [vp]),
        "cofree_partition_host_array": (i32, [vp, i32, P(vp), P(i64)]),
        "cofree_partition_device_array": (i32, [vp, i32, P(vp), P(i64)]),
        "cofree_dropedge_k": (i32, [vp, i32, f64, u64, u32, vp, P(vp)]),
        "cofree_masks_free": (None, [vp]),
        "cofree_masks_count": (i32, [vp]),
        "cofree_masks_host_bits": (i32, [vp, i32, P(vp), P(i64)]),
        "cofree_masks_host_graph": (i32, [vp, i32, P(vp), P(vp), P(i64)]),
        "cofree_dropedge_pick": (i32, [u64, u64, i32, P(i32)]),
        "cofree_aggregate": (i32, [vp, vp, i32, i32, vp, vp, i32, i32, vp]),
        "cofree_layer_workspace_bytes": (sz, [P(LayerDesc), i64, i32]),
        "cofree_layer_fwd": (i32, [vp, vp, i32, P(LayerDesc), vp, P(LayerParams), vp, P(LayerSaved), vp, sz, vp]),
        "cofree_layer_bwd": (i32, [vp, vp, i32, P(LayerDesc), vp, vp, P(LayerParams), P(LayerSaved), vp, vp,
                                   P(LayerGrads), i32, vp, sz, vp]),
        "cofree_loss_workspace_bytes": (sz, []),
        "cofree_loss_weighted": (i32, [vp, i32, vp, vp, i32, vp, vp, i32, f32, vp, vp, vp, sz, vp]),
        "cofree_loss_weighted_static": (i32, [vp, i32, vp, vp, i32, vp, vp, i32, f32, vp, vp, vp]),
        "cofree_loss_bce_weighted": (i32, [vp, i32, vp, vp, i32, vp, vp, i32, f32, vp, vp, vp, sz, vp]),
        "cofree_grad_gap": (i32, [i64, vp, vp, vp, vp, sz, vp]),
        "cofree_step": (i32, [i32, i64, vp, vp, vp, vp, f32, f32, f32, f32, i64, vp]),
        "cofree_dense_nt_f32": (i32, [vp, vp, vp, vp, i64, i32, i32, i32, vp]),
        "cofree_profile_enable": (i32, [i32]),
        "cofree_profile_read": (i32, [P(KernelStat), i32, P(i32)]),
    }
    for name, (res, args) in sig.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    if lib.cofree_layer_desc_size() != C.sizeof(LayerDesc):
        raise ImportError(f"{LIB_PATH} was built with another layer descriptor layout "
                          f"({lib.cofree_layer_desc_size()} bytes, binding {C.sizeof(LayerDesc)}): rebuild it")
    return lib


lib = _load()


def last_error() -> str:
    return lib.cofree_last_error().decode()


def _check(rc: int) -> None:
    if rc != OK:
        raise CofreeError(rc, last_error())


def device_count() -> int:
    return int(lib.cofree_device_count())


def _ptr(t) -> Optional[int]:
    """Device (torch tensor) or raw pointer -> integer address; None stays NULL."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return t.data_ptr()


def _stream() -> Optional[int]:
    return torch.cuda.current_stream().cuda_stream or None


class Partition:
    """Owns a cofree_partition* (cofree_build_partition / cofree_partition_free)."""

    def __init__(self, handle: int):
        self.handle = handle

    def __del__(self):
        # at interpreter shutdown the module global may already be cleared
        if getattr(self, "handle", None) and lib is not None:
            lib.cofree_partition_free(self.handle)
            self.handle = None

    @property
    def num_nodes(self) -> int:
        return int(lib.cofree_partition_num_nodes(self.handle))

    @property
    def num_edges(self) -> int:
        return int(lib.cofree_partition_num_edges(self.handle))

    @property
    def num_nnz(self) -> int:
        return int(lib.cofree_partition_num_nnz(self.handle))

    def host_array(self, which: int) -> np.ndarray:
        p, n = C.c_void_p(), C.c_int64()
        _check(lib.cofree_partition_host_array(self.handle, which, C.byref(p), C.byref(n)))
        dt = np.dtype(_ARR_DTYPE[which])
        if n.value == 0:
            return np.empty(0, dt)
        buf = (C.c_char * (n.value * dt.itemsize)).from_address(p.value)
        return np.frombuffer(buf, dtype=dt).copy()

    def device_array(self, which: int):
        """(device pointer, element count) of an array kept on the device."""
        p, n = C.c_void_p(), C.c_int64()
        _check(lib.cofree_partition_device_array(self.handle, which, C.byref(p), C.byref(n)))
        return p.value, n.value


def build_partition(n_nodes: int, src: np.ndarray, dst: np.ndarray, n_parts: int, part_id: int, seed: int,
                    assignment: Optional[np.ndarray] = None, flags: int = 0) -> Partition:
    src = np.ascontiguousarray(src, dtype=np.int64)
    dst = np.ascontiguousarray(dst, dtype=np.int64)
    if src.shape != dst.shape or src.ndim != 1:
        raise ValueError("src/dst must be 1-d arrays of equal length")
    a_ptr = None
    if assignment is not None:
        assignment = np.ascontiguousarray(assignment, dtype=np.int32)
        if assignment.shape != src.shape:
            raise ValueError("assignment must have one entry per edge")
        a_ptr = assignment.ctypes.data
    out = C.c_void_p()
    _check(lib.cofree_build_partition(n_nodes, src.shape[0], src.ctypes.data, dst.ctypes.data, n_parts, part_id,
                                      seed, a_ptr, flags, C.byref(out)))
    return Partition(out.value)


def replication_factor(n_nodes_full: int, partitions: Sequence[Partition]) -> float:
    """Eq. 1 over the given partitions of one cut."""
    arr = (C.c_void_p * len(partitions))(*[p.handle for p in partitions])
    out = C.c_double()
    _check(lib.cofree_replication_factor(n_nodes_full, arr, len(partitions), C.byref(out)))
    return float(out.value)


class PartitionBuilder:
    """Owns a cofree_partition_builder* between cofree_partition_builder_begin and _finish / _free."""

    def __init__(self, n_nodes: int, n_parts: int, part_id: int, seed: int, flags: int = 0):
        out = C.c_void_p()
        _check(lib.cofree_partition_builder_begin(n_nodes, n_parts, part_id, seed, flags, C.byref(out)))
        self.handle = out.value

    def add_edges(self, src: np.ndarray, dst: np.ndarray) -> None:
        src = np.ascontiguousarray(src, dtype=np.int64)
        dst = np.ascontiguousarray(dst, dtype=np.int64)
        if src.shape != dst.shape or src.ndim != 1:
            raise ValueError("src/dst must be 1-d arrays of equal length")
        _check(lib.cofree_partition_builder_add_edges(self.handle, src.shape[0], src.ctypes.data, dst.ctypes.data))

    def finish(self) -> Partition:
        out = C.c_void_p()
        handle, self.handle = self.handle, None      # the library frees the builder, also on error
        _check(lib.cofree_partition_builder_finish(handle, C.byref(out)))
        return Partition(out.value)

    def __del__(self):
        if getattr(self, "handle", None) and lib is not None:
            lib.cofree_partition_builder_free(self.handle)
            self.handle = None


class Masks:
    """Owns a cofree_masks* (cofree_dropedge_k / cofree_masks_free)."""

    def __init__(self, handle: int, part: Partition):
        self.handle = handle
        self.part = part   # the masks refer to the partition's arrays: keep it alive

    def __del__(self):
        if getattr(self, "handle", None) and lib is not None:
            lib.cofree_masks_free(self.handle)
            self.handle = None

    @property
    def count(self) -> int:
        return int(lib.cofree_masks_count(self.handle))

    def host_bits(self, k: int) -> np.ndarray:
        p, n = C.c_void_p(), C.c_int64()
        _check(lib.cofree_masks_host_bits(self.handle, k, C.byref(p), C.byref(n)))
        if n.value == 0:
            return np.empty(0, np.uint64)
        buf = (C.c_char * (n.value * 8)).from_address(p.value)
        return np.frombuffer(buf, dtype=np.uint64).copy()

    def host_graph(self, k: int):
        rp, cp, nnz = C.c_void_p(), C.c_void_p(), C.c_int64()
        _check(lib.cofree_masks_host_graph(self.handle, k, C.byref(rp), C.byref(cp), C.byref(nnz)))
        n = self.part.num_nodes
        rowptr = np.frombuffer((C.c_char * ((n + 1) * 8)).from_address(rp.value), dtype=np.int64).copy()
        if nnz.value == 0:
            return rowptr, np.empty(0, np.int32)
        col = np.frombuffer((C.c_char * (nnz.value * 4)).from_address(cp.value), dtype=np.int32).copy()
        return rowptr, col


def dropedge_k(part: Partition, K: int, p_drop: float, seed: int, flags: int = 0) -> Masks:
    out = C.c_void_p()
    _check(lib.cofree_dropedge_k(part.handle, K, p_drop, seed, flags, _stream(), C.byref(out)))
    return Masks(out.value, part)


def dropedge_pick(seed: int, epoch: int, K: int) -> int:
    k = C.c_int32()
    _check(lib.cofree_dropedge_pick(seed, epoch, K, C.byref(k)))
    return int(k.value)


def _mh(masks: Optional[Masks]):
    return masks.handle if masks is not None else None


def aggregate(part: Partition, masks: Optional[Masks], mask_id: int, mode: int, X, Y, width: int,
              dtype: int = F32) -> None:
    _check(lib.cofree_aggregate(part.handle, _mh(masks), mask_id, mode, _ptr(X), _ptr(Y), width, dtype, _stream()))


def layer_desc(kind: int, d_in: int, d_msg: int, d_out: int, act: int = 0, dropout_q: float = 0.0, layer_id: int = 0,
               seed: int = 0, epoch: int = 0, dtype: int = F32, grad_flags: int = 0,
               dropout_q_below: float = 0.0) -> LayerDesc:
    return LayerDesc(kind, dtype, d_in, d_msg, d_out, act, dropout_q, layer_id, seed, epoch, grad_flags,
                     dropout_q_below)


def layer_workspace_bytes(desc: LayerDesc, n_nodes: int, backward: bool) -> int:
    return int(lib.cofree_layer_workspace_bytes(C.byref(desc), n_nodes, 1 if backward else 0))


def _params(p: dict, cls):
    return cls(_ptr(p.get("W")), _ptr(p.get("bW")), _ptr(p.get("U")), _ptr(p.get("bU")))


def layer_fwd(part: Partition, masks: Optional[Masks], mask_id: int, desc: LayerDesc, H_in, params: dict, H_out,
              saved: dict, workspace) -> None:
    sv = LayerSaved(_ptr(saved.get("Z")), _ptr(saved.get("A")))
    prm = _params(params, LayerParams)
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib.cofree_layer_fwd(part.handle, _mh(masks), mask_id, C.byref(desc), _ptr(H_in), C.byref(prm),
                                _ptr(H_out), C.byref(sv), _ptr(workspace), ws_bytes, _stream()))


def layer_bwd(part: Partition, masks: Optional[Masks], mask_id: int, desc: LayerDesc, H_in, H_out, params: dict,
              saved: dict, dH_out, dH_in, grads: dict, accumulate: bool, workspace) -> None:
    sv = LayerSaved(_ptr(saved.get("Z")), _ptr(saved.get("A")))
    prm = _params(params, LayerParams)
    gr = _params(grads, LayerGrads)
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib.cofree_layer_bwd(part.handle, _mh(masks), mask_id, C.byref(desc), _ptr(H_in), _ptr(H_out),
                                C.byref(prm), C.byref(sv), _ptr(dH_out), _ptr(dH_in), C.byref(gr),
                                1 if accumulate else 0, _ptr(workspace), ws_bytes, _stream()))


def loss_workspace_bytes() -> int:
    return int(lib.cofree_loss_workspace_bytes())


def loss_weighted(part: Partition, weight_kind: int, custom_w, logits, labels, train_mask, n_classes: int,
                  scale_c: float, loss_out, dlogits, workspace, dtype: int = F32) -> None:
    ws_bytes = workspace.numel() * workspace.element_size()
    _check(lib.cofree_loss_weighted(part.handle, weight_kind, _ptr(custom_w), _ptr(logits), dtype, _ptr(labels),
                                    _ptr(train_mask), n_classes, scale_c, _ptr(loss_out), _ptr(dlogits),
                                    _ptr(workspace), ws_bytes, _stream()))


def loss_weighted_static(part: Partition, weight_kind: int, custom_w, logits, labels, train_mask, n_classes: int,
                         scale_c: float, loss_out, dlogits, dtype: int = F32) -> None:
    """cofree_loss_weighted without a workspace (partial sums in the library's static device array)."""
    _check(lib.cofree_loss_weighted_static(part.handle, weight_kind, _ptr(custom_w), _ptr(logits), dtype,
                                           _ptr(labels), _ptr(train_mask), n_classes, scale_c, _ptr(loss_out),
                                           _ptr(dlogits), _stream()))


def loss_bce_weighted(part: Partition, weight_kind: int, custom_w, logits, targets, train_mask, n_classes: int,
                      scale_c: float, loss_out, dlogits, workspace, dtype: int = F32) -> None:
    """targets: uint8 [n_nodes, n_classes] on the device."""
    ws_bytes = workspace.numel() * workspace.element_size()
    _check(lib.cofree_loss_bce_weighted(part.handle, weight_kind, _ptr(custom_w), _ptr(logits), dtype, _ptr(targets),
                                        _ptr(train_mask), n_classes, scale_c, _ptr(loss_out), _ptr(dlogits),
                                        _ptr(workspace), ws_bytes, _stream()))


def grad_gap(g_full, g_sum, out, workspace) -> None:
    """out[0] = ||g_full - g_sum||_F, out[1] = ||g_full||_F (float32 device tensors; out has 2 elements)."""
    if g_full.numel() != g_sum.numel():
        raise ValueError("gradient buffers differ in size")
    ws_bytes = workspace.numel() * workspace.element_size()
    _check(lib.cofree_grad_gap(g_full.numel(), _ptr(g_full), _ptr(g_sum), _ptr(out), _ptr(workspace), ws_bytes,
                               _stream()))


def step(kind: int, theta, grad, m=None, v=None, lr: float = 0.01, b1: float = 0.9, b2: float = 0.999,
         eps: float = 1e-8, t: int = 1) -> None:
    _check(lib.cofree_step(kind, theta.numel(), _ptr(theta), _ptr(grad), _ptr(m), _ptr(v), lr, b1, b2, eps, t,
                           _stream()))


def dense_nt_f32(A, B, bias, Cout, relu: bool) -> None:
    M, K = A.shape
    N = B.shape[0]
    _check(lib.cofree_dense_nt_f32(_ptr(A), _ptr(B), _ptr(bias), _ptr(Cout), M, N, K, 1 if relu else 0, _stream()))


def profile_enable(on: bool) -> None:
    _check(lib.cofree_profile_enable(1 if on else 0))


def profile_read() -> dict:
    """{kernel name: dict(launches, ms_total, alg_bytes, alg_flops)}; waits for the recorded events."""
    arr = (KernelStat * 256)()
    n = C.c_int32()
    _check(lib.cofree_profile_read(arr, 256, C.byref(n)))
    return {arr[i].name.decode(): dict(launches=int(arr[i].launches), ms_total=float(arr[i].ms_total),
                                       alg_bytes=float(arr[i].alg_bytes), alg_flops=float(arr[i].alg_flops))
            for i in range(n.value)}

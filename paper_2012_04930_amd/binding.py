"""Thin ctypes binding of libgcn355.so: argument marshalling only.

Every step of the training path runs in the library's HIP kernels.  PyTorch supplies
device memory (tensors own the workspaces) and the stream.  There is no CPU fallback:
if the library has not been built, importing this module's `lib()` raises.
The Python functions carry the same names as the C entry points in include/gcn355.h and
include/gcn355_debug.h.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libgcn355.so")

GCN_F32, GCN_BF16 = 0, 1
GCN_T_W, GCN_T_DW, GCN_T_H, GCN_T_LOGITS, GCN_T_G, GCN_T_DZ = 0, 1, 2, 3, 4, 5

STATUS = {0: "GCN_OK", -1: "GCN_EINVAL", -2: "GCN_EGRAPH", -3: "GCN_ELABEL", -4: "GCN_EWORKSPACE", -5: "GCN_EHIP"}

EXPORTS = [
    "gcn_last_error", "gcn_graph_workspace_bytes", "gcn_graph_create", "gcn_graph_destroy", "gcn_graph_info",
    "gcn_graph_get_csr", "gcn_graph_tile_info", "gcn_graph_get_tiles", "gcn_graph_get_masked_pattern", "gcn_aggregate_workspace_bytes", "gcn_aggregate", "gcn_aggregate_static", "gcn_model_workspace_bytes",
    "gcn_model_create", "gcn_model_destroy", "gcn_set_weights", "gcn_get_tensor", "gcn_forward", "gcn_loss_acc",
    "gcn_loss_acc_counts", "gcn_backward", "gcn_sgd_step", "gcn_timing_enable", "gcn_timing_reset", "gcn_timing_read",
    "gcn_calibration_copy", "gcn_set_tunable", "gcn_adam_step", "gcn_adam_update",
    "gcn_augment_workspace_bytes", "gcn_augment_partition", "gcn_gather_rows", "gcn_average_weights", "gcn_xcc_ids",
    "gcn_sage_workspace_bytes", "gcn_sage_create", "gcn_sage_destroy", "gcn_sage_set_weights", "gcn_sage_forward",
    "gcn_sage_loss_acc", "gcn_sage_backward", "gcn_sage_adam_step", "gcn_sage_get_tensor",
    "gcn_ceiling_gather", "gcn_ceiling_mfma_bf16",
]

_lib = None


class GcnError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__("%s (%d): %s" % (STATUS.get(code, "?"), code, text))
        self.code = code


def lib():
    """Load the shared library (once).  Fails loudly when it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libgcn355.so is missing at %s: build it with "
                              "`python -c 'import __graft_entry__ as g; g.build()'` "
                              "(or python paper_2012_04930_amd/build.py)" % LIB_PATH)
        L = C.CDLL(LIB_PATH)
        vp, i64, i32, sz = C.c_void_p, C.c_int64, C.c_int32, C.c_size_t
        L.gcn_last_error.restype = C.c_char_p
        L.gcn_last_error.argtypes = []
        L.gcn_graph_workspace_bytes.argtypes = [i64, i64, i32, C.c_int, C.POINTER(sz)]
        L.gcn_graph_create.argtypes = [C.POINTER(vp), i64, i64, vp, vp, vp, i32, C.c_int, vp, vp, i32, vp, sz, vp]
        L.gcn_graph_destroy.argtypes = [vp]
        L.gcn_graph_info.argtypes = [vp, C.POINTER(i64), C.POINTER(i64), C.POINTER(i64), C.POINTER(i32)]
        L.gcn_graph_get_csr.argtypes = [vp, vp, vp, vp, vp, vp]
        L.gcn_graph_tile_info.argtypes = [vp, C.POINTER(i64), C.POINTER(i64), C.POINTER(i32)]
        L.gcn_graph_get_tiles.argtypes = [vp, vp, vp, vp, vp, vp, C.POINTER(i64), vp]
        L.gcn_graph_get_masked_pattern.argtypes = [vp, vp, vp, C.POINTER(i64), vp]
        L.gcn_aggregate_workspace_bytes.argtypes = [vp, i32, C.c_int, C.POINTER(sz)]
        L.gcn_aggregate.argtypes = [vp, vp, vp, i32, C.c_int, vp, sz, vp]
        L.gcn_aggregate_static.argtypes = [vp, vp, vp, i32, C.c_int, vp]
        L.gcn_model_workspace_bytes.argtypes = [vp, i32, C.POINTER(i32), C.c_int, C.POINTER(sz)]
        L.gcn_model_create.argtypes = [C.POINTER(vp), vp, i32, C.POINTER(i32), C.c_int, C.c_float, C.c_uint64, vp, sz,
                                       vp]
        L.gcn_model_destroy.argtypes = [vp]
        L.gcn_set_weights.argtypes = [vp, vp, C.c_int, vp]
        L.gcn_get_tensor.argtypes = [vp, C.c_int, C.c_int, vp, sz, vp]
        L.gcn_forward.argtypes = [vp, C.c_int, vp]
        L.gcn_loss_acc.argtypes = [vp, C.POINTER(C.c_float), C.POINTER(C.c_float), vp]
        L.gcn_loss_acc_counts.argtypes = [vp, C.POINTER(i64), C.POINTER(i64), vp]
        L.gcn_backward.argtypes = [vp, vp]
        L.gcn_sgd_step.argtypes = [vp, C.c_float, vp]
        L.gcn_sage_workspace_bytes.argtypes = [vp, i32, i32, i32, i32, C.POINTER(sz)]
        L.gcn_sage_create.argtypes = [C.POINTER(vp), vp, i32, i32, i32, i32, C.c_uint64, vp, sz, vp]
        L.gcn_sage_destroy.argtypes = [vp]
        L.gcn_sage_set_weights.argtypes = [vp, vp, vp, vp]
        L.gcn_sage_forward.argtypes = [vp, vp, i32, C.c_uint64, vp]
        L.gcn_sage_loss_acc.argtypes = [vp, C.POINTER(C.c_float), C.POINTER(C.c_float), C.POINTER(i64), vp]
        L.gcn_sage_backward.argtypes = [vp, vp]
        L.gcn_sage_adam_step.argtypes = [vp, C.c_float, C.c_float, C.c_float, C.c_float, vp]
        L.gcn_sage_get_tensor.argtypes = [vp, C.c_int, vp, sz, vp]
        L.gcn_timing_enable.argtypes = [C.c_int]
        L.gcn_timing_reset.argtypes = []
        L.gcn_timing_read.argtypes = [i32, i32, C.POINTER(i64), C.POINTER(C.c_double)]
        L.gcn_ceiling_gather.argtypes = [vp, i64, i32, i64, i32, C.c_int, vp, vp]
        L.gcn_ceiling_mfma_bf16.argtypes = [i64, i32, vp, vp]
        L.gcn_calibration_copy.argtypes = [vp, vp, sz, vp]
        L.gcn_set_tunable.argtypes = [C.c_char_p, i64]
        L.gcn_augment_workspace_bytes.argtypes = [i64, C.POINTER(sz)]
        L.gcn_augment_partition.argtypes = [i64, i64, vp, vp, vp, i32, i32, C.c_double, C.c_uint64, vp, sz,
                                            C.POINTER(i64), C.POINTER(i64), C.POINTER(i64), vp, vp, vp, vp]
        L.gcn_gather_rows.argtypes = [vp, sz, vp, i64, vp, vp]
        L.gcn_xcc_ids.argtypes = [vp, i32, vp]
        L.gcn_average_weights.argtypes = [C.POINTER(vp), i32, vp]
        L.gcn_adam_step.argtypes = [vp, C.c_float, C.c_float, C.c_float, C.c_float, vp]
        L.gcn_adam_update.argtypes = [vp, vp, vp, vp, sz, C.c_float, C.c_float, C.c_float, C.c_float, i64, vp]
        for name in EXPORTS:
            if name != "gcn_last_error":
                getattr(L, name).restype = C.c_int
        _lib = L
    return _lib


def _check(rc: int):
    if rc != 0:
        raise GcnError(rc, lib().gcn_last_error().decode("utf-8", "replace"))


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dev(t: torch.Tensor, dtype) -> int:
    assert t.is_cuda and t.is_contiguous() and t.dtype == dtype, (t.device, t.dtype, dtype)
    return t.data_ptr()


def _workspace(nbytes: int) -> torch.Tensor:
    # torch's caching allocator returns 512-byte aligned blocks
    ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
    assert ws.data_ptr() % 256 == 0
    return ws


class Graph:
    """Owns the graph handle and the torch tensor that backs its workspace."""

    def __init__(self, handle, ws, n, f, n_classes):
        self.handle, self.ws, self.n, self.f, self.n_classes = handle, ws, n, f, n_classes

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.gcn_graph_destroy(self.handle)
            self.handle = None


def gcn_graph_create(rowptr: torch.Tensor, col: torch.Tensor, feat: torch.Tensor, labels: torch.Tensor,
                     train_mask: torch.Tensor, n_classes: int, store_dtype: int = GCN_F32) -> Graph:
    L = lib()
    n = rowptr.numel() - 1
    nnz = col.numel()
    f = feat.shape[1]
    need = C.c_size_t()
    _check(L.gcn_graph_workspace_bytes(n, nnz, f, store_dtype, C.byref(need)))
    ws = _workspace(need.value)
    h = C.c_void_p()
    _check(L.gcn_graph_create(C.byref(h), n, nnz, _dev(rowptr, torch.int64), _dev(col, torch.int32) if nnz else None,
                              _dev(feat, torch.float32), f, store_dtype, _dev(labels, torch.int32),
                              _dev(train_mask, torch.uint8), n_classes, ws.data_ptr(), ws.numel(), _stream()))
    return Graph(h, ws, n, f, n_classes)


def gcn_graph_info(g: Graph) -> dict:
    n, nnz, nt, md = C.c_int64(), C.c_int64(), C.c_int64(), C.c_int32()
    _check(lib().gcn_graph_info(g.handle, C.byref(n), C.byref(nnz), C.byref(nt), C.byref(md)))
    return {"n": n.value, "nnz": nnz.value, "n_train": nt.value, "max_degree": md.value}


def gcn_graph_get_csr(g: Graph):
    info = gcn_graph_info(g)
    rowptr = torch.empty(info["n"] + 1, dtype=torch.int64, device="cuda")
    col = torch.empty(info["nnz"], dtype=torch.int32, device="cuda")
    deg = torch.empty(info["n"], dtype=torch.int32, device="cuda")
    dinv = torch.empty(info["n"], dtype=torch.float32, device="cuda")
    _check(lib().gcn_graph_get_csr(g.handle, rowptr.data_ptr(), col.data_ptr(), deg.data_ptr(), dinv.data_ptr(),
                                   _stream()))
    return rowptr, col, deg, dinv


def gcn_graph_tile_info(g: Graph) -> dict:
    nt, nd, use = C.c_int64(), C.c_int64(), C.c_int32()
    _check(lib().gcn_graph_tile_info(g.handle, C.byref(nt), C.byref(nd), C.byref(use)))
    return {"n_tiles": nt.value, "nnz_dense": nd.value, "in_use": bool(use.value)}


TILE_ROWS = 128     # a dense tile covers 128 rows by 32 columns


def gcn_graph_get_tiles(g: Graph):
    """-> (tile_ptr, tile_col, bits [n_tiles x 128], res_rowptr, res_col)"""
    info = gcn_graph_info(g)
    ti = gcn_graph_tile_info(g)
    res_nnz = info["nnz"] - ti["nnz_dense"]
    tile_ptr = torch.empty((info["n"] + TILE_ROWS - 1) // TILE_ROWS + 1, dtype=torch.int64, device="cuda")
    tile_col = torch.empty(ti["n_tiles"], dtype=torch.int32, device="cuda")
    bits = torch.empty((ti["n_tiles"], TILE_ROWS), dtype=torch.int32, device="cuda")
    res_rowptr = torch.empty(info["n"] + 1, dtype=torch.int64, device="cuda")
    res_col = torch.empty(max(res_nnz, 1), dtype=torch.int32, device="cuda")
    got = C.c_int64()
    _check(lib().gcn_graph_get_tiles(g.handle, tile_ptr.data_ptr(), tile_col.data_ptr(), bits.data_ptr(),
                                     res_rowptr.data_ptr(), res_col.data_ptr(), C.byref(got), _stream()))
    assert got.value == res_nnz
    return tile_ptr, tile_col, bits, res_rowptr, res_col[:res_nnz]


def gcn_graph_get_masked_pattern(g: Graph):
    """-> (rowptr, col) of the pattern the last layer's backward aggregation gathers over; raises if there is none."""
    nnz = C.c_int64()
    _check(lib().gcn_graph_get_masked_pattern(g.handle, None, None, C.byref(nnz), _stream()))
    rowptr = torch.empty(g.n + 1, dtype=torch.int64, device="cuda")
    col = torch.empty(max(nnz.value, 1), dtype=torch.int32, device="cuda")
    _check(lib().gcn_graph_get_masked_pattern(g.handle, rowptr.data_ptr(), col.data_ptr(), C.byref(nnz), _stream()))
    return rowptr, col[:nnz.value]


def gcn_aggregate(g: Graph, x: torch.Tensor, dtype: int = GCN_F32, ws: torch.Tensor | None = None) -> torch.Tensor:
    """A_hat x; with dtype = GCN_BF16 the scaled input is stored as bfloat16 before the aggregation."""
    L = lib()
    assert x.shape[0] == g.n
    width = x.shape[1]
    need = C.c_size_t()
    _check(L.gcn_aggregate_workspace_bytes(g.handle, width, dtype, C.byref(need)))
    if ws is None:
        ws = _workspace(need.value)
    out = torch.empty_like(x)
    _check(L.gcn_aggregate(g.handle, _dev(x, torch.float32), out.data_ptr(), width, dtype, ws.data_ptr(), ws.numel(),
                           _stream()))
    return out


GCN_STATIC_SCRATCH_BYTES = 32 << 20


def gcn_aggregate_static(g: Graph, x: torch.Tensor, out: torch.Tensor, dtype: int = GCN_F32) -> torch.Tensor:
    """A_hat x into `out` (caller's tensors), with the library's built-in scratch array: nothing is allocated."""
    assert x.shape[0] == g.n and out.shape == x.shape
    _check(lib().gcn_aggregate_static(g.handle, _dev(x, torch.float32), _dev(out, torch.float32), x.shape[1], dtype,
                                      _stream()))
    return out


class Model:
    def __init__(self, handle, ws, graph, dims):
        self.handle, self.ws, self.graph, self.dims = handle, ws, graph, list(dims)

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.gcn_model_destroy(self.handle)
            self.handle = None


def gcn_model_create(g: Graph, dims, dtype: int = GCN_F32, dropout_p: float = 0.0, seed: int = 0) -> Model:
    L = lib()
    nl = len(dims) - 1
    arr = (C.c_int32 * (nl + 1))(*dims)
    need = C.c_size_t()
    _check(L.gcn_model_workspace_bytes(g.handle, nl, arr, dtype, C.byref(need)))
    ws = _workspace(need.value)
    h = C.c_void_p()
    _check(L.gcn_model_create(C.byref(h), g.handle, nl, arr, dtype, dropout_p, seed, ws.data_ptr(), ws.numel(),
                              _stream()))
    return Model(h, ws, g, dims)


def gcn_set_weights(m: Model, weights) -> None:
    """weights: list of [d_in, d_out] float32 arrays/tensors, or one flat tensor."""
    if isinstance(weights, (list, tuple)):
        flat = np.concatenate([np.asarray(w, dtype=np.float32).reshape(-1) for w in weights])
    else:
        flat = weights
    if isinstance(flat, torch.Tensor) and flat.is_cuda:
        _check(lib().gcn_set_weights(m.handle, _dev(flat, torch.float32), 0, _stream()))
    else:
        flat = np.ascontiguousarray(np.asarray(flat, dtype=np.float32))
        _check(lib().gcn_set_weights(m.handle, flat.ctypes.data, 1, _stream()))


def gcn_get_tensor(m: Model, which: int, layer: int = 0) -> torch.Tensor:
    n = m.graph.n
    if which == GCN_T_LOGITS:
        layer = len(m.dims) - 1
    rows = m.dims[layer - 1] if which in (GCN_T_W, GCN_T_DW) else n
    cols = m.dims[layer]
    out = torch.empty((rows, cols), dtype=torch.float32, device="cuda")
    _check(lib().gcn_get_tensor(m.handle, which, layer, out.data_ptr(), out.numel(), _stream()))
    return out


def gcn_forward(m: Model, training: bool = True) -> None:
    _check(lib().gcn_forward(m.handle, 1 if training else 0, _stream()))


def gcn_loss_acc(m: Model, sync: bool = True):
    """-> (loss, accuracy) as Python floats, or None when sync is False (work is only enqueued)."""
    if not sync:
        _check(lib().gcn_loss_acc(m.handle, None, None, _stream()))
        return None
    loss, acc = C.c_float(), C.c_float()
    _check(lib().gcn_loss_acc(m.handle, C.byref(loss), C.byref(acc), _stream()))
    return loss.value, acc.value


def gcn_loss_acc_counts(m: Model):
    """-> (correct, n_train) integers of the last gcn_loss_acc."""
    c, n = C.c_int64(), C.c_int64()
    _check(lib().gcn_loss_acc_counts(m.handle, C.byref(c), C.byref(n), _stream()))
    return c.value, n.value


def gcn_backward(m: Model) -> None:
    _check(lib().gcn_backward(m.handle, _stream()))


def gcn_sgd_step(m: Model, lr: float) -> None:
    _check(lib().gcn_sgd_step(m.handle, lr, _stream()))


# parts of gcn_timing_read (gcn_timed_part of include/gcn355_debug.h)
GCN_TIME_AGGREGATE, GCN_TIME_GATHER, GCN_TIME_TILES, GCN_TIME_PLANES, GCN_TIME_JOIN, GCN_TIME_GEMM_NN, \
    GCN_TIME_GEMM_TN, GCN_TIME_GEMM_NT, GCN_TIME_LOSS, GCN_TIME_SAGE_GATHER = range(10)


def gcn_timing_enable(level) -> None:
    """0 / False: off; 1 / True: whole aggregations; 2: also their parts, the dense products and the loss."""
    _check(lib().gcn_timing_enable(int(level)))


def gcn_timing_reset() -> None:
    _check(lib().gcn_timing_reset())


def gcn_timing_read(width: int, part: int = GCN_TIME_AGGREGATE):
    """-> (launches, total milliseconds) of the timed intervals of (part, width) since the last reset."""
    cnt, ms = C.c_int64(), C.c_double()
    _check(lib().gcn_timing_read(part, width, C.byref(cnt), C.byref(ms)))
    return cnt.value, ms.value


def gcn_ceiling_gather(table: torch.Tensor, waves: int, per_wave: int, spread: bool) -> torch.Tensor:
    """Runs the gather ceiling kernel over table [rows x row_floats float32]; -> the waves' sums."""
    rows, row_floats = table.shape
    out = torch.empty((waves, row_floats), dtype=torch.float32, device="cuda")
    _check(lib().gcn_ceiling_gather(_dev(table, torch.float32), rows, row_floats, waves, per_wave, 1 if spread else 0,
                                    out.data_ptr(), _stream()))
    return out


def gcn_ceiling_mfma_bf16(waves: int, per_wave: int) -> torch.Tensor:
    out = torch.empty((waves, 64), dtype=torch.float32, device="cuda")
    _check(lib().gcn_ceiling_mfma_bf16(waves, per_wave, out.data_ptr(), _stream()))
    return out


def gcn_calibration_copy(src: torch.Tensor, dst: torch.Tensor) -> None:
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes
    _check(lib().gcn_calibration_copy(src.data_ptr(), dst.data_ptr(), nbytes, _stream()))


def gcn_set_tunable(name: str, value: int) -> None:
    _check(lib().gcn_set_tunable(name.encode(), value))


def gcn_adam_step(m: Model, lr: float, beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8) -> None:
    _check(lib().gcn_adam_step(m.handle, lr, beta1, beta2, eps, _stream()))


def gcn_adam_update(w: torch.Tensor, dw: torch.Tensor, mom1: torch.Tensor, mom2: torch.Tensor, lr: float, step: int,
                    beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8) -> None:
    n = w.numel()
    assert dw.numel() == n and mom1.numel() == n and mom2.numel() == n
    _check(lib().gcn_adam_update(_dev(w, torch.float32), _dev(dw, torch.float32), _dev(mom1, torch.float32),
                                 _dev(mom2, torch.float32), n, lr, beta1, beta2, eps, step, _stream()))


def gcn_augment_partition(rowptr: torch.Tensor, col: torch.Tensor, part: torch.Tensor, n_parts: int, p: int,
                          overlap: float, seed: int = 0):
    """-> (vertices, n_local, rowptr_out, col_out): device tensors trimmed to their used length."""
    L = lib()
    n = rowptr.numel() - 1
    nnz = col.numel()
    need = C.c_size_t()
    _check(L.gcn_augment_workspace_bytes(n, C.byref(need)))
    ws = _workspace(need.value)
    vertices = torch.empty(n, dtype=torch.int32, device="cuda")
    rp = torch.empty(n + 1, dtype=torch.int64, device="cuda")
    cl = torch.empty(max(nnz, 1), dtype=torch.int32, device="cuda")
    n_out, n_local, nnz_out = C.c_int64(), C.c_int64(), C.c_int64()
    _check(L.gcn_augment_partition(n, nnz, _dev(rowptr, torch.int64), _dev(col, torch.int32) if nnz else None,
                                   _dev(part, torch.int32), n_parts, p, overlap, seed, ws.data_ptr(), ws.numel(),
                                   C.byref(n_out), C.byref(n_local), C.byref(nnz_out), vertices.data_ptr(),
                                   rp.data_ptr(), cl.data_ptr(), _stream()))
    return vertices[:n_out.value], n_local.value, rp[:n_out.value + 1], cl[:nnz_out.value]


def gcn_gather_rows(src: torch.Tensor, idx: torch.Tensor) -> torch.Tensor:
    """src[idx] for a contiguous 1-D or 2-D tensor whose rows are a multiple of 4 bytes."""
    assert src.is_cuda and src.is_contiguous() and idx.dtype == torch.int32
    row_elems = src.shape[1] if src.dim() == 2 else 1
    out = torch.empty((idx.numel(),) + tuple(src.shape[1:]), dtype=src.dtype, device="cuda")
    _check(lib().gcn_gather_rows(src.data_ptr(), row_elems * src.element_size(), idx.data_ptr(), idx.numel(),
                                 out.data_ptr(), _stream()))
    return out


def gcn_average_weights(models) -> None:
    arr = (C.c_void_p * len(models))(*[m.handle for m in models])
    _check(lib().gcn_average_weights(arr, len(models), _stream()))


def gcn_xcc_ids(n_blocks: int) -> torch.Tensor:
    out = torch.empty(n_blocks, dtype=torch.int32, device="cuda")
    _check(lib().gcn_xcc_ids(out.data_ptr(), n_blocks, _stream()))
    return out


# ---------------------------------------------------------------------------------------------- GraphSAGE-mean
GCN_SAGE_W1, GCN_SAGE_W2, GCN_SAGE_DW1, GCN_SAGE_DW2, GCN_SAGE_H1, GCN_SAGE_LOGITS, GCN_SAGE_C1_MEAN, \
    GCN_SAGE_INNER, GCN_SAGE_OUTER = range(9)


class Sage:
    """Owns the GraphSAGE handle and its workspace; keeps the graph alive."""

    def __init__(self, handle, ws, graph, hidden, s1, s2, max_batch):
        self.handle, self.ws, self.graph = handle, ws, graph
        self.hidden, self.s1, self.s2, self.max_batch = hidden, s1, s2, max_batch
        self.n_batch = 0

    def __del__(self):
        if getattr(self, "handle", None) and _lib is not None:
            _lib.gcn_sage_destroy(self.handle)
            self.handle = None


def gcn_sage_create(g: Graph, hidden: int, s1: int, s2: int, max_batch: int, seed: int = 0) -> Sage:
    L = lib()
    need = C.c_size_t()
    _check(L.gcn_sage_workspace_bytes(g.handle, hidden, s1, s2, max_batch, C.byref(need)))
    ws = _workspace(need.value)
    h = C.c_void_p()
    _check(L.gcn_sage_create(C.byref(h), g.handle, hidden, s1, s2, max_batch, seed, ws.data_ptr(), ws.numel(),
                             _stream()))
    return Sage(h, ws, g, hidden, s1, s2, max_batch)


def gcn_sage_set_weights(s: Sage, w1, w2) -> None:
    w1 = torch.as_tensor(w1, dtype=torch.float32).contiguous().cuda()
    w2 = torch.as_tensor(w2, dtype=torch.float32).contiguous().cuda()
    assert tuple(w1.shape) == (2 * s.graph.f, s.hidden) and tuple(w2.shape) == (2 * s.hidden, s.graph.n_classes)
    _check(lib().gcn_sage_set_weights(s.handle, w1.data_ptr(), w2.data_ptr(), _stream()))
    torch.cuda.current_stream().synchronize()       # w1, w2 may be temporaries


def gcn_sage_forward(s: Sage, batch: torch.Tensor, step: int) -> None:
    _check(lib().gcn_sage_forward(s.handle, _dev(batch, torch.int32), batch.numel(), step, _stream()))
    s.n_batch = batch.numel()


def gcn_sage_loss_acc(s: Sage, sync: bool = True):
    if not sync:
        _check(lib().gcn_sage_loss_acc(s.handle, None, None, None, _stream()))
        return None
    loss, acc, correct = C.c_float(), C.c_float(), C.c_int64()
    _check(lib().gcn_sage_loss_acc(s.handle, C.byref(loss), C.byref(acc), C.byref(correct), _stream()))
    return loss.value, acc.value, correct.value


def gcn_sage_backward(s: Sage) -> None:
    _check(lib().gcn_sage_backward(s.handle, _stream()))


def gcn_sage_adam_step(s: Sage, lr: float, beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8) -> None:
    _check(lib().gcn_sage_adam_step(s.handle, lr, beta1, beta2, eps, _stream()))


def gcn_sage_get_tensor(s: Sage, which: int) -> torch.Tensor:
    f, h, c, B = s.graph.f, s.hidden, s.graph.n_classes, s.n_batch
    n1 = B * (1 + s.s2)
    shape, dt = {
        GCN_SAGE_W1: ((2 * f, h), torch.float32), GCN_SAGE_DW1: ((2 * f, h), torch.float32),
        GCN_SAGE_W2: ((2 * h, c), torch.float32), GCN_SAGE_DW2: ((2 * h, c), torch.float32),
        GCN_SAGE_H1: ((n1, h), torch.float32), GCN_SAGE_LOGITS: ((B, c), torch.float32),
        GCN_SAGE_C1_MEAN: ((n1, f), torch.float32), GCN_SAGE_INNER: ((B, s.s2), torch.int32),
        GCN_SAGE_OUTER: ((n1, s.s1), torch.int32),
    }[which]
    out = torch.empty(shape, dtype=dt, device="cuda")
    _check(lib().gcn_sage_get_tensor(s.handle, which, out.data_ptr(), out.numel(), _stream()))
    return out

"""Python face of the CPU oracle (TEST INFRASTRUCTURE ONLY).

Only the tests, the smoke check and the benchmark's CPU-baseline leg may import this
module.  It loads `liboracle.so`, built by gcc from `gcn_oracle.c` in this folder, and
strings its plain loops together in the order the method states them:

    forward   for l = 1..L:  T = H_{l-1} W_l ;  Z_l = A_hat T ;  H_l = relu(Z_l)  (l < L)
    loss      softmax cross-entropy averaged over the train mask; accuracy (Section 2.2)
    backward  dZ_L from the loss; for l = L..1:  G = A_hat dZ_l  (A_hat is symmetric);
              dW_l = H_{l-1}^T G ;  dZ_{l-1} = (G W_l^T) * [Z_{l-1} > 0]
    update    W_l <- W_l - lr dW_l

(Section 4.1 gives the layer rule; Section 2.1 the inputs.)  Everything is fp64; the
only Python loops are over the handful of layers.  This module imports nothing from
the GPU package and the GPU package imports nothing from here.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gcn_oracle.c")
# GCN_ORACLE_SANITIZE=1 selects a build with AddressSanitizer and UndefinedBehaviorSanitizer (the process must then
# be started with libasan preloaded; tests/test_oracle_sanitized.py does that for the pins)
_SANITIZE = os.environ.get("GCN_ORACLE_SANITIZE", "0") == "1"
_LIB = os.path.join(_HERE, "liboracle_san.so" if _SANITIZE else "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile gcn_oracle.c with gcc -O2 -fopenmp into liboracle.so (next to the source)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        flags = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"] \
            if _SANITIZE else ["-O2"]
        subprocess.check_call(["gcc", *flags, "-fopenmp", "-fPIC", "-shared", "-std=c11", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def lib():
    global _lib
    if _lib is None:
        build()
        L = C.CDLL(_LIB)
        i64, i32p, i64p, f64p, u8p = C.c_int64, C.POINTER(C.c_int32), C.POINTER(C.c_int64), C.POINTER(C.c_double), \
            C.POINTER(C.c_uint8)
        L.orc_validate_csr.argtypes = [i64, i64, i64p, i32p]
        L.orc_canonical_degrees.argtypes = [i64, i64p, i32p, i32p]
        L.orc_canonical_fill.argtypes = [i64, i64p, i32p, i64p, i32p]
        L.orc_is_symmetric.argtypes = [i64, i64p, i32p]
        L.orc_dinv.argtypes = [i64, i64p, f64p]
        L.orc_dinv.restype = None
        L.orc_aggregate.argtypes = [i64, i64p, i32p, f64p, i64, f64p, f64p]
        L.orc_aggregate.restype = None
        for name in ("orc_matmul_nn", "orc_matmul_tn", "orc_matmul_nt"):
            f = getattr(L, name)
            f.argtypes = [i64, i64, i64, f64p, f64p, f64p]
            f.restype = None
        L.orc_dropout_keep.argtypes = [C.c_uint64, C.c_uint64, C.c_uint64, i64, i64, C.c_double, u8p]
        L.orc_dropout_keep.restype = None
        L.orc_relu_dropout.argtypes = [i64, f64p, u8p, C.c_double, f64p]
        L.orc_relu_dropout.restype = None
        L.orc_relu_dropout_backward.argtypes = [i64, f64p, u8p, C.c_double, f64p, f64p]
        L.orc_relu_dropout_backward.restype = None
        L.orc_loss_acc.argtypes = [i64, i64, f64p, i32p, u8p, f64p, i64p, i64p, f64p]
        L.orc_sgd.argtypes = [i64, C.c_double, f64p, f64p]
        L.orc_sgd.restype = None
        L.orc_adam.argtypes = [i64, C.c_double, C.c_double, C.c_double, C.c_double, i64, f64p, f64p, f64p, f64p]
        L.orc_adam.restype = None
        _lib = L
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(C.POINTER(ct))


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


class OracleError(ValueError):
    def __init__(self, code, what):
        super().__init__("%s (code %d)" % (what, code))
        self.code = code


# ------------------------------------------------------------------ graph
@dataclass
class Graph:
    n: int
    rowptr: np.ndarray   # int64 [n+1], canonical A + I
    col: np.ndarray      # int32 [E]
    deg: np.ndarray      # int32 [n]   row sums of A + I
    dinv: np.ndarray     # float64 [n] deg^-1/2


def canonicalise(n: int, rowptr, col, require_symmetric: bool = True) -> Graph:
    """Raw CSR of A -> canonical pattern of A + I, degrees, D^-1/2."""
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int64)
    col = np.ascontiguousarray(col, dtype=np.int32)
    L = lib()
    if rowptr.size != n + 1:
        raise OracleError(-2, "rowptr length")
    rc = L.orc_validate_csr(n, col.size, _p(rowptr, C.c_int64), _p(col, C.c_int32))
    if rc:
        raise OracleError(rc, "invalid CSR")
    deg = np.empty(n, dtype=np.int32)
    rc = L.orc_canonical_degrees(n, _p(rowptr, C.c_int64), _p(col, C.c_int32), _p(deg, C.c_int32))
    if rc:
        raise OracleError(rc, "canonical degrees")
    out_rp = np.zeros(n + 1, dtype=np.int64)
    np.cumsum(deg, out=out_rp[1:])
    out_col = np.empty(int(out_rp[-1]), dtype=np.int32)
    rc = L.orc_canonical_fill(n, _p(rowptr, C.c_int64), _p(col, C.c_int32), _p(out_rp, C.c_int64),
                              _p(out_col, C.c_int32))
    if rc:
        raise OracleError(rc, "canonical fill")
    if require_symmetric and not L.orc_is_symmetric(n, _p(out_rp, C.c_int64), _p(out_col, C.c_int32)):
        raise OracleError(-2, "adjacency is not symmetric")
    dinv = np.empty(n, dtype=np.float64)
    L.orc_dinv(n, _p(out_rp, C.c_int64), _p(dinv, C.c_double))
    return Graph(n, out_rp, out_col, deg, dinv)


# ------------------------------------------------------------------ primitive steps
def aggregate(g: Graph, T) -> np.ndarray:
    """A_hat T."""
    T = _f64(T)
    Z = np.empty_like(T)
    lib().orc_aggregate(g.n, _p(g.rowptr, C.c_int64), _p(g.col, C.c_int32), _p(g.dinv, C.c_double), T.shape[1],
                        _p(T, C.c_double), _p(Z, C.c_double))
    return Z


def matmul_nn(A, B):
    A, B = _f64(A), _f64(B)
    assert A.shape[1] == B.shape[0]
    out = np.empty((A.shape[0], B.shape[1]))
    lib().orc_matmul_nn(A.shape[0], A.shape[1], B.shape[1], _p(A, C.c_double), _p(B, C.c_double), _p(out, C.c_double))
    return out


def matmul_tn(A, B):
    """A^T B with A [k x m], B [k x n]."""
    A, B = _f64(A), _f64(B)
    assert A.shape[0] == B.shape[0]
    out = np.empty((A.shape[1], B.shape[1]))
    lib().orc_matmul_tn(A.shape[1], A.shape[0], B.shape[1], _p(A, C.c_double), _p(B, C.c_double), _p(out, C.c_double))
    return out


def matmul_nt(A, B):
    """A B^T with A [m x k], B [n x k]."""
    A, B = _f64(A), _f64(B)
    assert A.shape[1] == B.shape[1]
    out = np.empty((A.shape[0], B.shape[0]))
    lib().orc_matmul_nt(A.shape[0], A.shape[1], B.shape[0], _p(A, C.c_double), _p(B, C.c_double), _p(out, C.c_double))
    return out


def dropout_keep(seed: int, epoch: int, layer: int, rows: int, width: int, p: float) -> np.ndarray:
    keep = np.empty((rows, width), dtype=np.uint8)
    lib().orc_dropout_keep(seed, epoch, layer, rows, width, p, _p(keep, C.c_uint8))
    return keep


def loss_acc(logits, labels, mask, want_grad: bool = True):
    """-> (loss, correct, n_train, dZ_L or None)."""
    logits = _f64(logits)
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    n, c = logits.shape
    loss = C.c_double()
    correct = C.c_int64()
    ntrain = C.c_int64()
    dZ = np.empty_like(logits) if want_grad else None
    rc = lib().orc_loss_acc(n, c, _p(logits, C.c_double), _p(labels, C.c_int32), _p(mask, C.c_uint8),
                            C.byref(loss), C.byref(correct), C.byref(ntrain),
                            _p(dZ, C.c_double) if want_grad else None)
    if rc:
        raise OracleError(rc, "loss/accuracy")
    return loss.value, correct.value, ntrain.value, dZ


# ------------------------------------------------------------------ the training step
@dataclass
class Trace:
    """Everything one epoch computes, kept for element-by-element comparison."""
    T: list
    Z: list          # Z[l-1] = A_hat T_l ; Z[-1] are the logits
    H: list          # H[0] = X, H[l] = activation of layer l (l < L)
    keep: list
    loss: float = 0.0
    correct: int = 0
    n_train: int = 0
    dZ: list = None  # dZ[l-1] = dLoss/dZ_l
    G: list = None   # G[l-1]  = A_hat dZ_l
    dW: list = None


def forward(g: Graph, X, Ws, p: float = 0.0, training: bool = False, seed: int = 0, epoch: int = 0) -> Trace:
    H = [_f64(X)]
    Ts, Zs, keeps = [], [], []
    nl = len(Ws)
    for l in range(1, nl + 1):
        T = matmul_nn(H[l - 1], Ws[l - 1])
        Z = aggregate(g, T)
        Ts.append(T)
        Zs.append(Z)
        if l < nl:
            keep = dropout_keep(seed, epoch, l, Z.shape[0], Z.shape[1], p) if (training and p > 0.0) else None
            Hl = np.empty_like(Z)
            lib().orc_relu_dropout(Z.size, _p(Z, C.c_double), _p(keep, C.c_uint8) if keep is not None else None,
                                   p, _p(Hl, C.c_double))
            H.append(Hl)
            keeps.append(keep)
    return Trace(Ts, Zs, H, keeps)


def backward(g: Graph, tr: Trace, Ws, labels, mask, p: float = 0.0) -> Trace:
    """Loss, then the chain rule through the layers in descending order.  The ReLU decision [Z_l > 0] is taken on
    this trace's own fp64 pre-activations; nothing enters but the trace of `forward` and the inputs."""
    nl = len(Ws)
    tr.loss, tr.correct, tr.n_train, dZL = loss_acc(tr.Z[-1], labels, mask)
    tr.dZ = [None] * nl
    tr.G = [None] * nl
    tr.dW = [None] * nl
    tr.dZ[nl - 1] = dZL
    for l in range(nl, 0, -1):
        G = aggregate(g, tr.dZ[l - 1])
        tr.G[l - 1] = G
        tr.dW[l - 1] = matmul_tn(tr.H[l - 1], G)
        if l > 1:
            dH = matmul_nt(G, Ws[l - 1])
            Zp = tr.Z[l - 2]
            keep = tr.keep[l - 2]
            dZ = np.empty_like(dH)
            lib().orc_relu_dropout_backward(dH.size, _p(Zp, C.c_double),
                                            _p(keep, C.c_uint8) if keep is not None else None, p,
                                            _p(dH, C.c_double), _p(dZ, C.c_double))
            tr.dZ[l - 2] = dZ
    return tr


def sgd(Ws, dWs, lr: float):
    out = []
    for W, dW in zip(Ws, dWs):
        W2 = _f64(W).copy()
        d = _f64(dW)
        lib().orc_sgd(W2.size, lr, _p(d, C.c_double), _p(W2, C.c_double))
        out.append(W2)
    return out


def adam(Ws, dWs, state, lr: float, beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8):
    """One Adam step on every layer.  state = {"t": steps so far, "m": [...], "v": [...]} (updated in place;
    pass {} for a fresh optimiser).  -> new weights."""
    if not state:
        state.update(t=0, m=[np.zeros_like(_f64(W)) for W in Ws], v=[np.zeros_like(_f64(W)) for W in Ws])
    state["t"] += 1
    out = []
    for l, (W, dW) in enumerate(zip(Ws, dWs)):
        W2 = _f64(W).copy()
        d = _f64(dW)
        lib().orc_adam(W2.size, lr, beta1, beta2, eps, state["t"], _p(d, C.c_double), _p(state["m"][l], C.c_double),
                       _p(state["v"][l], C.c_double), _p(W2, C.c_double))
        out.append(W2)
    return out


def train_epoch(g: Graph, X, Ws, labels, mask, lr: float, p: float = 0.0, seed: int = 0, epoch: int = 0):
    """One full-batch epoch: forward, loss, backward, SGD.  -> (new weights, Trace)."""
    tr = forward(g, X, Ws, p=p, training=True, seed=seed, epoch=epoch)
    backward(g, tr, Ws, labels, mask, p=p)
    return sgd(Ws, tr.dW, lr), tr

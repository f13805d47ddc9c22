"""Python face of the fp64 CPU oracle (``slicegcn_oracle.c``) -- TEST INFRASTRUCTURE.

Only the tests, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may
import this package.  The HIP library and its binding never do, and this package imports
nothing from them.  All arithmetic is in the C file; this module only marshals numpy arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "slicegcn_oracle.c")
# SLICEGCN_SANITIZE=1 (with the AddressSanitizer runtime preloaded into the interpreter) runs the tests against
# a build of the same source with -fsanitize=address,undefined
_SANITIZE = os.environ.get("SLICEGCN_SANITIZE") == "1"
_LIB = os.path.join(_HERE, "libslicegcn_oracle_san.so" if _SANITIZE else "libslicegcn_oracle.so")

SYMMETRIZE = 1
ADD_SELF_LOOPS = 2


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (idempotent unless ``force``)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        opt = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-omit-frame-pointer"] if _SANITIZE else ["-O2"]
        subprocess.check_call(["gcc", *opt, "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
    return _lib


def _check(rc: int, what: str):
    if rc != 0:
        raise ValueError(f"oracle {what} failed with status {rc}")


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct)) if a is not None else None


def _f64(a, ld_ok=True):
    return np.ascontiguousarray(a, dtype=np.float64) if a is not None else None


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def set_num_threads(n: int) -> None:
    """Threads the oracle's row loops use from now on (results do not depend on it)."""
    lib().oracle_set_num_threads(ctypes.c_int(int(n)))


# ---------------------------------------------------------------------------------------
def slice_strategy(in_d: int, p: int, slice_size_scale: float = 1.0):
    """Algorithm 1 of the paper: list of (start, end) and the slice size."""
    starts = np.zeros(max(p, 1), dtype=np.int32)
    ends = np.zeros(max(p, 1), dtype=np.int32)
    size = ctypes.c_int32(0)
    rc = lib().oracle_slice_strategy(ctypes.c_int32(in_d), ctypes.c_int32(p), ctypes.c_double(slice_size_scale),
                                     _p(starts, ctypes.c_int32), _p(ends, ctypes.c_int32), ctypes.byref(size))
    _check(rc, "slice_strategy")
    return [(int(s), int(e)) for s, e in zip(starts[:p], ends[:p])], int(size.value)


@dataclass
class NormCSR:
    n: int
    rowptr: np.ndarray   # int64 [n+1]
    colidx: np.ndarray   # int32 [nnz], ascending and distinct per row
    deg: np.ndarray      # int32 [n]
    dinv: np.ndarray     # float64 [n]
    vals: np.ndarray     # float64 [nnz]

    @property
    def nnz(self) -> int:
        return int(self.rowptr[-1])


def build_norm_csr(src, dst, n_nodes: int, flags: int = SYMMETRIZE | ADD_SELF_LOOPS) -> NormCSR:
    src = np.ascontiguousarray(src, dtype=np.int64)
    dst = np.ascontiguousarray(dst, dtype=np.int64)
    if src.shape != dst.shape or src.ndim != 1:
        raise ValueError("src and dst must be 1-D arrays of equal length")
    rowptr = np.zeros(max(n_nodes, 0) + 1, dtype=np.int64)
    deg = np.zeros(max(n_nodes, 1), dtype=np.int32)
    dinv = np.zeros(max(n_nodes, 1), dtype=np.float64)
    col_p = ctypes.POINTER(ctypes.c_int32)()
    val_p = ctypes.POINTER(ctypes.c_double)()
    L = lib()
    rc = L.oracle_build_norm_csr(_p(src, ctypes.c_int64), _p(dst, ctypes.c_int64), ctypes.c_int64(src.size),
                                 ctypes.c_int64(n_nodes), ctypes.c_uint32(flags),
                                 _p(rowptr, ctypes.c_int64), _p(deg, ctypes.c_int32), _p(dinv, ctypes.c_double),
                                 ctypes.byref(col_p), ctypes.byref(val_p))
    _check(rc, "build_norm_csr")
    nnz = int(rowptr[-1])
    try:
        colidx = np.ctypeslib.as_array(col_p, shape=(max(nnz, 1),))[:nnz].copy()
        vals = np.ctypeslib.as_array(val_p, shape=(max(nnz, 1),))[:nnz].copy()
    finally:
        L.oracle_free.argtypes = [ctypes.c_void_p]
        L.oracle_free(ctypes.cast(col_p, ctypes.c_void_p))
        L.oracle_free(ctypes.cast(val_p, ctypes.c_void_p))
    return NormCSR(n_nodes, rowptr, colidx, deg[:n_nodes], dinv[:n_nodes], vals)


ORDER_DEGREE, ORDER_BFS = 1, 2
BFS_MAX_TREES = 16


def row_order(g: NormCSR, mode: int, max_trees: int = BFS_MAX_TREES) -> np.ndarray:
    """Processing order of the rows (ORDER_DEGREE or ORDER_BFS): order[p] = id of the row at position p."""
    order = np.empty(g.n, dtype=np.int32)
    rc = lib().oracle_row_order(ctypes.c_int64(g.n), _p(g.rowptr, ctypes.c_int64), _p(g.colidx, ctypes.c_int32),
                                ctypes.c_int(mode), ctypes.c_int32(max_trees), _p(order, ctypes.c_int32))
    _check(rc, "row_order")
    return order


def _csr_args(g: NormCSR):
    return (ctypes.c_int64(g.n), _p(g.rowptr, ctypes.c_int64), _p(g.colidx, ctypes.c_int32), _p(g.vals, ctypes.c_double))


def spmm(g: NormCSR, X, transpose: bool = False) -> np.ndarray:
    """Z = A^ X (or A^^T X): the aggregation sum of the layer equation."""
    X = _f64(X)
    n, w = X.shape
    if n != g.n:
        raise ValueError("X has the wrong number of rows")
    Z = np.empty((n, w), dtype=np.float64)
    rc = lib().oracle_spmm(*_csr_args(g), ctypes.c_int(int(transpose)), _p(X, ctypes.c_double), ctypes.c_int64(w),
                           ctypes.c_int32(w), _p(Z, ctypes.c_double), ctypes.c_int64(w))
    _check(rc, "spmm")
    return Z


def spmm_rows(g: NormCSR, X, rows) -> np.ndarray:
    """Selected rows of A^ X."""
    X = _f64(X)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    n, w = X.shape
    Z = np.empty((rows.size, w), dtype=np.float64)
    rc = lib().oracle_spmm_rows(*_csr_args(g), _p(X, ctypes.c_double), ctypes.c_int64(w), ctypes.c_int32(w),
                                _p(rows, ctypes.c_int64), ctypes.c_int64(rows.size), _p(Z, ctypes.c_double),
                                ctypes.c_int64(w))
    _check(rc, "spmm_rows")
    return Z


def layer_fwd(g: NormCSR, Hin, W_agg, b=None, W_self=None, b_self=None, act: int = 1):
    """Forward of one SliceGCN layer.  Returns (Hout, Z, P)."""
    Hin, W_agg, b, W_self, b_self = map(_f64, (Hin, W_agg, b, W_self, b_self))
    n, w_in = Hin.shape
    w_out = W_agg.shape[1]
    if W_agg.shape[0] != w_in or (W_self is not None and W_self.shape != W_agg.shape):
        raise ValueError("weight shapes do not match the input width")
    Z = np.empty((n, w_in)); P = np.empty((n, w_out)); Hout = np.empty((n, w_out))
    d = ctypes.c_double
    rc = lib().oracle_layer_fwd(*_csr_args(g), ctypes.c_int32(w_in), ctypes.c_int32(w_out), ctypes.c_int(act),
                                _p(Hin, d), ctypes.c_int64(w_in), _p(W_agg, d), _p(b, d), _p(W_self, d), _p(b_self, d),
                                _p(Z, d), _p(P, d), _p(Hout, d), ctypes.c_int64(w_out))
    _check(rc, "layer_fwd")
    return Hout, Z, P


def layer_bwd(g: NormCSR, Hin, Z, mask, W_agg, W_self, dHout, need_dHin: bool = True):
    """Backward of one SliceGCN layer.  ``mask`` is the n x w_out 0/1 pattern of passed activations.

    Returns dict(dW_agg, db, dW_self, db_self, dHin)."""
    Hin, Z, W_agg, W_self, dHout = map(_f64, (Hin, Z, W_agg, W_self, dHout))
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    n, w_in = Hin.shape
    w_out = W_agg.shape[1]
    if mask.shape != (n, w_out) or dHout.shape != (n, w_out) or Z.shape != (n, w_in):
        raise ValueError("shape mismatch")
    d = ctypes.c_double
    dW_agg = np.empty((w_in, w_out)); db = np.empty(w_out)
    dW_self = np.empty((w_in, w_out)); db_self = np.empty(w_out)
    dHin = np.empty((n, w_in)) if need_dHin else None
    rc = lib().oracle_layer_bwd(*_csr_args(g), ctypes.c_int32(w_in), ctypes.c_int32(w_out),
                                _p(Hin, d), ctypes.c_int64(w_in), _p(Z, d), _p(mask, ctypes.c_uint8),
                                _p(W_agg, d), _p(W_self, d), _p(dHout, d), ctypes.c_int64(w_out),
                                _p(dW_agg, d), _p(db, d), _p(dW_self, d), _p(db_self, d),
                                _p(dHin, d), ctypes.c_int64(w_in))
    _check(rc, "layer_bwd")
    return dict(dW_agg=dW_agg, db=db, dW_self=dW_self if W_self is not None else None, db_self=db_self, dHin=dHin)


def encode_concat(Hs, E=None) -> np.ndarray:
    """H = CONCAT_i (H^i + E[i, :]) -- slice encoding then concatenation."""
    Hs = [_f64(h) for h in Hs]
    k = len(Hs)
    n = Hs[0].shape[0]
    widths = np.array([h.shape[1] for h in Hs], dtype=np.int32)
    lds = np.array([h.shape[1] for h in Hs], dtype=np.int64)
    H = np.empty((n, int(widths.sum())))
    E = _f64(E)
    ptrs = (ctypes.POINTER(ctypes.c_double) * k)(*[_p(h, ctypes.c_double) for h in Hs])
    rc = lib().oracle_encode_concat(ctypes.c_int32(k), ptrs, _p(lds, ctypes.c_int64), _p(widths, ctypes.c_int32),
                                    _p(E, ctypes.c_double), ctypes.c_int64(E.shape[1] if E is not None else 0),
                                    ctypes.c_int64(n), _p(H, ctypes.c_double), ctypes.c_int64(H.shape[1]))
    _check(rc, "encode_concat")
    return H


def encode_concat_bwd(dH, widths, want_dE: bool = True):
    """Returns (list of dH^i copies, dE or None).  dE has max(widths) columns."""
    dH = _f64(dH)
    n = dH.shape[0]
    k = len(widths)
    widths = np.ascontiguousarray(widths, dtype=np.int32)
    lds = widths.astype(np.int64)
    outs = [np.empty((n, int(w))) for w in widths]
    ptrs = (ctypes.POINTER(ctypes.c_double) * k)(*[_p(o, ctypes.c_double) for o in outs])
    lde = int(widths.max())
    dE = np.zeros((k, lde)) if want_dE else None
    rc = lib().oracle_encode_concat_bwd(ctypes.c_int32(k), _p(dH, ctypes.c_double), ctypes.c_int64(dH.shape[1]),
                                        ctypes.c_int64(n), _p(widths, ctypes.c_int32), ptrs, _p(lds, ctypes.c_int64),
                                        _p(dE, ctypes.c_double), ctypes.c_int64(lde))
    _check(rc, "encode_concat_bwd")
    return outs, dE


def linear_fwd(X, W, b=None, act: int = 0):
    """Dense layer Y = act(X W + b).  Returns (Y, P) with P the pre-activation."""
    X, W, b = map(_f64, (X, W, b))
    n, w_in = X.shape
    if W.shape[0] != w_in:
        raise ValueError("weight shape does not match the input width")
    w_out = W.shape[1]
    P = np.empty((n, w_out)); Y = np.empty((n, w_out))
    d = ctypes.c_double
    rc = lib().oracle_linear_fwd(ctypes.c_int64(n), ctypes.c_int32(w_in), ctypes.c_int32(w_out), ctypes.c_int(act),
                                 _p(X, d), ctypes.c_int64(w_in), _p(W, d), _p(b, d), _p(P, d), _p(Y, d), ctypes.c_int64(w_out))
    _check(rc, "linear_fwd")
    return Y, P


def linear_bwd(X, W, mask, dY, need_dX: bool = True):
    """Backward of the dense layer for the given 0/1 activation pattern.  Returns dict(dX, dW, db)."""
    X, W, dY = map(_f64, (X, W, dY))
    n, w_in = X.shape
    w_out = W.shape[1]
    mask = np.ascontiguousarray(mask, dtype=np.uint8)
    if mask.shape != (n, w_out) or dY.shape != (n, w_out):
        raise ValueError("shape mismatch")
    d = ctypes.c_double
    dX = np.empty((n, w_in)) if need_dX else None
    dW = np.empty((w_in, w_out)); db = np.empty(w_out)
    rc = lib().oracle_linear_bwd(ctypes.c_int64(n), ctypes.c_int32(w_in), ctypes.c_int32(w_out), _p(X, d), ctypes.c_int64(w_in),
                                 _p(W, d), _p(mask, ctypes.c_uint8), _p(dY, d), ctypes.c_int64(w_out),
                                 _p(dX, d), ctypes.c_int64(w_in), _p(dW, d), _p(db, d))
    _check(rc, "linear_bwd")
    return dict(dX=dX, dW=dW, db=db)


def softmax_ce(logits, labels, want_grad: bool = True):
    """Mean softmax cross-entropy over all rows.  Returns (loss, dlogits or None)."""
    logits = _f64(logits)
    n, c = logits.shape
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    if labels.shape != (n,):
        raise ValueError("one label per row expected")
    loss = ctypes.c_double(0.0)
    dl = np.empty((n, c)) if want_grad else None
    rc = lib().oracle_softmax_ce(ctypes.c_int64(n), ctypes.c_int32(c), _p(logits, ctypes.c_double), ctypes.c_int64(c),
                                 _p(labels, ctypes.c_int32), ctypes.byref(loss), _p(dl, ctypes.c_double), ctypes.c_int64(c))
    _check(rc, "softmax_ce")
    return loss.value, dl


def adam_step(p, g, m, v, lr, t, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0):
    """One Adam step in place on the fp64 arrays p, m, v (t >= 1 is the step count)."""
    for a in (p, g, m, v):
        if a.dtype != np.float64 or not a.flags.c_contiguous or a.shape != p.shape:
            raise ValueError("contiguous fp64 arrays of one shape expected")
    d = ctypes.c_double
    rc = lib().oracle_adam_step(_p(p, d), _p(g, d), _p(m, d), _p(v, d), ctypes.c_int64(p.size), d(lr), d(beta1), d(beta2),
                                d(eps), d(weight_decay), ctypes.c_int32(t))
    _check(rc, "adam_step")


def cosine_lr(lr_max: float, lr_min: float, t: int, t_max: int) -> float:
    f = lib().oracle_cosine_lr
    f.restype = ctypes.c_double
    return float(f(ctypes.c_double(lr_max), ctypes.c_double(lr_min), ctypes.c_int32(t), ctypes.c_int32(t_max)))

"""ctypes binding of ``libslicegcn.so``: same names as the C ABI, argument marshalling only.

Tensors are torch CUDA (ROCm) tensors used purely as device memory: every function passes
``data_ptr()``, the row stride as leading dimension and the current HIP stream to the library.
No arithmetic of the method happens here, and there is no CPU fallback: if the library has not
been built, loading it raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import numpy as np
import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
# SLICEGCN_SANITIZE=1 selects the build whose host code carries sanitizer checks (CPU-only test runs)
LIB_PATH = os.path.join(_PKG, "libslicegcn_hostsan.so" if os.environ.get("SLICEGCN_SANITIZE") == "1" else "libslicegcn.so")

SYMMETRIZE = 1
ADD_SELF_LOOPS = 2
REORDER_DEGREE = 4
REORDER_BFS = 8
SCHED_SHORT_ITEMS = 16
SCHED_LONG_ITEMS = 32
ACT_NONE = 0
ACT_RELU = 1
LAYER_Z_VALID = 1
LAYER_TRANSFORM_FIRST = 2
LAYER_ORDER_AUTO = 4
LAYER_IN_SCALED = 8
LAYER_OUT_SCALED = 16

OK, EINVAL, ERANGE, ENOMEM, EHIP, EUNSUPPORTED, EWORKSPACE = 0, -1, -2, -3, -4, -5, -6

EXPORTS = [
    "slicegcn_slice_strategy", "slicegcn_build_norm_csr", "slicegcn_graph_view", "slicegcn_graph_destroy",
    "slicegcn_slice_feature", "slicegcn_scale_rows", "slicegcn_spmm_workspace_bytes", "slicegcn_spmm_slice", "slicegcn_spmm_slice_static",
    "slicegcn_layer_fwd_workspace_bytes",
    "slicegcn_layer_fwd", "slicegcn_layer_bwd_workspace_bytes",
    "slicegcn_layer_bwd", "slicegcn_concat", "slicegcn_concat_bwd_workspace_bytes", "slicegcn_concat_bwd",
    "slicegcn_strerror", "slicegcn_last_error", "slicegcn_profile_reserve", "slicegcn_profile_begin", "slicegcn_profile_end",
    "slicegcn_linear_fwd", "slicegcn_linear_bwd_workspace_bytes", "slicegcn_linear_bwd",
    "slicegcn_softmax_ce_workspace_bytes", "slicegcn_softmax_ce", "slicegcn_accumulate",
    "slicegcn_adam_step", "slicegcn_cosine_lr",
]

PROF_KINDS = {0: "spmm", 1: "dense_fwd", 2: "dense_bwd", 3: "grad_reduce", 4: "concat", 5: "spmm_add",
              6: "linear_fwd", 7: "linear_bwd", 8: "linear_grad", 9: "loss", 10: "accumulate"}


class SliceGCNError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"slicegcn status {status}: {text}")
        self.status = status


class _CsrView(ctypes.Structure):
    _fields_ = [("n_nodes", ctypes.c_int64), ("nnz", ctypes.c_int64), ("rowptr", ctypes.c_void_p),
                ("colidx", ctypes.c_void_p), ("deg", ctypes.c_void_p), ("dinv", ctypes.c_void_p),
                ("vals", ctypes.c_void_p), ("symmetric", ctypes.c_int32), ("order", ctypes.c_void_p)]


class _LayerDesc(ctypes.Structure):
    _fields_ = [("w_in", ctypes.c_int32), ("w_out", ctypes.c_int32), ("act", ctypes.c_int32), ("flags", ctypes.c_uint32)]


class _LayerParams(ctypes.Structure):
    _fields_ = [("W_agg", ctypes.c_void_p), ("b", ctypes.c_void_p), ("W_self", ctypes.c_void_p), ("b_self", ctypes.c_void_p)]


class _LayerSaved(ctypes.Structure):
    _fields_ = [("Z", ctypes.c_void_p), ("ldz", ctypes.c_int64), ("mask", ctypes.c_void_p), ("mask_words", ctypes.c_int64)]


class _ProfileEntry(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("width", ctypes.c_int32), ("launches", ctypes.c_int64),
                ("total_ms", ctypes.c_double), ("min_ms", ctypes.c_double), ("max_ms", ctypes.c_double),
                ("median_ms", ctypes.c_double)]


class _LayerGrads(ctypes.Structure):
    _fields_ = [("dW_agg", ctypes.c_void_p), ("db", ctypes.c_void_p), ("dW_self", ctypes.c_void_p), ("db_self", ctypes.c_void_p)]


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded HIP library.  Raises if it has not been built (there is no other path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2408_11500_amd.build` "
                               "(or __graft_entry__.build()); the library has no CPU fallback")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
        L.slicegcn_slice_strategy.argtypes = [i32, i32, ctypes.c_double, vp, vp, vp]
        L.slicegcn_build_norm_csr.argtypes = [vp, vp, i64, i64, ctypes.c_uint32, vp, ctypes.POINTER(vp)]
        L.slicegcn_graph_view.argtypes = [vp, ctypes.POINTER(_CsrView)]
        L.slicegcn_graph_destroy.argtypes = [vp]
        L.slicegcn_slice_feature.argtypes = [vp, i64, i64, i32, i32, vp, i64, vp]
        L.slicegcn_scale_rows.argtypes = [vp, vp, i64, i32, vp, i64, vp]
        L.slicegcn_spmm_workspace_bytes.argtypes = [vp, ctypes.c_int, i32]
        L.slicegcn_spmm_workspace_bytes.restype = sz
        L.slicegcn_spmm_slice.argtypes = [vp, ctypes.c_int, vp, i64, i32, vp, i64, vp, sz, vp]
        L.slicegcn_spmm_slice_static.argtypes = [vp, ctypes.c_int, vp, i64, i32, vp, i64, vp]
        L.slicegcn_layer_fwd_workspace_bytes.argtypes = [vp, ctypes.POINTER(_LayerDesc)]
        L.slicegcn_layer_fwd_workspace_bytes.restype = sz
        L.slicegcn_layer_fwd.argtypes = [vp, ctypes.POINTER(_LayerDesc), ctypes.POINTER(_LayerParams), vp, i64, vp, i64,
                                         ctypes.POINTER(_LayerSaved), vp, sz, vp]
        L.slicegcn_layer_bwd_workspace_bytes.argtypes = [vp, ctypes.POINTER(_LayerDesc), ctypes.c_int]
        L.slicegcn_layer_bwd_workspace_bytes.restype = sz
        L.slicegcn_layer_bwd.argtypes = [vp, ctypes.POINTER(_LayerDesc), ctypes.POINTER(_LayerParams), vp, i64,
                                         ctypes.POINTER(_LayerSaved), vp, i64, vp, i64, ctypes.POINTER(_LayerGrads),
                                         vp, sz, vp]
        L.slicegcn_concat.argtypes = [i32, vp, vp, vp, vp, i64, i64, vp, i64, vp]
        L.slicegcn_concat_bwd_workspace_bytes.argtypes = [i64, i32, vp]
        L.slicegcn_concat_bwd_workspace_bytes.restype = sz
        L.slicegcn_concat_bwd.argtypes = [i32, vp, i64, i64, vp, vp, vp, vp, i64, vp, sz, vp]
        L.slicegcn_profile_end.argtypes = [ctypes.POINTER(_ProfileEntry), i32, ctypes.POINTER(i32)]
        L.slicegcn_linear_fwd.argtypes = [vp, i64, i64, i32, i32, vp, vp, i32, vp, i64, vp, i64, vp]
        L.slicegcn_linear_bwd_workspace_bytes.argtypes = [i64, i32, i32]
        L.slicegcn_linear_bwd_workspace_bytes.restype = sz
        L.slicegcn_linear_bwd.argtypes = [vp, i64, i64, i32, i32, vp, i32, vp, i64, vp, i64, vp, i64, vp, vp, vp, sz, vp]
        L.slicegcn_softmax_ce_workspace_bytes.argtypes = [i64]
        L.slicegcn_softmax_ce_workspace_bytes.restype = sz
        L.slicegcn_softmax_ce.argtypes = [vp, i64, i64, i32, vp, vp, vp, i64, vp, sz, vp]
        L.slicegcn_accumulate.argtypes = [vp, i64, vp, i64, i64, i32, vp]
        f64 = ctypes.c_double
        L.slicegcn_adam_step.argtypes = [vp, vp, vp, vp, i64, f64, f64, f64, f64, f64, i32, vp]
        L.slicegcn_cosine_lr.argtypes = [ctypes.c_double, ctypes.c_double, i32, i32]
        L.slicegcn_cosine_lr.restype = ctypes.c_double
        L.slicegcn_strerror.argtypes = [ctypes.c_int]
        L.slicegcn_strerror.restype = ctypes.c_char_p
        L.slicegcn_last_error.restype = ctypes.c_char_p
        _lib = L
    return _lib


def _check(rc: int):
    if rc != 0:
        L = lib()
        detail = L.slicegcn_last_error().decode()
        raise SliceGCNError(rc, f"{L.slicegcn_strerror(rc).decode()}: {detail}")


def _stream() -> int:
    return int(torch.cuda.current_stream().cuda_stream)


def _mat(t: torch.Tensor, name: str, dtype=torch.float32):
    """(pointer, leading dimension) of a 2-D device tensor with unit column stride."""
    if not t.is_cuda or t.dtype != dtype or t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
        raise TypeError(f"{name}: expected a 2-D {dtype} device tensor with unit column stride")
    return t.data_ptr(), int(t.stride(0)) if t.shape[0] > 1 else max(int(t.stride(0)), int(t.shape[1]))


def _vec(t, name: str, dtype=torch.float32):
    if t is None:
        return None
    if not t.is_cuda or t.dtype != dtype or not t.is_contiguous():
        raise TypeError(f"{name}: expected a contiguous {dtype} device tensor")
    return t.data_ptr()


def _ws(ws):
    return (ws.data_ptr(), ws.numel() * ws.element_size()) if ws is not None else (None, 0)


# ---------------------------------------------------------------------------------------
def slicegcn_slice_strategy(in_d: int, p: int, slice_size_scale: float = 1.0):
    """Host call: returns ([(start, end)] * p, slice_size)."""
    n = max(int(p), 1)
    starts = (ctypes.c_int32 * n)()
    ends = (ctypes.c_int32 * n)()
    size = ctypes.c_int32(0)
    _check(lib().slicegcn_slice_strategy(in_d, p, slice_size_scale, ctypes.addressof(starts), ctypes.addressof(ends),
                                         ctypes.addressof(size)))
    return [(int(starts[i]), int(ends[i])) for i in range(p)], int(size.value)


@dataclass
class CsrView:
    n_nodes: int
    nnz: int
    rowptr: int
    colidx: int
    deg: int
    dinv: int
    vals: int
    symmetric: int
    order: int = 0


class Graph:
    """Owner of a ``slicegcn_graph`` handle.  The handle itself is read-only; ``default_ws`` hands out one
    cached device buffer for callers that pass no workspace of their own (such calls must then be ordered
    on one stream; callers that overlap calls on several streams pass one workspace per stream)."""

    def __init__(self, handle: int):
        self._h = handle
        self._ws = None

    def default_ws(self, nbytes: int):
        if nbytes == 0:
            return None
        if self._ws is None or self._ws.numel() < nbytes:
            self._ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        return self._ws

    @property
    def handle(self) -> int:
        if not self._h:
            raise ValueError("graph handle already destroyed")
        return self._h

    def view(self) -> CsrView:
        v = _CsrView()
        _check(lib().slicegcn_graph_view(self.handle, ctypes.byref(v)))
        return CsrView(v.n_nodes, v.nnz, v.rowptr or 0, v.colidx or 0, v.deg or 0, v.dinv or 0, v.vals or 0, v.symmetric,
                       v.order or 0)

    def to_host(self) -> dict:
        """Copies of the CSR arrays as numpy arrays (for checks)."""
        v = self.view()
        return dict(n=v.n_nodes, nnz=v.nnz,
                    rowptr=_to_host(v.rowptr, v.n_nodes + 1, np.int32), colidx=_to_host(v.colidx, v.nnz, np.int32),
                    deg=_to_host(v.deg, v.n_nodes, np.int32), dinv=_to_host(v.dinv, v.n_nodes, np.float32),
                    vals=_to_host(v.vals, v.nnz, np.float32),
                    order=_to_host(v.order, v.n_nodes, np.int32) if v.order else None)

    def destroy(self):
        if self._h:
            lib().slicegcn_graph_destroy(self._h)
            self._h = 0
            self._ws = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


_hip = None


def _to_host(ptr: int, count: int, dtype) -> np.ndarray:
    """Device-to-host copy of a raw device array (hipMemcpy)."""
    global _hip
    out = np.empty(count, dtype=dtype)
    if count == 0:
        return out
    if _hip is None:
        _hip = ctypes.CDLL("libamdhip64.so")
        _hip.hipMemcpy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int]
    torch.cuda.synchronize()
    rc = _hip.hipMemcpy(out.ctypes.data, ptr, out.nbytes, 2)  # 2 = device to host
    if rc != 0:
        raise RuntimeError(f"hipMemcpy failed with {rc}")
    return out


def slicegcn_build_norm_csr(src: torch.Tensor, dst: torch.Tensor, n_nodes: int,
                            flags: int = SYMMETRIZE | ADD_SELF_LOOPS) -> Graph:
    ps = _vec(src, "src", torch.int64) if src.numel() else None
    pd = _vec(dst, "dst", torch.int64) if dst.numel() else None
    if src.numel() != dst.numel():
        raise ValueError("src and dst differ in length")
    h = ctypes.c_void_p(0)
    _check(lib().slicegcn_build_norm_csr(ps, pd, src.numel(), n_nodes, flags, _stream(), ctypes.byref(h)))
    return Graph(h.value)


def slicegcn_slice_feature(X: torch.Tensor, start: int, end: int, Xs: torch.Tensor):
    px, ldx = _mat(X, "X")
    pxs, ldxs = _mat(Xs, "Xs")
    if Xs.shape[0] != X.shape[0]:
        raise ValueError("Xs has the wrong number of rows")
    _check(lib().slicegcn_slice_feature(px, X.shape[0], ldx, start, end, pxs, ldxs, _stream()))
    return Xs


def slicegcn_spmm_workspace_bytes(g: Graph, width: int, transpose: bool = False) -> int:
    return int(lib().slicegcn_spmm_workspace_bytes(g.handle, int(transpose), width))


def slicegcn_scale_rows(g: Graph, X: torch.Tensor, Xs: torch.Tensor, width: int | None = None):
    """Xs = D~^-1/2 X: the operand form ``slicegcn_spmm_slice(..., prescaled=True)`` expects."""
    px, ldx = _mat(X, "X")
    ps, lds = _mat(Xs, "Xs")
    w = int(X.shape[1] if width is None else width)
    _check(lib().slicegcn_scale_rows(g.handle, px, ldx, w, ps, lds, _stream()))
    return Xs


def slicegcn_spmm_slice(g: Graph, X: torch.Tensor, Y: torch.Tensor, width: int | None = None, transpose: bool = False,
                        ws: torch.Tensor | None = None, prescaled: bool = False):
    """``ws``: uint8 device tensor of slicegcn_spmm_workspace_bytes bytes; None = the graph object's cached buffer.
    ``prescaled``: X already holds D~^-1/2 X (see slicegcn_scale_rows)."""
    px, ldx = _mat(X, "X")
    py, ldy = _mat(Y, "Y")
    if X.shape[0] != Y.shape[0]:
        raise ValueError("X and Y differ in rows")
    w = int(X.shape[1] if width is None else width)
    if ws is None and w >= 1:
        ws = g.default_ws(slicegcn_spmm_workspace_bytes(g, w, transpose))
    pws, nws = _ws(ws)
    _check(lib().slicegcn_spmm_slice(g.handle, int(transpose) | (2 if prescaled else 0), px, ldx, w, py, ldy, pws, nws, _stream()))
    return Y


STATIC_WS_BYTES = 16 << 20


def slicegcn_spmm_slice_static(g: Graph, X: torch.Tensor, Y: torch.Tensor, width: int | None = None, transpose: bool = False,
                               prescaled: bool = False):
    """The aggregation with the library's built-in partial-sum buffer: no workspace, no allocation."""
    px, ldx = _mat(X, "X")
    py, ldy = _mat(Y, "Y")
    if X.shape[0] != Y.shape[0]:
        raise ValueError("X and Y differ in rows")
    w = int(X.shape[1] if width is None else width)
    _check(lib().slicegcn_spmm_slice_static(g.handle, int(transpose) | (2 if prescaled else 0), px, ldx, w, py, ldy, _stream()))
    return Y


def _layer_structs(w_in, w_out, act, W_agg, b, W_self, b_self, flags=0):
    desc = _LayerDesc(w_in, w_out, act, flags)
    for name, W in (("W_agg", W_agg), ("W_self", W_self)):
        if W is not None and (tuple(W.shape) != (w_in, w_out)):
            raise ValueError(f"{name} must be w_in x w_out")
    params = _LayerParams(_vec(W_agg, "W_agg"), _vec(b, "b"), _vec(W_self, "W_self"), _vec(b_self, "b_self"))
    return desc, params


def _saved_struct(Z, mask):
    pz, ldz = _mat(Z, "Z") if Z is not None else (None, 0)
    if mask is None:
        return _LayerSaved(pz, ldz, None, 0)
    pm, ldm = _mat(mask, "mask", torch.int32)
    return _LayerSaved(pz, ldz, pm, ldm)


def slicegcn_layer_fwd_workspace_bytes(g: Graph, w_in: int, w_out: int, flags: int = 0) -> int:
    desc = _LayerDesc(w_in, w_out, ACT_RELU, flags)
    return int(lib().slicegcn_layer_fwd_workspace_bytes(g.handle, ctypes.byref(desc)))


def slicegcn_layer_fwd(g: Graph, Hin, W_agg, b, W_self, b_self, Hout, Z, mask, act: int = ACT_RELU,
                       w_in: int | None = None, w_out: int | None = None, z_valid: bool = False,
                       ws: torch.Tensor | None = None, order: int = 0, layout: int = 0):
    """Hout = act(A^ Hin W_agg + b) + Hin W_self + b_self; fills Z (and mask for ReLU).
    ``z_valid``: Z already holds A^ Hin (same graph and Hin as an earlier call): skip the aggregation.
    ``ws``: uint8 device tensor of slicegcn_layer_fwd_workspace_bytes bytes; None = the graph object's cached buffer.
    ``order``: 0, LAYER_TRANSFORM_FIRST or LAYER_ORDER_AUTO (then Z may be None when the transform-first order runs).
    ``layout``: LAYER_IN_SCALED and/or LAYER_OUT_SCALED (activations kept as D~^-1/2 H)."""
    w_in = int(W_agg.shape[0] if w_in is None else w_in)
    w_out = int(W_agg.shape[1] if w_out is None else w_out)
    desc, params = _layer_structs(w_in, w_out, act, W_agg, b, W_self, b_self, (LAYER_Z_VALID if z_valid else 0) | order | layout)
    pi, ldi = _mat(Hin, "Hin")
    po, ldo = _mat(Hout, "Hout")
    saved = _saved_struct(Z, mask)
    if ws is None:
        ws = g.default_ws(int(lib().slicegcn_layer_fwd_workspace_bytes(g.handle, ctypes.byref(desc))))
    pws, nws = _ws(ws)
    _check(lib().slicegcn_layer_fwd(g.handle, ctypes.byref(desc), ctypes.byref(params), pi, ldi, po, ldo,
                                    ctypes.byref(saved), pws, nws, _stream()))
    return Hout


def slicegcn_layer_bwd_workspace_bytes(g: Graph, w_in: int, w_out: int, need_dHin: bool, flags: int = 0) -> int:
    desc = _LayerDesc(w_in, w_out, ACT_RELU, flags)
    return int(lib().slicegcn_layer_bwd_workspace_bytes(g.handle, ctypes.byref(desc), int(need_dHin)))


def slicegcn_layer_bwd(g: Graph, Hin, W_agg, W_self, Z, mask, dHout, dHin, dW_agg, db, dW_self, db_self, ws,
                       act: int = ACT_RELU, order: int = 0, layout: int = 0):
    """Gradients of one layer.  ``dHin`` may be None (skipped).  ``ws`` is a uint8 workspace tensor.
    ``order``, ``layout``: the flags the forward call was given."""
    w_in, w_out = int(W_agg.shape[0]), int(W_agg.shape[1])
    desc, params = _layer_structs(w_in, w_out, act, W_agg, None, W_self, None, order | layout)
    pi, ldi = _mat(Hin, "Hin")
    pg, ldo = _mat(dHout, "dHout")
    pgi, ldgi = _mat(dHin, "dHin") if dHin is not None else (None, 0)
    saved = _saved_struct(Z, mask)
    grads = _LayerGrads(_vec(dW_agg, "dW_agg"), _vec(db, "db"), _vec(dW_self, "dW_self"), _vec(db_self, "db_self"))
    _check(lib().slicegcn_layer_bwd(g.handle, ctypes.byref(desc), ctypes.byref(params), pi, ldi, ctypes.byref(saved),
                                    pg, ldo, pgi, ldgi, ctypes.byref(grads),
                                    ws.data_ptr() if ws is not None else None, ws.numel() * ws.element_size() if ws is not None else 0,
                                    _stream()))


def slicegcn_concat(Hs, E, H: torch.Tensor):
    """H[:, off_i : off_i + w_i] = Hs[i] + E[i, :w_i]  (E may be None)."""
    k = len(Hs)
    ptrs = (ctypes.c_void_p * k)()
    lds = (ctypes.c_int64 * k)()
    widths = (ctypes.c_int32 * k)()
    for i, h in enumerate(Hs):
        ptrs[i], lds[i] = _mat(h, f"Hs[{i}]")
        widths[i] = h.shape[1]
    pe, lde = _mat(E, "E") if E is not None else (None, 0)
    ph, ldh = _mat(H, "H")
    _check(lib().slicegcn_concat(k, ctypes.addressof(ptrs), ctypes.addressof(lds), ctypes.addressof(widths), pe, lde,
                                 H.shape[0], ph, ldh, _stream()))
    return H


def slicegcn_concat_bwd_workspace_bytes(n: int, widths) -> int:
    k = len(widths)
    w = (ctypes.c_int32 * k)(*[int(x) for x in widths])
    return int(lib().slicegcn_concat_bwd_workspace_bytes(n, k, ctypes.addressof(w)))


def slicegcn_concat_bwd(dH: torch.Tensor, widths, dHs=None, dE=None, ws=None):
    """dE[i, :w_i] = column sums of dH's block i; optional copies of the blocks into dHs[i]."""
    k = len(widths)
    w = (ctypes.c_int32 * k)(*[int(x) for x in widths])
    pdh, ldh = _mat(dH, "dH")
    ptrs = lds = None
    if dHs is not None:
        ptrs = (ctypes.c_void_p * k)()
        lds = (ctypes.c_int64 * k)()
        for i, t in enumerate(dHs):
            if t is not None:
                ptrs[i], lds[i] = _mat(t, f"dHs[{i}]")
    pe, lde = _mat(dE, "dE") if dE is not None else (None, 0)
    _check(lib().slicegcn_concat_bwd(k, pdh, ldh, dH.shape[0], ctypes.addressof(w),
                                     ctypes.addressof(ptrs) if ptrs is not None else None,
                                     ctypes.addressof(lds) if lds is not None else None, pe, lde,
                                     ws.data_ptr() if ws is not None else None,
                                     ws.numel() * ws.element_size() if ws is not None else 0, _stream()))


def slicegcn_linear_fwd(X, W, b, Y, mask=None, act: int = ACT_NONE):
    """Y = act(X W + b); fills mask (n x ceil(w_out/32) int32) for ReLU."""
    w_in, w_out = int(W.shape[0]), int(W.shape[1])
    px, ldx = _mat(X, "X")
    py, ldy = _mat(Y, "Y")
    if X.shape[1] != w_in or Y.shape[1] != w_out or X.shape[0] != Y.shape[0]:
        raise ValueError("X, W, Y shapes do not match")
    pm, ldm = _mat(mask, "mask", torch.int32) if mask is not None else (None, 0)
    _check(lib().slicegcn_linear_fwd(px, ldx, X.shape[0], w_in, w_out, _vec(W, "W"), _vec(b, "b"), act, py, ldy, pm, ldm,
                                     _stream()))
    return Y


def slicegcn_linear_bwd_workspace_bytes(n: int, w_in: int, w_out: int) -> int:
    return int(lib().slicegcn_linear_bwd_workspace_bytes(n, w_in, w_out))


def slicegcn_linear_bwd(X, W, mask, dY, dX, dW, db, ws, act: int = ACT_NONE):
    """dX = (dY * mask) W^T, dW = X^T (dY * mask), db = colsum(dY * mask); None outputs are skipped."""
    w_in, w_out = int(W.shape[0]), int(W.shape[1])
    px, ldx = _mat(X, "X")
    pg, ldg = _mat(dY, "dY")
    pdx, lddx = _mat(dX, "dX") if dX is not None else (None, 0)
    pm, ldm = _mat(mask, "mask", torch.int32) if mask is not None else (None, 0)
    if dW is not None and tuple(dW.shape) != (w_in, w_out):
        raise ValueError("dW must be w_in x w_out")
    pws, nws = _ws(ws)
    _check(lib().slicegcn_linear_bwd(px, ldx, X.shape[0], w_in, w_out, _vec(W, "W"), act, pm, ldm, pg, ldg, pdx, lddx,
                                     _vec(dW, "dW"), _vec(db, "db"), pws, nws, _stream()))


def slicegcn_accumulate(dst, src):
    """dst += src (same shape; leading dimensions may differ)."""
    pd, ldd = _mat(dst, "dst")
    ps, lds = _mat(src, "src")
    if dst.shape != src.shape:
        raise ValueError("dst and src differ in shape")
    _check(lib().slicegcn_accumulate(pd, ldd, ps, lds, dst.shape[0], dst.shape[1], _stream()))
    return dst


def slicegcn_adam_step(param, grad, m, v, lr: float, step: int, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0):
    """One Adam step in place on flat (contiguous) fp32 device tensors of equal size."""
    n = param.numel()
    for t, name in ((grad, "grad"), (m, "m"), (v, "v")):
        if t.numel() != n:
            raise ValueError(f"{name} differs in size from param")
    _check(lib().slicegcn_adam_step(_vec(param, "param"), _vec(grad, "grad"), _vec(m, "m"), _vec(v, "v"), n, lr, beta1, beta2,
                                    eps, weight_decay, step, _stream()))


def slicegcn_cosine_lr(lr_max: float, lr_min: float, t: int, t_max: int) -> float:
    return float(lib().slicegcn_cosine_lr(lr_max, lr_min, t, t_max))


def slicegcn_softmax_ce_workspace_bytes(n: int) -> int:
    return int(lib().slicegcn_softmax_ce_workspace_bytes(n))


def slicegcn_softmax_ce(logits, labels, loss, dlogits, ws):
    """loss[0] = mean softmax cross-entropy over the rows; dlogits (or None) its gradient."""
    pl, ld = _mat(logits, "logits")
    pd, ldd = _mat(dlogits, "dlogits") if dlogits is not None else (None, 0)
    if labels.shape != (logits.shape[0],):
        raise ValueError("one label per row expected")
    pws, nws = _ws(ws)
    _check(lib().slicegcn_softmax_ce(pl, ld, logits.shape[0], logits.shape[1], _vec(labels, "labels", torch.int32),
                                     _vec(loss, "loss"), pd, ldd, pws, nws, _stream()))
    return loss


def slicegcn_profile_reserve(scopes: int):
    """Create the events of ``scopes`` kernel groups ahead of a profiled region."""
    _check(lib().slicegcn_profile_reserve(int(scopes)))


def slicegcn_profile_begin():
    _check(lib().slicegcn_profile_begin())


def slicegcn_profile_end(capacity: int = 64, with_range: bool = False):
    """[(kind name, width, launches, total_ms)] of the kernels launched since profile_begin;
    with_range appends (min_ms, max_ms, median_ms) of a single launch group."""
    arr = (_ProfileEntry * capacity)()
    count = ctypes.c_int32(0)
    _check(lib().slicegcn_profile_end(arr, capacity, ctypes.byref(count)))
    return [(PROF_KINDS.get(e.kind, str(e.kind)), int(e.width), int(e.launches), float(e.total_ms))
            + ((float(e.min_ms), float(e.max_ms), float(e.median_ms)) if with_range else ())
            for e in arr[:min(count.value, capacity)]]

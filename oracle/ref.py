"""ctypes access to the CPU oracle (`mggcn_ref.c`).

TEST INFRASTRUCTURE ONLY: imported by tests, by the smoke check and by the bench's
cpu_baseline leg.  It shares nothing with the HIP library and the product package never
imports it.  All arrays are host numpy arrays; dense data is float64.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libmggcn_ref.so")
_lib = None

NORM_SYM, NORM_MEAN_IN = 0, 1
OP_N, OP_T = 0, 1
GEMM_FIRST, SPMM_FIRST = 0, 1


def build(force: bool = True) -> str:
    src = os.path.join(_HERE, "mggcn_ref.c")
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(src):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _SO, src, "-lm"]
        )
    return _SO


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_SO):
            build(force=False)
        lib = C.CDLL(_SO)
        vp, i32, i64, dbl = C.c_void_p, C.c_int, C.c_int64, C.c_double
        lib.mggcn_ref_csr_validate.restype = i32
        lib.mggcn_ref_csr_validate.argtypes = [i32, i32, vp, vp]
        lib.mggcn_ref_csr_normalize.restype = i64
        lib.mggcn_ref_csr_normalize.argtypes = [i32, i32, vp, vp, i32, vp, vp, vp, vp, vp]
        lib.mggcn_ref_csr_transpose.restype = i32
        lib.mggcn_ref_csr_transpose.argtypes = [i32, i32, vp, vp, vp, vp, vp, vp]
        lib.mggcn_ref_spmm.restype = i32
        lib.mggcn_ref_spmm.argtypes = [i32, i32, i32, vp, vp, vp, vp, i64, i32, dbl, vp, i64]
        lib.mggcn_ref_gemm.restype = i32
        lib.mggcn_ref_gemm.argtypes = [i32, i32, i32, i32, i32, vp, i64, vp, i64, dbl, vp, i64]
        lib.mggcn_ref_relu.restype = None
        lib.mggcn_ref_relu.argtypes = [i64, i32, vp, i64]
        lib.mggcn_ref_relu_bwd.restype = None
        lib.mggcn_ref_relu_bwd.argtypes = [i64, i32, vp, i64, vp, i64]
        lib.mggcn_ref_softmax_ce.restype = i32
        lib.mggcn_ref_softmax_ce.argtypes = [i64, i32, vp, i64, vp, vp, vp, i64]
        lib.mggcn_ref_order.restype = i32
        lib.mggcn_ref_order.argtypes = [i32, i32]
        lib.mggcn_ref_layer_fwd.restype = i32
        lib.mggcn_ref_layer_fwd.argtypes = [i32, vp, vp, vp, i32, i32, i32, i32, vp, i64, vp, i64, vp, i64]
        lib.mggcn_ref_layer_bwd.restype = i32
        lib.mggcn_ref_layer_bwd.argtypes = [
            i32, vp, vp, vp, i32, i32, i32, i32, vp, i64, vp, i64, vp, i64, vp, i64, vp, i64, vp, i64,
        ]
        lib.mggcn_ref_epoch.restype = i32
        lib.mggcn_ref_epoch.argtypes = [i32, vp, vp, vp, i32, vp, vp, vp, i64, vp, vp, vp, vp, vp, vp]
        lib.mggcn_ref_epoch_bf16.restype = i32
        lib.mggcn_ref_epoch_bf16.argtypes = [i32, vp, vp, vp, i32, vp, vp, vp, i64, vp, vp, vp, vp, vp, vp,
                                             vp, vp, vp, vp]
        lib.mggcn_ref_bf16_round.restype = None
        lib.mggcn_ref_bf16_round.argtypes = [i64, vp, vp, vp]
        lib.mggcn_ref_adam_step.restype = i32
        lib.mggcn_ref_adam_step.argtypes = [i64, vp, vp, vp, vp, i32, dbl, dbl, dbl, dbl]
        _lib = lib
    return _lib


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _check(rc, what):
    if rc != 0:
        raise RuntimeError(f"oracle {what} failed with code {rc}")


def _ld(a: np.ndarray) -> int:
    """leading dimension of a 2-D row-major (possibly column-sliced) array"""
    assert a.ndim == 2 and (a.shape[1] <= 1 or a.strides[1] == a.itemsize), "need unit column stride"
    if a.shape[0] <= 1:
        return max(a.shape[1], 1)
    return max(a.strides[0] // a.itemsize, a.shape[1], 1)


def csr_validate(n_rows, n_cols, rowptr, colidx) -> int:
    rowptr, colidx = _i32(rowptr), _i32(colidx)
    return _load().mggcn_ref_csr_validate(n_rows, n_cols, rowptr.ctypes.data, colidx.ctypes.data)


def csr_normalize(n_rows, n_cols, rowptr, colidx, mode=NORM_SYM, deg_row=None, deg_col=None):
    """-> (rowptr', colidx', val' float64) of the normalised adjacency with self-loops."""
    rowptr, colidx = _i32(rowptr), _i32(colidx)
    cap = int(rowptr[-1]) + min(n_rows, n_cols)
    rp = np.empty(n_rows + 1, dtype=np.int32)
    ci = np.empty(cap, dtype=np.int32)
    va = np.empty(cap, dtype=np.float64)
    dr = None if deg_row is None else _f64(deg_row)
    dc = None if deg_col is None else _f64(deg_col)
    nnz = _load().mggcn_ref_csr_normalize(
        n_rows, n_cols, rowptr.ctypes.data, colidx.ctypes.data, mode,
        None if dr is None else dr.ctypes.data, None if dc is None else dc.ctypes.data,
        rp.ctypes.data, ci.ctypes.data, va.ctypes.data,
    )
    if nnz < 0:
        raise RuntimeError(f"oracle csr_normalize failed with code {nnz}")
    return rp, ci[:nnz].copy(), va[:nnz].copy()


def csr_transpose(n_rows, n_cols, rowptr, colidx, val):
    rowptr, colidx, val = _i32(rowptr), _i32(colidx), _f64(val)
    nnz = int(rowptr[-1])
    rpt = np.empty(n_cols + 1, dtype=np.int32)
    cit = np.empty(nnz, dtype=np.int32)
    vat = np.empty(nnz, dtype=np.float64)
    _check(
        _load().mggcn_ref_csr_transpose(
            n_rows, n_cols, rowptr.ctypes.data, colidx.ctypes.data, val.ctypes.data,
            rpt.ctypes.data, cit.ctypes.data, vat.ctypes.data,
        ),
        "csr_transpose",
    )
    return rpt, cit, vat


def spmm(op, n_rows, n_cols, rowptr, colidx, val, X, beta=0.0, Y=None, F=None):
    """Y = op(A) X + beta Y.  X may be a column slice view (its ld is honoured)."""
    rowptr, colidx, val = _i32(rowptr), _i32(colidx), _f64(val)
    if X.dtype != np.float64:
        X = X.astype(np.float64)
    F = X.shape[1] if F is None else F
    out_rows = n_rows if op == OP_N else n_cols
    if Y is None:
        Y = np.zeros((out_rows, F), dtype=np.float64)
    _check(
        _load().mggcn_ref_spmm(
            op, n_rows, n_cols, rowptr.ctypes.data, colidx.ctypes.data, val.ctypes.data,
            X.ctypes.data, _ld(X), F, float(beta), Y.ctypes.data, _ld(Y),
        ),
        "spmm",
    )
    return Y


def gemm(opA, opB, A, B, beta=0.0, Cmat=None):
    A, B = _f64(A), _f64(B)
    M = A.shape[0] if opA == OP_N else A.shape[1]
    K = A.shape[1] if opA == OP_N else A.shape[0]
    N = B.shape[1] if opB == OP_N else B.shape[0]
    assert (B.shape[0] if opB == OP_N else B.shape[1]) == K
    if Cmat is None:
        Cmat = np.zeros((M, N), dtype=np.float64)
    _check(
        _load().mggcn_ref_gemm(
            opA, opB, M, N, K, A.ctypes.data, _ld(A), B.ctypes.data, _ld(B), float(beta),
            Cmat.ctypes.data, _ld(Cmat),
        ),
        "gemm",
    )
    return Cmat


def relu(Z):
    Z = _f64(Z).copy()
    _load().mggcn_ref_relu(Z.shape[0], Z.shape[1], Z.ctypes.data, _ld(Z))
    return Z


def relu_bwd(act, G):
    act, G = _f64(act), _f64(G).copy()
    _load().mggcn_ref_relu_bwd(G.shape[0], G.shape[1], act.ctypes.data, _ld(act), G.ctypes.data, _ld(G))
    return G


def softmax_ce(Z, labels):
    """-> (mean loss, dZ)"""
    Z, labels = _f64(Z), _i32(labels)
    dZ = np.empty_like(Z)
    loss = C.c_double(0.0)
    _check(
        _load().mggcn_ref_softmax_ce(
            Z.shape[0], Z.shape[1], Z.ctypes.data, _ld(Z), labels.ctypes.data, C.byref(loss),
            dZ.ctypes.data, _ld(dZ),
        ),
        "softmax_ce",
    )
    return loss.value, dZ


def order(d_in, d_out) -> int:
    return _load().mggcn_ref_order(d_in, d_out)


def layer_fwd(n, rowptr, colidx, val, H_in, W, order_, relu_):
    rowptr, colidx, val, H_in, W = _i32(rowptr), _i32(colidx), _f64(val), _f64(H_in), _f64(W)
    d_in, d_out = W.shape
    out = np.zeros((n, d_out), dtype=np.float64)
    _check(
        _load().mggcn_ref_layer_fwd(
            n, rowptr.ctypes.data, colidx.ctypes.data, val.ctypes.data, d_in, d_out, order_,
            int(relu_), H_in.ctypes.data, _ld(H_in), W.ctypes.data, _ld(W), out.ctypes.data, _ld(out),
        ),
        "layer_fwd",
    )
    return out


def layer_bwd(n, rowptr, colidx, val, H_in, H_out, G, W, order_, relu_, need_input_grad=True):
    """-> (W_G, H_G or None, Z_G)"""
    rowptr, colidx, val = _i32(rowptr), _i32(colidx), _f64(val)
    H_in, H_out, G, W = _f64(H_in), _f64(H_out), _f64(G).copy(), _f64(W)
    d_in, d_out = W.shape
    W_G = np.zeros((d_in, d_out), dtype=np.float64)
    H_G = np.zeros((n, d_in), dtype=np.float64) if need_input_grad else None
    _check(
        _load().mggcn_ref_layer_bwd(
            n, rowptr.ctypes.data, colidx.ctypes.data, val.ctypes.data, d_in, d_out, order_,
            int(relu_), H_in.ctypes.data, _ld(H_in), H_out.ctypes.data, _ld(H_out), G.ctypes.data,
            _ld(G), W.ctypes.data, _ld(W), W_G.ctypes.data, _ld(W_G),
            None if H_G is None else H_G.ctypes.data, d_in,
        ),
        "layer_bwd",
    )
    return W_G, H_G, G


def epoch(n, rowptr, colidx, val, X, labels, Ws, orders=None, want_logits=False, relu_masks=None):
    """-> (loss, [W_G...], logits or None).  relu_masks: optional list of L-1 (n, d_{l+1}) 0/1 byte
    arrays with the hidden layers' ReLU' decisions to use in the backward pass."""
    rowptr, colidx, val, X, labels = _i32(rowptr), _i32(colidx), _f64(val), _f64(X), _i32(labels)
    Ws = [_f64(w) for w in Ws]
    L = len(Ws)
    dims = np.array([Ws[0].shape[0]] + [w.shape[1] for w in Ws], dtype=np.int32)
    for l, w in enumerate(Ws):
        assert w.shape == (dims[l], dims[l + 1])
    WG = [np.zeros_like(w) for w in Ws]
    Wp = (C.c_void_p * L)(*[w.ctypes.data for w in Ws])
    WGp = (C.c_void_p * L)(*[w.ctypes.data for w in WG])
    ords = None if orders is None else _i32(orders)
    logits = np.zeros((n, int(dims[-1])), dtype=np.float64) if want_logits else None
    loss = C.c_double(0.0)
    Mp = None
    if relu_masks is not None:
        assert len(relu_masks) == L - 1
        relu_masks = [np.ascontiguousarray(m, dtype=np.uint8) for m in relu_masks]
        for l, m in enumerate(relu_masks):
            assert m.shape == (n, int(dims[l + 1]))
        Mp = (C.c_void_p * max(L - 1, 1))(*[m.ctypes.data for m in relu_masks])
    _check(
        _load().mggcn_ref_epoch(
            n, rowptr.ctypes.data, colidx.ctypes.data, val.ctypes.data, L, dims.ctypes.data,
            None if ords is None else ords.ctypes.data, X.ctypes.data, _ld(X), labels.ctypes.data,
            Wp, C.byref(loss), WGp, None if logits is None else logits.ctypes.data, Mp,
        ),
        "epoch",
    )
    return loss.value, WG, logits


def bf16_round(x):
    """float32 array -> (bfloat16 codes as uint16, the rounded values as float32), same shape."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    codes = np.empty(x.shape, dtype=np.uint16)
    values = np.empty(x.shape, dtype=np.float32)
    _load().mggcn_ref_bf16_round(x.size, x.ctypes.data, codes.ctypes.data, values.ctypes.data)
    return codes, values


def gather_widths(dims, orders):
    """Per layer: (width of the forward SpMM's operand, width of the backward SpMM's operand or 0)."""
    out = []
    for l in range(len(dims) - 1):
        o = orders[l] if orders is not None else order(int(dims[l]), int(dims[l + 1]))
        if o == GEMM_FIRST:
            out.append((int(dims[l + 1]), int(dims[l + 1])))
        else:
            out.append((int(dims[l]), int(dims[l]) if l > 0 else 0))
    return out


def epoch_bf16(n, rowptr, colidx, val, X, labels, Ws, orders=None, relu_masks=None, fwd_codes=None,
               bwd_codes=None):
    """The epoch with every SpMM gathering a bfloat16 copy of its operand.
    fwd_codes / bwd_codes: optional lists of L entries (None or (n, width) uint16 arrays) used as the
    operands instead of the oracle's own roundings.
    -> (loss, [W_G...], own_fwd_codes, own_bwd_codes)  (own_*[l] is None where layer l has no such SpMM)"""
    rowptr, colidx, val, X, labels = _i32(rowptr), _i32(colidx), _f64(val), _f64(X), _i32(labels)
    Ws = [_f64(w) for w in Ws]
    L = len(Ws)
    dims = np.array([Ws[0].shape[0]] + [w.shape[1] for w in Ws], dtype=np.int32)
    WG = [np.zeros_like(w) for w in Ws]
    Wp = (C.c_void_p * L)(*[w.ctypes.data for w in Ws])
    WGp = (C.c_void_p * L)(*[w.ctypes.data for w in WG])
    ords = None if orders is None else _i32(orders)
    loss = C.c_double(0.0)
    Mp = None
    if relu_masks is not None:
        assert len(relu_masks) == L - 1
        relu_masks = [np.ascontiguousarray(m, dtype=np.uint8) for m in relu_masks]
        Mp = (C.c_void_p * max(L - 1, 1))(*[m.ctypes.data for m in relu_masks])
    widths = gather_widths(dims, None if orders is None else list(orders))

    def ptrs(given, which):
        if given is None:
            return None, None
        keep = []
        for l in range(L):
            a = given[l]
            if a is not None:
                a = np.ascontiguousarray(a, dtype=np.uint16)
                assert a.shape == (n, widths[l][which]), (a.shape, widths[l])
            keep.append(a)
        return (C.c_void_p * L)(*[None if a is None else a.ctypes.data for a in keep]), keep

    fin, _k1 = ptrs(fwd_codes, 0)
    bin_, _k2 = ptrs(bwd_codes, 1)
    own_f = [np.zeros((n, w[0]), dtype=np.uint16) for w in widths]
    own_b = [np.zeros((n, w[1]), dtype=np.uint16) if w[1] else None for w in widths]
    fout = (C.c_void_p * L)(*[a.ctypes.data for a in own_f])
    bout = (C.c_void_p * L)(*[None if a is None else a.ctypes.data for a in own_b])
    _check(
        _load().mggcn_ref_epoch_bf16(
            n, rowptr.ctypes.data, colidx.ctypes.data, val.ctypes.data, L, dims.ctypes.data,
            None if ords is None else ords.ctypes.data, X.ctypes.data, _ld(X), labels.ctypes.data,
            Wp, C.byref(loss), WGp, None, Mp, fin, bin_, fout, bout,
        ),
        "epoch_bf16",
    )
    return loss.value, WG, own_f, own_b


def adam_step(W, G, m, v, t, lr=1e-3, b1=0.9, b2=0.999, eps=1e-8):
    """In-place Adam update of float64 arrays W, m, v (all contiguous, same size as G)."""
    for a in (W, m, v):
        assert a.dtype == np.float64 and a.flags.c_contiguous
    G = _f64(G)
    _check(_load().mggcn_ref_adam_step(W.size, W.ctypes.data, G.ctypes.data, m.ctypes.data, v.ctypes.data,
                                        int(t), lr, b1, b2, eps), "adam_step")
    return W, m, v

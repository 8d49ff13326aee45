"""MI355X-native hot path of full-batch GCN training (MG-GCN, arXiv 2110.08688).

Python face of the C-ABI library `libmggcn.so` (see include/mggcn.h).  The functions here carry
the same names as the C entry points and only marshal arguments: PyTorch supplies device memory
(tensors) and the current HIP stream, every step of the computation runs in the library's own
kernels.  Nothing here falls back to PyTorch or CPU arithmetic.
"""
from __future__ import annotations

import ctypes as C

from . import binding as B
from .binding import (  # noqa: F401  (re-exported constants)
    EPI_NONE, EPI_RELU, EPI_RELU_MASK, NORM_MEAN_IN, NORM_SYM_SELFLOOP, OP_N, OP_T, ORDER_AUTO,
    ORDER_GEMM_FIRST, ORDER_SPMM_FIRST, MODEL_CACHE_INPUT, MODEL_GATHER_BF16, MODEL_GEMM_BF16X3, MggcnError,
)


def _torch():
    import torch

    return torch


def _ws(nbytes: int, device):
    torch = _torch()
    return torch.empty(max(int(nbytes), 256) + 256, dtype=torch.uint8, device=device)


def _ws_ptr(t):
    """256-byte aligned address inside a workspace tensor"""
    p = t.data_ptr()
    return (p + 255) // 256 * 256


def _stream(stream):
    return B.current_stream() if stream is None else stream


def _sync(stream):
    """Wait for the work enqueued on the stream a call used, before its workspace tensor is dropped
    (PyTorch's allocator would hand the memory to someone else while kernels still use it)."""
    torch = _torch()
    if stream is None:
        torch.cuda.current_stream().synchronize()
    else:
        torch.cuda.ExternalStream(int(stream)).synchronize()


def mggcn_version() -> int:
    return B.lib().mggcn_version()


# ------------------------------------------------------------------------------------------
# setup: normalised adjacency, transpose
# ------------------------------------------------------------------------------------------

def mggcn_csr_normalize(n_rows, n_cols, rowptr_in, colidx_in, mode=NORM_SYM_SELFLOOP, deg_row=None,
                        deg_col=None, validate=False, stream=None):
    """-> (rowptr, colidx, val) device tensors of the normalised adjacency with self-loops.
    An int64 rowptr_in selects the 64-bit entry points (rowptr comes back as int64)."""
    torch = _torch()
    L = B.lib()
    dev = rowptr_in.device
    st = _stream(stream)
    wide = rowptr_in.dtype == torch.int64
    count_fn = L.mggcn_csr_normalize_count64 if wide else L.mggcn_csr_normalize_count
    fill_fn = L.mggcn_csr_normalize64 if wide else L.mggcn_csr_normalize
    nbytes = L.mggcn_csr_normalize_workspace_bytes(n_rows, n_cols)
    ws = _ws(nbytes, dev)
    rowptr = torch.empty(n_rows + 1, dtype=rowptr_in.dtype, device=dev)
    nnz = C.c_int64(0)
    B.check(count_fn(n_rows, n_cols, B.ptr(rowptr_in), B.ptr(colidx_in), int(validate),
                                        B.ptr(rowptr), C.byref(nnz), _ws_ptr(ws), nbytes, st))
    colidx = torch.empty(nnz.value, dtype=torch.int32, device=dev)
    val = torch.empty(nnz.value, dtype=torch.float32, device=dev)
    B.check(fill_fn(n_rows, n_cols, B.ptr(rowptr_in), B.ptr(colidx_in), mode, B.ptr(deg_row),
                                  B.ptr(deg_col), B.ptr(rowptr), B.ptr(colidx), B.ptr(val), _ws_ptr(ws),
                                  nbytes, st))
    _sync(stream)  # ws may be freed now
    return rowptr, colidx, val


def mggcn_csr_transpose(n_rows, n_cols, rowptr, colidx, val, stream=None):
    """-> (rowptr_t, colidx_t, val_t); an int64 rowptr selects the 64-bit entry point"""
    torch = _torch()
    L = B.lib()
    dev = rowptr.device
    nnz = int(colidx.numel())
    nbytes = L.mggcn_csr_transpose_workspace_bytes(n_rows, n_cols, nnz)
    ws = _ws(nbytes, dev)
    rowptr_t = torch.empty(n_cols + 1, dtype=rowptr.dtype, device=dev)
    colidx_t = torch.empty(nnz, dtype=torch.int32, device=dev)
    val_t = torch.empty(nnz, dtype=torch.float32, device=dev)
    fn = L.mggcn_csr_transpose64 if rowptr.dtype == torch.int64 else L.mggcn_csr_transpose
    B.check(fn(n_rows, n_cols, nnz, B.ptr(rowptr), B.ptr(colidx), B.ptr(val), B.ptr(rowptr_t),
                                  B.ptr(colidx_t), B.ptr(val_t), _ws_ptr(ws), nbytes, _stream(stream)))
    _sync(stream)
    return rowptr_t, colidx_t, val_t


# ------------------------------------------------------------------------------------------
# graph handle + SpMM
# ------------------------------------------------------------------------------------------

class Graph:
    """Owns an mggcn_graph handle, keeps the CSR tensors and the bound workspace alive."""

    def __init__(self, n_rows, n_cols, rowptr, colidx, val, transpose=None, F_max=256, seg_len=0, n_panels=0,
                 panel_mib=0, chunk_lanes=0, stream=None):
        L = B.lib()
        self.n_rows, self.n_cols = n_rows, n_cols
        self._keep = [rowptr, colidx, val, transpose]
        rpt, cit, vat = transpose if transpose is not None else (None, None, None)
        h = C.c_void_p(None)
        wide = str(rowptr.dtype).endswith("int64")  # 64-bit row offsets: matrices of 2^31 entries and more
        create = L.mggcn_graph_create64 if wide else L.mggcn_graph_create
        B.check(create(n_rows, n_cols, B.ptr(rowptr), B.ptr(colidx), B.ptr(val), B.ptr(rpt),
                                     B.ptr(cit), B.ptr(vat), seg_len, n_panels, _stream(stream), C.byref(h)))
        self.handle = h
        self.device = rowptr.device
        self.ws = None
        self.F_max = 0
        if panel_mib or chunk_lanes:
            self.tune(panel_mib, chunk_lanes)
        self.bind(F_max, stream)

    def bind(self, F_max, stream=None):
        L = B.lib()
        nbytes = L.mggcn_graph_workspace_bytes(self.handle, F_max)
        ws = _ws(nbytes, self.device)
        B.check(L.mggcn_graph_bind(self.handle, F_max, _ws_ptr(ws), nbytes, _stream(stream)))
        self.ws, self.F_max = ws, F_max

    def tune(self, panel_mib=0, chunk_lanes=0):
        B.check(B.lib().mggcn_graph_tune(self.handle, int(panel_mib), int(chunk_lanes)))

    def tables(self, op=OP_N, form=0):
        """Segment tables of the handle as host arrays (tests): dict with n_panels, tasks (n x 4 int32 view of the
        records: row, first entry, length | flags, slot), task_begin, fix (n x 4 int32), fix_begin, n_slots, n_forms."""
        torch = _torch()
        n_panels, n_tasks, n_fix, n_slots = C.c_int32(0), C.c_int64(0), C.c_int64(0), C.c_int64(0)
        tp, fp = C.c_void_p(None), C.c_void_p(None)
        tb, fb = (C.c_int64 * 65)(), (C.c_int64 * 65)()
        n_forms = B.check(B.lib().mggcn_graph_tables(self.handle, op, form, C.byref(n_panels), C.byref(n_tasks), C.byref(tp), tb,
                                                     C.byref(n_fix), C.byref(fp), fb, C.byref(n_slots)))
        torch.cuda.synchronize()

        def grab(ptr, n):
            if n == 0:
                return torch.zeros((0, 4), dtype=torch.int32)
            base = _ws_ptr(self.ws)
            off = (ptr - base) // 4
            flat = self.ws[(base - self.ws.data_ptr()):].view(torch.int32)
            return flat[off: off + 4 * n].view(n, 4).cpu()

        P = n_panels.value
        return dict(n_panels=P, tasks=grab(tp.value, n_tasks.value), task_begin=list(tb[: P + 1]),
                    fix=grab(fp.value, n_fix.value), fix_begin=list(fb[: P + 1]), n_slots=n_slots.value, n_forms=n_forms)

    def panels(self, F, op=OP_N) -> int:
        return B.check(B.lib().mggcn_graph_panels(self.handle, op, F))

    def close(self):
        if getattr(self, "handle", None):
            B.lib().mggcn_graph_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def mggcn_spmm(graph: Graph, op, X, F=None, beta=0.0, epilogue=EPI_NONE, Y=None, stream=None):
    """Y = epilogue(op(A^) X + beta Y); returns Y (allocated if not given)."""
    torch = _torch()
    F = int(X.shape[1]) if F is None else F
    out_rows = graph.n_rows if op == OP_N else graph.n_cols
    if Y is None:
        Y = torch.empty((out_rows, F), dtype=torch.float32, device=X.device)
    B.check(B.lib().mggcn_spmm(graph.handle, op, B.ptr(X), B.ld_of(X), F, float(beta), epilogue, B.ptr(Y),
                               B.ld_of(Y), _stream(stream)))
    return Y


def mggcn_f32_to_bf16(src, dst=None, stream=None):
    """bfloat16 copy (round to nearest even) of a 2-D fp32 tensor, as an int16 tensor of bit patterns."""
    torch = _torch()
    rows, cols = src.shape
    if dst is None:
        ld = (cols + 15) // 16 * 16
        dst = torch.empty((rows, ld), dtype=torch.int16, device=src.device)[:, :cols]
    B.check(B.lib().mggcn_f32_to_bf16(rows, cols, B.ptr(src), B.ld_of(src), B.ptr(dst), B.ld_of(dst),
                                      _stream(stream)))
    return dst


def mggcn_spmm_bf16(graph: Graph, op, Xb, F=None, beta=0.0, epilogue=EPI_NONE, Y=None, stream=None):
    """Y = epilogue(op(A^) X + beta Y) with X given as bfloat16 bit patterns (int16 tensor); Y is fp32."""
    torch = _torch()
    assert Xb.element_size() == 2
    F = int(Xb.shape[1]) if F is None else F
    out_rows = graph.n_rows if op == OP_N else graph.n_cols
    if Y is None:
        Y = torch.empty((out_rows, F), dtype=torch.float32, device=Xb.device)
    B.check(B.lib().mggcn_spmm_bf16(graph.handle, op, B.ptr(Xb), B.ld_of(Xb), F, float(beta), epilogue, B.ptr(Y),
                                    B.ld_of(Y), _stream(stream)))
    return Y


# ------------------------------------------------------------------------------------------
# GeMM, ReLU', loss
# ------------------------------------------------------------------------------------------

def gemm_workspace(opA, opB, M, N, K, device):
    """A workspace tensor for repeated mggcn_gemm calls of one shape (None if the shape needs none)."""
    nbytes = B.lib().mggcn_gemm_workspace_bytes(opA, opB, M, N, K)
    return _ws(nbytes, device) if nbytes else None


def mggcn_gemm(opA, opB, A, Bm, beta=0.0, epilogue=EPI_NONE, Cm=None, stream=None, entry="mggcn_gemm", ws=None):
    """ws: a tensor from gemm_workspace() that the caller keeps alive; without it a workspace is allocated for
    this call and the stream is drained before it is dropped."""
    torch = _torch()
    L = B.lib()
    M = A.shape[0] if opA == OP_N else A.shape[1]
    K = A.shape[1] if opA == OP_N else A.shape[0]
    N = Bm.shape[1] if opB == OP_N else Bm.shape[0]
    if Cm is None:
        Cm = torch.empty((M, N), dtype=torch.float32, device=A.device)
    nbytes = L.mggcn_gemm_workspace_bytes(opA, opB, M, N, K)
    own = ws is None and nbytes > 0
    if own:
        ws = _ws(nbytes, A.device)
    ws_bytes = 0 if ws is None else ws.numel() - (_ws_ptr(ws) - ws.data_ptr())
    B.check(getattr(L, entry)(opA, opB, M, N, K, B.ptr(A), B.ld_of(A), B.ptr(Bm), B.ld_of(Bm), float(beta), epilogue,
                              B.ptr(Cm), B.ld_of(Cm), _ws_ptr(ws) if ws is not None else None, ws_bytes,
                              _stream(stream)))
    if own:
        _sync(stream)
    return Cm


def mggcn_gemm_bf16x3(opA, opB, A, Bm, beta=0.0, epilogue=EPI_NONE, Cm=None, stream=None, ws=None):
    """The same product on the bfloat16 matrix instructions (three exact pieces per operand)."""
    return mggcn_gemm(opA, opB, A, Bm, beta=beta, epilogue=epilogue, Cm=Cm, stream=stream, entry="mggcn_gemm_bf16x3", ws=ws)


def mggcn_relu_bwd(act, G, stream=None):
    B.check(B.lib().mggcn_relu_bwd(G.shape[0], G.shape[1], B.ptr(act), B.ld_of(act), B.ptr(G), B.ld_of(G),
                                   _stream(stream)))
    return G


def mggcn_softmax_ce(logits, labels, dlogits=None, stream=None):
    """-> (loss: 1-element device tensor, dlogits).  dlogits=None writes the gradient in place."""
    torch = _torch()
    L = B.lib()
    n, Cn = logits.shape
    if dlogits is None:
        dlogits = logits
    nbytes = L.mggcn_softmax_ce_workspace_bytes(n)
    ws = _ws(nbytes, logits.device)
    loss = torch.empty(1, dtype=torch.float32, device=logits.device)
    B.check(L.mggcn_softmax_ce(n, Cn, B.ptr(logits), B.ld_of(logits), B.ptr(labels), B.ptr(loss), B.ptr(dlogits),
                               B.ld_of(dlogits), _ws_ptr(ws), nbytes, _stream(stream)))
    _sync(stream)
    return loss, dlogits


def mggcn_softmax_ce_static(logits, labels, loss, dlogits=None, stream=None):
    """mggcn_softmax_ce without any allocation: the caller passes every buffer (loss: 1-element fp32 device
    tensor), the partial sums live in the library's own built-in device buffer.  -> (loss, dlogits)"""
    n, Cn = logits.shape
    if dlogits is None:
        dlogits = logits
    B.check(B.lib().mggcn_softmax_ce_static(n, Cn, B.ptr(logits), B.ld_of(logits), B.ptr(labels), B.ptr(loss),
                                            B.ptr(dlogits), B.ld_of(dlogits), _stream(stream)))
    return loss, dlogits


def mggcn_adam_step(W, G, m, v, step, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, stream=None):
    """In-place Adam update of a contiguous parameter tensor W with moments m, v."""
    assert W.is_contiguous() and G.is_contiguous() and m.is_contiguous() and v.is_contiguous()
    B.check(B.lib().mggcn_adam_step(W.numel(), B.ptr(W), B.ptr(G), B.ptr(m), B.ptr(v), int(step), lr, beta1, beta2,
                                    eps, _stream(stream)))
    return W


# ------------------------------------------------------------------------------------------
# model: layers and epoch
# ------------------------------------------------------------------------------------------

def mggcn_model_spmm_width_max(dims, orders=None, flags=0) -> int:
    L = len(dims) - 1
    d = (C.c_int32 * (L + 1))(*dims)
    o = (C.c_int32 * L)(*orders) if orders is not None else None
    return B.lib().mggcn_model_spmm_width_max(d, o, L, flags)


class Model:
    """Owns an mggcn_model handle and its activation arena (a device tensor)."""

    def __init__(self, graph: Graph, dims, orders=None, flags=0):
        L = B.lib()
        self.graph, self.dims = graph, list(dims)
        self.L = len(dims) - 1
        need = mggcn_model_spmm_width_max(dims, orders, flags)
        if graph.F_max < need:
            graph.bind(need)
        d = (C.c_int32 * (self.L + 1))(*dims)
        o = (C.c_int32 * self.L)(*orders) if orders is not None else None
        h = C.c_void_p(None)
        B.check(L.mggcn_model_create(graph.handle, self.L, d, o, flags, C.byref(h)))
        self.handle = h
        nbytes = L.mggcn_model_arena_bytes(h)
        self.arena = _ws(nbytes, graph.device)
        B.check(L.mggcn_model_bind(h, _ws_ptr(self.arena), nbytes))

    def order(self, l) -> int:
        return B.check(B.lib().mggcn_model_order(self.handle, l))

    def cache_input(self, X, stream=None):
        """MODEL_CACHE_INPUT: form and keep A^ X (call once, and again whenever X changes)."""
        B.check(B.lib().mggcn_model_cache_input(self.handle, B.ptr(X), B.ld_of(X), _stream(stream)))

    def activation(self, l):
        """(device address, ld) of layer l's result buffer"""
        p, ld = C.c_void_p(None), C.c_int64(0)
        B.check(B.lib().mggcn_model_activation(self.handle, l, C.byref(p), C.byref(ld)))
        return p.value, ld.value

    def activation_tensor(self, l):
        """A clone of layer l's result buffer as an (n, d_{l+1}) tensor (debug / tests)."""
        torch = _torch()
        p, ld = self.activation(l)
        n, d = self.graph.n_rows, self.dims[l + 1]
        base = _ws_ptr(self.arena)
        off = (p - base) // 4
        flat = self.arena[(base - self.arena.data_ptr()):].view(torch.float32)
        return flat[off: off + n * ld].view(n, ld)[:, :d].clone()

    def gather_operand(self, width):
        """MODEL_GATHER_BF16: a clone of the bfloat16 operand of the most recent SpMM, (n, width) int16."""
        torch = _torch()
        p, ld = C.c_void_p(None), C.c_int64(0)
        B.check(B.lib().mggcn_model_gather_operand(self.handle, width, C.byref(p), C.byref(ld)))
        n = self.graph.n_rows
        base = self.arena.data_ptr()
        off = p.value - base
        flat = self.arena[off: off + n * ld.value * 2].view(torch.int16)
        return flat.view(n, ld.value)[:, :width].clone()

    def close(self):
        if getattr(self, "handle", None):
            B.lib().mggcn_model_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def mggcn_layer_fwd(model: Model, l, H_in, W, relu=True, H_out=None, stream=None):
    torch = _torch()
    if H_out is None:
        H_out = torch.empty((H_in.shape[0], W.shape[1]), dtype=torch.float32, device=H_in.device)
    B.check(B.lib().mggcn_layer_fwd(model.handle, l, B.ptr(H_in), B.ld_of(H_in), B.ptr(W), B.ld_of(W), int(relu),
                                    B.ptr(H_out), B.ld_of(H_out), _stream(stream)))
    return H_out


def mggcn_layer_bwd(model: Model, l, H_in, act, G, W, need_input_grad=True, H_G=None, hg_relu_mask=False,
                    W_G=None, stream=None):
    """-> (W_G, H_G or None).  G is masked in place when `act` is given (Eq. 8)."""
    torch = _torch()
    if W_G is None:
        W_G = torch.empty_like(W)
    if need_input_grad and H_G is None:
        H_G = torch.empty((H_in.shape[0], W.shape[0]), dtype=torch.float32, device=H_in.device)
    if not need_input_grad:
        H_G = None
    B.check(B.lib().mggcn_layer_bwd(
        model.handle, l, B.ptr(H_in), B.ld_of(H_in), B.ptr(act), B.ld_of(act) if act is not None else 0,
        B.ptr(G), B.ld_of(G), B.ptr(W), B.ld_of(W), B.ptr(W_G), B.ld_of(W_G), B.ptr(H_G),
        B.ld_of(H_G) if H_G is not None else 0, int(hg_relu_mask), _stream(stream)))
    return W_G, H_G


def mggcn_epoch(model: Model, X, labels, Ws, W_Gs=None, loss=None, stream=None):
    """One epoch without optimiser: -> (loss 1-element device tensor, [W_G...])."""
    torch = _torch()
    if W_Gs is None:
        W_Gs = [torch.empty_like(w) for w in Ws]
    if loss is None:
        loss = torch.empty(1, dtype=torch.float32, device=labels.device)
    Wp = (C.c_void_p * model.L)(*[w.data_ptr() for w in Ws])
    Gp = (C.c_void_p * model.L)(*[w.data_ptr() for w in W_Gs])
    B.check(B.lib().mggcn_epoch(model.handle, B.ptr(X), B.ld_of(X) if X is not None else 0, B.ptr(labels), Wp,
                                B.ptr(loss), Gp, _stream(stream)))
    return loss, W_Gs


# ------------------------------------------------------------------------------------------
# memory-system probes (measurement aids for bench.py)
# ------------------------------------------------------------------------------------------

def mggcn_probe_read(buf, sink=None, stream=None):
    """Read a device tensor once, contiguously (timed by the caller)."""
    torch = _torch()
    if sink is None:
        sink = torch.empty(B.lib().mggcn_probe_sink_floats(), dtype=torch.float32, device=buf.device)
    B.check(B.lib().mggcn_probe_read(B.ptr(buf), buf.numel() * buf.element_size(), B.ptr(sink), _stream(stream)))
    return sink


def mggcn_probe_write(buf, value=0.0, stream=None):
    """Fill a device tensor once, contiguously (timed by the caller)."""
    B.check(B.lib().mggcn_probe_write(B.ptr(buf), buf.numel() * buf.element_size(), float(value), _stream(stream)))
    return buf


def mggcn_probe_mfma(iters, sink, stream=None) -> int:
    """Enqueue the fp32 matrix-instruction probe; -> floating-point operations it performs."""
    return B.check(B.lib().mggcn_probe_mfma(int(iters), B.ptr(sink), _stream(stream)))


def mggcn_probe_gather(X, idx, row_bytes=None, sink=None, stream=None):
    """Fetch the rows idx (int32 device tensor) of the 2-D device tensor X, `row_bytes` of each."""
    torch = _torch()
    if sink is None:
        sink = torch.empty(B.lib().mggcn_probe_sink_floats(), dtype=torch.float32, device=X.device)
    stride = B.ld_of(X) * X.element_size()
    if row_bytes is None:
        row_bytes = X.shape[1] * X.element_size()
    B.check(B.lib().mggcn_probe_gather(B.ptr(X), X.shape[0], int(row_bytes), stride, B.ptr(idx), idx.numel(), B.ptr(sink),
                                       _stream(stream)))
    return sink

"""ctypes binding of libsaga (argument marshalling only).

Every step of the layer runs inside the library's HIP kernels; torch is used
for device memory and the stream handle. Loading fails loudly when the shared
library is missing: there is no CPU fallback.
"""
from __future__ import annotations

import atexit
import ctypes
import os
import sys
import weakref
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsaga.so")

SAGA_OK = 0
STATUS_NAMES = {0: "OK", 1: "INVALID_ARG", 2: "BAD_GRAPH", 3: "UNSUPPORTED", 4: "BUDGET", 5: "HIP", 6: "INTERNAL"}
F32, BF16 = 0, 1
AGG = {"sum": 0, "max": 1}
ACT = {"none": 0, "relu": 1, "sigmoid": 2}
EDGE_OP = {"copy": 0, "mul_weight": 1, "gated": 2, "pool": 3}
MEM_DEVICE, MEM_HOST = 0, 1

# every entry point include/saga.h declares
EXPORTS = ["saga_create", "saga_destroy", "saga_graph_create_csc", "saga_graph_destroy",
           "saga_graph_set_edge_data", "saga_layer_forward", "saga_layer_forward_noalloc", "saga_layer_backward", "saga_set_profiling", "saga_reset_timings",
           "saga_get_timings", "saga_set_option", "saga_peak_device_bytes", "saga_last_error",
           "saga_graph_info", "saga_plan_work_list", "saga_plan_reencoding", "saga_copy_bytes", "saga_version"]


class SagaError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"saga: {STATUS_NAMES.get(status, status)}: {text}")
        self.status = status


class Tensor(ctypes.Structure):
    _fields_ = [("data", ctypes.c_void_p), ("rows", ctypes.c_int64), ("cols", ctypes.c_int64),
                ("ld", ctypes.c_int64), ("dtype", ctypes.c_int32), ("mem", ctypes.c_int32)]


class EdgeParams(ctypes.Structure):
    _fields_ = [("op", ctypes.c_int32), ("edge_weight", ctypes.c_void_p), ("W_gate", ctypes.POINTER(Tensor)),
                ("b_gate", ctypes.POINTER(Tensor)), ("W_msg", ctypes.POINTER(Tensor)),
                ("W_pool", ctypes.POINTER(Tensor)), ("b_pool", ctypes.POINTER(Tensor))]


class VertexParams(ctypes.Structure):
    _fields_ = [("W", ctypes.POINTER(Tensor)), ("bias", ctypes.POINTER(Tensor)), ("act", ctypes.c_int32),
                ("reserved", ctypes.c_int32), ("W_self", ctypes.POINTER(Tensor))]


class LayerGrads(ctypes.Structure):
    _fields_ = [("dX", ctypes.POINTER(Tensor)), ("dW", ctypes.POINTER(Tensor)), ("dbias", ctypes.POINTER(Tensor)),
                ("dW_self", ctypes.POINTER(Tensor)), ("dW_gate", ctypes.POINTER(Tensor)),
                ("db_gate", ctypes.POINTER(Tensor)), ("dW_msg", ctypes.POINTER(Tensor)),
                ("dW_pool", ctypes.POINTER(Tensor)), ("db_pool", ctypes.POINTER(Tensor))]


class Timings(ctypes.Structure):
    _fields_ = [("n_calls", ctypes.c_int64), ("ms_total", ctypes.c_double), ("ms_hoist", ctypes.c_double),
                ("ms_gather", ctypes.c_double), ("ms_combine", ctypes.c_double), ("ms_apply_vertex", ctypes.c_double),
                ("n_gather_launches", ctypes.c_int64), ("bytes_h2d", ctypes.c_int64), ("bytes_d2h", ctypes.c_int64),
                ("ms_wall_streamed", ctypes.c_double), ("plan_dst_intervals", ctypes.c_int32),
                ("plan_src_intervals", ctypes.c_int32), ("reserved", ctypes.c_int32),
                ("n_work_items", ctypes.c_int64), ("n_split_vertices", ctypes.c_int64), ("ms_dense_blocks", ctypes.c_double),
                ("n_dense_blocks", ctypes.c_int64), ("n_dense_edges", ctypes.c_int64), ("n_partial_rows", ctypes.c_int64),
                ("n_hoist_row_cols", ctypes.c_int64)]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_ if k != "reserved"}


_lib = None
_live_contexts = weakref.WeakSet()


@atexit.register
def _destroy_live_contexts():
    # Contexts still alive at interpreter exit are released here, while the HIP runtime is
    # still up; a destructor running during finalisation must not call into it any more.
    for c in list(_live_contexts):
        try:
            c.destroy()
        except Exception:
            pass


def load_library() -> ctypes.CDLL:
    """dlopen libsaga.so; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_1810_08403_amd.build` "
                          "(hipcc, gfx950). There is no CPU fallback.")
    _lib = declare_signatures(ctypes.CDLL(LIB_PATH))
    return _lib


def declare_signatures(L: ctypes.CDLL) -> ctypes.CDLL:
    """Argument and result types of every entry point of include/saga.h on a loaded library."""
    P, I64, I32, SZ = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_size_t
    L.saga_create.restype = I32
    L.saga_create.argtypes = [ctypes.POINTER(P), ctypes.c_int, P, SZ]
    L.saga_destroy.restype = I32
    L.saga_destroy.argtypes = [P]
    L.saga_graph_create_csc.restype = I32
    L.saga_graph_create_csc.argtypes = [P, I64, I64, P, P, I32, ctypes.POINTER(P)]
    L.saga_graph_destroy.restype = I32
    L.saga_graph_destroy.argtypes = [P]
    L.saga_graph_set_edge_data.restype = I32
    L.saga_graph_set_edge_data.argtypes = [P, P]
    L.saga_layer_forward.restype = I32
    L.saga_layer_forward.argtypes = [P, P, ctypes.POINTER(Tensor), ctypes.POINTER(EdgeParams), I32,
                                     ctypes.POINTER(VertexParams), ctypes.POINTER(Tensor), ctypes.POINTER(Tensor)]
    L.saga_layer_forward_noalloc.restype = I32
    L.saga_layer_forward_noalloc.argtypes = L.saga_layer_forward.argtypes
    L.saga_layer_backward.restype = I32
    L.saga_layer_backward.argtypes = [P, P, ctypes.POINTER(Tensor), ctypes.POINTER(Tensor), ctypes.POINTER(Tensor),
                                      ctypes.POINTER(Tensor), ctypes.POINTER(EdgeParams), I32,
                                      ctypes.POINTER(VertexParams), ctypes.POINTER(LayerGrads)]
    L.saga_set_profiling.restype = I32
    L.saga_set_profiling.argtypes = [P, I32]
    L.saga_reset_timings.restype = I32
    L.saga_reset_timings.argtypes = [P]
    L.saga_get_timings.restype = I32
    L.saga_get_timings.argtypes = [P, ctypes.POINTER(Timings)]
    L.saga_set_option.restype = I32
    L.saga_set_option.argtypes = [P, ctypes.c_char_p, I64]
    L.saga_peak_device_bytes.restype = SZ
    L.saga_peak_device_bytes.argtypes = [P]
    L.saga_last_error.restype = ctypes.c_char_p
    L.saga_last_error.argtypes = [P]
    L.saga_graph_info.restype = I32
    L.saga_graph_info.argtypes = [P, ctypes.POINTER(I64), ctypes.POINTER(I64), ctypes.POINTER(I64)]
    L.saga_plan_work_list.restype = I32
    L.saga_plan_work_list.argtypes = [I64, P, P, I64, I64, I64, I32, P, I64, ctypes.POINTER(I64), ctypes.POINTER(I64),
                                      ctypes.POINTER(I64), ctypes.POINTER(I64)]
    L.saga_copy_bytes.restype = I32
    L.saga_copy_bytes.argtypes = [P, P, P, SZ]
    L.saga_version.restype = ctypes.c_char_p
    L.saga_version.argtypes = []
    return L


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def as_tensor(t: Optional[torch.Tensor]) -> Optional[Tensor]:
    """View a 1-D or 2-D row-major torch tensor (unit stride along columns) as a saga_tensor."""
    if t is None:
        return None
    if t.dim() == 1:
        t = t.view(1, -1)
    if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1):
        raise ValueError("need a 2-D tensor with unit column stride")
    ld = t.stride(0) if t.shape[0] > 1 else max(t.shape[1], t.stride(0))
    mem = MEM_DEVICE if t.is_cuda else MEM_HOST
    return Tensor(t.data_ptr(), t.shape[0], t.shape[1], ld, _dtype_code(t), mem)


def _ref(s):
    return ctypes.byref(s) if s is not None else None


class Graph:
    def __init__(self, ctx: "Context", handle: int, n: int, nnz: int, device: bool):
        self.ctx, self._h, self.n, self.nnz, self.on_device = ctx, ctypes.c_void_p(handle), n, nnz, device

    def set_edge_data(self, w: torch.Tensor):
        assert w.dtype == torch.float32 and w.is_contiguous() and w.numel() == self.nnz
        assert w.is_cuda == self.on_device
        if w.is_cuda:
            self.ctx.stream.wait_stream(torch.cuda.current_stream(self.ctx.device))
        self.ctx._check(self.ctx.lib.saga_graph_set_edge_data(self._h, w.data_ptr()))

    def info(self):
        a, b, c = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
        self.ctx._check(self.ctx.lib.saga_graph_info(self._h, ctypes.byref(a), ctypes.byref(b), ctypes.byref(c)))
        return {"max_in_degree": a.value, "n_work_items": b.value, "n_split_vertices": c.value}

    def destroy(self):
        if self._h:
            self.ctx.lib.saga_graph_destroy(self._h)
            self._h = None

    def __del__(self):
        if sys.is_finalizing():
            return
        try:
            self.destroy()
        except Exception:
            pass


class Context:
    """saga_ctx on one GPU.

    The library enqueues on `stream`, a torch.cuda.Stream of default priority
    (a fresh one unless given). layer_forward orders that stream after torch's
    current stream and torch's current stream after it, so tensors produced or
    consumed by torch ops need no extra synchronisation.
    """

    def __init__(self, device: int = 0, stream: Optional["torch.cuda.Stream"] = None, hbm_budget_bytes: int = 0):
        self.lib = load_library()
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU visible: libsaga has no CPU path")
        self.stream = stream if stream is not None else torch.cuda.Stream(device=device)
        h = ctypes.c_void_p()
        st = self.lib.saga_create(ctypes.byref(h), device, ctypes.c_void_p(self.stream.cuda_stream), hbm_budget_bytes)
        if st != SAGA_OK:
            raise SagaError(st, "saga_create failed")
        self._h = h
        self.device = device
        self._graphs = weakref.WeakSet()
        _live_contexts.add(self)

    def synchronize(self):
        self.stream.synchronize()

    def _check(self, st: int):
        if st != SAGA_OK:
            raise SagaError(st, (self.lib.saga_last_error(self._h) or b"").decode())

    def set_option(self, name: str, value: int):
        self._check(self.lib.saga_set_option(self._h, name.encode(), int(value)))

    def graph_create_csc(self, n: int, col_ptr: torch.Tensor, row_idx: torch.Tensor) -> Graph:
        assert col_ptr.dtype == torch.int64 and row_idx.dtype == torch.int32
        assert col_ptr.is_contiguous() and row_idx.is_contiguous() and col_ptr.numel() == n + 1
        assert col_ptr.is_cuda == row_idx.is_cuda
        g = ctypes.c_void_p()
        where = MEM_DEVICE if col_ptr.is_cuda else MEM_HOST
        if col_ptr.is_cuda:
            self.stream.wait_stream(torch.cuda.current_stream(self.device))
        self._check(self.lib.saga_graph_create_csc(self._h, n, row_idx.numel(), col_ptr.data_ptr(),
                                                   row_idx.data_ptr(), where, ctypes.byref(g)))
        graph = Graph(self, g.value, n, row_idx.numel(), col_ptr.is_cuda)
        self._graphs.add(graph)
        return graph

    def layer_forward(self, g: Graph, X: torch.Tensor, Y: torch.Tensor, edge_op: str = "copy",
                      edge_weight: Optional[torch.Tensor] = None, W_gate=None, b_gate=None, W_msg=None,
                      W_pool=None, b_pool=None, agg: str = "sum", W=None, bias=None, W_self=None, act: str = "none",
                      accum_out=None, no_alloc: bool = False):
        """saga_layer_forward, or saga_layer_forward_noalloc with no_alloc=True."""
        tx, ty = as_tensor(X), as_tensor(Y)
        twg, tbg, twm = as_tensor(W_gate), as_tensor(b_gate), as_tensor(W_msg)
        twp, tbp, tws = as_tensor(W_pool), as_tensor(b_pool), as_tensor(W_self)
        tw, tb, tacc = as_tensor(W), as_tensor(bias), as_tensor(accum_out)
        if edge_weight is not None:
            assert edge_weight.dtype == torch.float32 and edge_weight.is_contiguous()
            assert edge_weight.numel() == g.nnz
        ep = EdgeParams(EDGE_OP[edge_op], edge_weight.data_ptr() if edge_weight is not None else None,
                        ctypes.pointer(twg) if twg is not None else None,
                        ctypes.pointer(tbg) if tbg is not None else None,
                        ctypes.pointer(twm) if twm is not None else None,
                        ctypes.pointer(twp) if twp is not None else None,
                        ctypes.pointer(tbp) if tbp is not None else None)
        vp = VertexParams(ctypes.pointer(tw) if tw is not None else None,
                          ctypes.pointer(tb) if tb is not None else None, ACT[act], 0,
                          ctypes.pointer(tws) if tws is not None else None)
        cur = torch.cuda.current_stream(self.device)
        if cur != self.stream:
            self.stream.wait_stream(cur)
        entry = self.lib.saga_layer_forward_noalloc if no_alloc else self.lib.saga_layer_forward
        self._check(entry(self._h, g._h, ctypes.byref(tx), ctypes.byref(ep), AGG[agg], ctypes.byref(vp), ctypes.byref(ty), _ref(tacc)))
        if cur != self.stream:
            cur.wait_stream(self.stream)
        return Y

    def layer_backward(self, g: Graph, A: torch.Tensor, dY: torch.Tensor, W: torch.Tensor, dW: torch.Tensor,
                       X: Optional[torch.Tensor] = None, Y: Optional[torch.Tensor] = None, edge_op: str = "copy",
                       edge_weight: Optional[torch.Tensor] = None, agg: str = "sum", bias=None, W_self=None,
                       act: str = "none", dX=None, dbias=None, dW_self=None, W_gate=None, b_gate=None, W_msg=None,
                       dW_gate=None, db_gate=None, dW_msg=None, W_pool=None, b_pool=None, dW_pool=None, db_pool=None):
        """saga_layer_backward: gradients are written into dW (and dX, dbias, dW_self, dW_gate, db_gate, dW_msg, dW_pool,
        db_pool when given)."""
        tx, ta, ty, tdy = as_tensor(X), as_tensor(A), as_tensor(Y), as_tensor(dY)
        tw, tb, tws = as_tensor(W), as_tensor(bias), as_tensor(W_self)
        tdx, tdw, tdb, tdws = as_tensor(dX), as_tensor(dW), as_tensor(dbias), as_tensor(dW_self)
        if edge_weight is not None:
            assert edge_weight.dtype == torch.float32 and edge_weight.is_contiguous()
            assert edge_weight.numel() == g.nnz
        twg, tbg, twm = as_tensor(W_gate), as_tensor(b_gate), as_tensor(W_msg)
        tdwg, tdbg, tdwm = as_tensor(dW_gate), as_tensor(db_gate), as_tensor(dW_msg)
        twp, tbp, tdwp, tdbp = as_tensor(W_pool), as_tensor(b_pool), as_tensor(dW_pool), as_tensor(db_pool)
        ptr = lambda t: ctypes.pointer(t) if t is not None else None
        ep = EdgeParams(EDGE_OP[edge_op], edge_weight.data_ptr() if edge_weight is not None else None,
                        ptr(twg), ptr(tbg), ptr(twm), ptr(twp), ptr(tbp))
        vp = VertexParams(ptr(tw), ptr(tb), ACT[act], 0, ptr(tws))
        grads = LayerGrads(ptr(tdx), ptr(tdw), ptr(tdb), ptr(tdws), ptr(tdwg), ptr(tdbg), ptr(tdwm), ptr(tdwp), ptr(tdbp))
        cur = torch.cuda.current_stream(self.device)
        if cur != self.stream:
            self.stream.wait_stream(cur)
        self._check(self.lib.saga_layer_backward(self._h, g._h, _ref(tx), _ref(ta), _ref(ty), _ref(tdy), ctypes.byref(ep),
                                                 AGG[agg], ctypes.byref(vp), ctypes.byref(grads)))
        if cur != self.stream:
            cur.wait_stream(self.stream)
        return dW

    def copy_bytes(self, dst: torch.Tensor, src: torch.Tensor):
        """Plain copy kernel on the library's stream (counter calibration)."""
        nbytes = src.numel() * src.element_size()
        assert dst.numel() * dst.element_size() == nbytes and dst.is_cuda and src.is_cuda
        cur = torch.cuda.current_stream(self.device)
        self.stream.wait_stream(cur)
        self._check(self.lib.saga_copy_bytes(self._h, dst.data_ptr(), src.data_ptr(), nbytes))
        cur.wait_stream(self.stream)

    def set_profiling(self, on: bool):
        self._check(self.lib.saga_set_profiling(self._h, 1 if on else 0))

    def reset_timings(self):
        self._check(self.lib.saga_reset_timings(self._h))

    def get_timings(self) -> dict:
        t = Timings()
        self._check(self.lib.saga_get_timings(self._h, ctypes.byref(t)))
        return t.as_dict()

    def peak_device_bytes(self) -> int:
        return int(self.lib.saga_peak_device_bytes(self._h))

    def destroy(self):
        if self._h:
            for g in list(self._graphs):   # graphs point into the context: release them first
                g.destroy()
            self.lib.saga_destroy(self._h)
            self._h = None

    def __del__(self):
        if sys.is_finalizing():
            return
        try:
            self.destroy()
        except Exception:
            pass


def plan_work_list(col_ptr: torch.Tensor, row_idx: torch.Tensor, min_edges=64, cut_degree=128, stripe_rows=1024, team=1):
    """Host-only: the work list the library would build (int32 tensor [n_items, 4]) and its counts."""
    L = load_library()
    assert not col_ptr.is_cuda and col_ptr.dtype == torch.int64 and row_idx.dtype == torch.int32
    n = col_ptr.numel() - 1
    a, t, b, c = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
    args = (n, col_ptr.data_ptr(), row_idx.data_ptr(), min_edges, cut_degree, stripe_rows, team)
    refs = (ctypes.byref(a), ctypes.byref(t), ctypes.byref(b), ctypes.byref(c))
    st = L.saga_plan_work_list(*args, None, 0, *refs)
    if st != SAGA_OK:
        raise SagaError(st, "saga_plan_work_list")
    items = torch.empty(a.value, 4, dtype=torch.int32)
    st = L.saga_plan_work_list(*args, items.data_ptr(), a.value, *refs)
    if st != SAGA_OK:
        raise SagaError(st, "saga_plan_work_list")
    return items, {"n_items": a.value, "n_team_items": t.value, "n_split_vertices": b.value, "n_slots": c.value}


def plan_reencoding(col_ptr: torch.Tensor, row_idx: torch.Tensor, dst_intervals: int, src_intervals: int, seed: int = 0):
    """Host-only: new_id (int32 tensor [n]) that evens out the chunk edge counts of the tiling, and
    (max, min, chunks) of the chunk edge counts before and after."""
    L = load_library()
    assert not col_ptr.is_cuda and col_ptr.dtype == torch.int64 and row_idx.dtype == torch.int32
    L.saga_plan_reencoding.restype = ctypes.c_int32
    L.saga_plan_reencoding.argtypes = [ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32,
                                       ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
    n = col_ptr.numel() - 1
    new_id = torch.empty(n, dtype=torch.int32)
    before, after = (ctypes.c_int64 * 3)(), (ctypes.c_int64 * 3)()
    st = L.saga_plan_reencoding(n, col_ptr.data_ptr(), row_idx.data_ptr(), dst_intervals, src_intervals, seed,
                                new_id.data_ptr(), before, after)
    if st != SAGA_OK:
        raise SagaError(st, "saga_plan_reencoding")
    keys = ("max_chunk_edges", "min_chunk_edges", "chunks")
    return new_id, {"before": dict(zip(keys, before)), "after": dict(zip(keys, after))}


def version() -> str:
    return load_library().saga_version().decode()

"""Drive the host code of libsaga, built against the CPU stand-in of the HIP runtime, from Python.

Test infrastructure only. `StubContext` has the methods of `paper_1810_08403_amd.Context` that the
session tests use; tensors are CPU torch tensors, and one wrapped in `Dev` stands for device memory.
"""
from __future__ import annotations

import ctypes
import os

import torch

from paper_1810_08403_amd import binding as B

HERE = os.path.dirname(os.path.abspath(__file__))


class Dev:
    """A CPU tensor handed to the library as if it lived in device memory."""
    def __init__(self, t: torch.Tensor):
        self.t = t.contiguous()


def dev(t):
    return None if t is None else Dev(t)


def _as_tensor(x):
    if x is None:
        return None
    mem = B.MEM_HOST
    if isinstance(x, Dev):
        x, mem = x.t, B.MEM_DEVICE
    t = B.as_tensor(x)
    t.mem = mem
    return t


def _ptr(t):
    return ctypes.pointer(t) if t is not None else None


class _device_scope:
    """Declare the given Dev tensors device memory for the duration of one library call: the host code must not read
    or write them (on the real machine that is a segmentation fault), only the stand-ins for copies and kernels may."""
    def __init__(self, lib, *objs):
        self.lib, self.ts = lib, [o.t for o in objs if isinstance(o, Dev) and o.t.numel() > 0]

    def __enter__(self):
        for t in self.ts:
            self.lib.stub_register_device(t.data_ptr(), t.numel() * t.element_size())

    def __exit__(self, *exc):
        for t in self.ts:
            self.lib.stub_unregister_device(t.data_ptr())


class StubGraph:
    def __init__(self, ctx, handle, n, nnz, device):
        self.ctx, self._h, self.n, self.nnz, self.on_device = ctx, ctypes.c_void_p(handle), n, nnz, device

    def set_edge_data(self, w):
        if isinstance(w, Dev):
            assert self.on_device
            w = w.t
        else:
            assert not self.on_device
        assert w.dtype == torch.float32 and w.is_contiguous() and w.numel() == self.nnz
        with _device_scope(self.ctx.lib, Dev(w) if self.on_device else None):
            self.ctx._check(self.ctx.lib.saga_graph_set_edge_data(self._h, w.data_ptr()))

    def destroy(self):
        if self._h:
            self.ctx.lib.saga_graph_destroy(self._h)
            self._h = None


class StubContext:
    def __init__(self, lib_path: str, hbm_budget_bytes: int = 0):
        self.lib = B.declare_signatures(ctypes.CDLL(lib_path))
        self.lib.stub_set_mode.argtypes = [ctypes.c_int, ctypes.c_uint64]
        self.lib.stub_set_mode.restype = None
        self.lib.stub_live_counts.argtypes = [ctypes.POINTER(ctypes.c_int64)] * 4
        self.lib.stub_live_counts.restype = None
        self.lib.stub_fail_allocation.argtypes = [ctypes.c_int64]
        self.lib.stub_fail_allocation.restype = None
        self.lib.stub_register_device.argtypes = [ctypes.c_void_p, ctypes.c_size_t]
        self.lib.stub_register_device.restype = None
        self.lib.stub_unregister_device.argtypes = [ctypes.c_void_p]
        self.lib.stub_unregister_device.restype = None
        self.lib.stub_allocator_calls.argtypes = []
        self.lib.stub_allocator_calls.restype = ctypes.c_int64
        h = ctypes.c_void_p()
        st = self.lib.saga_create(ctypes.byref(h), 0, None, hbm_budget_bytes)
        if st != B.SAGA_OK:
            raise B.SagaError(st, "saga_create failed")
        self._h = h

    def set_mode(self, mode: int, seed: int = 0):
        self.lib.stub_set_mode(mode, seed)

    def synchronize(self):
        self.lib.stub_device_synchronize()

    def live_counts(self):
        v = [ctypes.c_int64() for _ in range(4)]
        self.lib.stub_live_counts(*[ctypes.byref(x) for x in v])
        return dict(zip(("allocations", "bytes", "streams", "events"), (x.value for x in v)))

    def _check(self, st):
        if st != B.SAGA_OK:
            raise B.SagaError(st, (self.lib.saga_last_error(self._h) or b"").decode())

    def set_option(self, name, value):
        self._check(self.lib.saga_set_option(self._h, name.encode(), int(value)))

    def set_profiling(self, on):
        self._check(self.lib.saga_set_profiling(self._h, 1 if on else 0))

    def reset_timings(self):
        self._check(self.lib.saga_reset_timings(self._h))

    def get_timings(self):
        t = B.Timings()
        self._check(self.lib.saga_get_timings(self._h, ctypes.byref(t)))
        return t.as_dict()

    def peak_device_bytes(self):
        return int(self.lib.saga_peak_device_bytes(self._h))

    def graph_create_csc(self, n, col_ptr, row_idx):
        device = isinstance(col_ptr, Dev)
        cp = col_ptr.t if device else col_ptr
        ri = row_idx.t if isinstance(row_idx, Dev) else row_idx
        assert cp.dtype == torch.int64 and ri.dtype == torch.int32 and cp.is_contiguous() and ri.is_contiguous()
        g = ctypes.c_void_p()
        with _device_scope(self.lib, col_ptr, row_idx):
            self._check(self.lib.saga_graph_create_csc(self._h, n, ri.numel(), cp.data_ptr(), ri.data_ptr(),
                                                       B.MEM_DEVICE if device else B.MEM_HOST, ctypes.byref(g)))
        return StubGraph(self, g.value, n, ri.numel(), device)

    def layer_forward(self, g, X, Y, edge_op="copy", edge_weight=None, W_gate=None, b_gate=None, W_msg=None, W_pool=None, b_pool=None,
                      agg="sum", W=None, bias=None, W_self=None, act="none", accum_out=None, no_alloc=False):
        keep = [_as_tensor(t) for t in (X, Y, W_gate, b_gate, W_msg, W_pool, b_pool, W, bias, W_self, accum_out)]
        tx, ty, twg, tbg, twm, twp, tbp, tw, tb, tws, tacc = keep
        ew = edge_weight.t if isinstance(edge_weight, Dev) else edge_weight
        ep = B.EdgeParams(B.EDGE_OP[edge_op], ew.data_ptr() if ew is not None else None, _ptr(twg), _ptr(tbg), _ptr(twm), _ptr(twp), _ptr(tbp))
        vp = B.VertexParams(_ptr(tw), _ptr(tb), B.ACT[act], 0, _ptr(tws))
        with _device_scope(self.lib, X, Y, W_gate, b_gate, W_msg, W_pool, b_pool, W, bias, W_self, accum_out, edge_weight):
            entry = self.lib.saga_layer_forward_noalloc if no_alloc else self.lib.saga_layer_forward
            self._check(entry(self._h, g._h, ctypes.byref(tx), ctypes.byref(ep), B.AGG[agg], ctypes.byref(vp), ctypes.byref(ty),
                              ctypes.byref(tacc) if tacc is not None else None))
        return Y

    def layer_backward(self, g, A, dY, W, dW, X=None, Y=None, edge_op="copy", edge_weight=None, agg="sum", bias=None, W_self=None, act="none",
                       dX=None, dbias=None, dW_self=None, W_gate=None, b_gate=None, W_msg=None, dW_gate=None, db_gate=None, dW_msg=None,
                       W_pool=None, b_pool=None, dW_pool=None, db_pool=None):
        T = _as_tensor
        tx, ta, ty, tdy, tw, tb, tws = T(X), T(A), T(Y), T(dY), T(W), T(bias), T(W_self)
        tdx, tdw, tdb, tdws = T(dX), T(dW), T(dbias), T(dW_self)
        twg, tbg, twm, tdwg, tdbg, tdwm = T(W_gate), T(b_gate), T(W_msg), T(dW_gate), T(db_gate), T(dW_msg)
        twp, tbp, tdwp, tdbp = T(W_pool), T(b_pool), T(dW_pool), T(db_pool)
        ew = edge_weight.t if isinstance(edge_weight, Dev) else edge_weight
        ep = B.EdgeParams(B.EDGE_OP[edge_op], ew.data_ptr() if ew is not None else None, _ptr(twg), _ptr(tbg), _ptr(twm), _ptr(twp), _ptr(tbp))
        vp = B.VertexParams(_ptr(tw), _ptr(tb), B.ACT[act], 0, _ptr(tws))
        grads = B.LayerGrads(_ptr(tdx), _ptr(tdw), _ptr(tdb), _ptr(tdws), _ptr(tdwg), _ptr(tdbg), _ptr(tdwm), _ptr(tdwp), _ptr(tdbp))
        ref = lambda t: ctypes.byref(t) if t is not None else None
        with _device_scope(self.lib, A, dY, W, dW, X, Y, edge_weight, bias, W_self, dX, dbias, dW_self, W_gate, b_gate, W_msg, dW_gate, db_gate,
                           dW_msg, W_pool, b_pool, dW_pool, db_pool):
            self._check(self.lib.saga_layer_backward(self._h, g._h, ref(tx), ref(ta), ref(ty), ref(tdy), ctypes.byref(ep), B.AGG[agg],
                                                     ctypes.byref(vp), ctypes.byref(grads)))
        return dW

    def destroy(self):
        if self._h:
            self.lib.saga_destroy(self._h)
            self._h = None

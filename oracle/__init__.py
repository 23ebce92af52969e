"""CPU oracle for the SAGA-NN layer: test infrastructure only.

Only tests/, the smoke check and the benchmark's cpu_baseline leg may import
this package. It never imports the HIP package, and the HIP package never
imports it. The arithmetic lives in saga_oracle.c (plain C loops, fp64
accumulation) and follows Section 2 (SAGA-NN stages, Example 2.1, Figure 2),
Figures 9 and 10 (CommNet and GCN programs) and Section 3.2 (hoisting) of the
NGra paper; this file only marshals numpy arrays into it.

Parity pins (tests/test_oracle_pins.py): dense brute force with numpy, the
sparse-dense product identity of Section 6.1 via scipy.sparse, the in-degree
invariant, brute-force max over the raw edge list, gated special cases that
reduce to the other edge functions, a dense broadcast formulation of the gate,
hoisted == naive, dense forms of the CommNet and max-pooling layers (Figures 9,
11), and hand-worked values under tests/golden/. The backward functions
(Section 2.2's backward stages) are pinned by dense matrix forms, finite
differences of the forward functions and automatic differentiation of dense
formulations of the layers.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

from .build import LIB, build

EDGE_OPS = {"copy": 0, "mul_weight": 1, "gated": 2, "pool": 3}
AGGS = {"sum": 0, "max": 1}
ACTS = {"none": 0, "relu": 1, "sigmoid": 2}

_lib = None
_P, _I64, _I32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32


class _Args(ctypes.Structure):
    """Mirror of saga_oracle_args in saga_oracle.c."""
    _fields_ = [("n", _I64), ("col_ptr", _P), ("row_idx", _P), ("X", _P), ("F", _I64),
                ("edge_op", _I32), ("agg", _I32), ("edge_w", _P),
                ("W_gate", _P), ("b_gate", _P), ("W_msg", _P),
                ("W_pool", _P), ("b_pool", _P), ("F_pool", _I64),
                ("Ps", _P), ("Pd", _P), ("M", _P), ("Ps_abs", _P), ("Pd_abs", _P), ("M_abs", _P),
                ("H", _P), ("H_abs", _P),
                ("W", _P), ("bias", _P), ("W_self", _P), ("F_out", _I64), ("act", _I32), ("pad", _I32),
                ("vlist", _P), ("nv", _I64), ("A", _P), ("A_abs", _P), ("Y", _P), ("Y_abs", _P)]


class _BwdArgs(ctypes.Structure):
    """Mirror of saga_oracle_bwd_args in saga_oracle.c."""
    _fields_ = [("n", _I64), ("col_ptr", _P), ("row_idx", _P), ("X", _P), ("F", _I64),
                ("edge_op", _I32), ("act", _I32), ("edge_w", _P), ("A", _P),
                ("W", _P), ("bias", _P), ("W_self", _P), ("F_out", _I64), ("dY", _P),
                ("dX", _P), ("dX_abs", _P), ("dW", _P), ("dW_abs", _P), ("dW_self", _P), ("dbias", _P), ("dA", _P),
                ("dW_self_abs", _P), ("dbias_abs", _P)]


class _GBwdArgs(ctypes.Structure):
    """Mirror of saga_oracle_gbwd_args in saga_oracle.c."""
    _fields_ = [("n", _I64), ("col_ptr", _P), ("row_idx", _P), ("X", _P), ("F", _I64),
                ("W_gate", _P), ("b_gate", _P), ("W_msg", _P), ("A", _P), ("W", _P), ("bias", _P),
                ("F_out", _I64), ("act", _I32), ("agg", _I32), ("dY", _P),
                ("dX", _P), ("dX_abs", _P), ("dW", _P), ("dW_abs", _P), ("dbias", _P),
                ("dW_gate", _P), ("dW_gate_abs", _P), ("db_gate", _P), ("db_gate_abs", _P),
                ("dW_msg", _P), ("dW_msg_abs", _P),
                ("W_self", _P), ("dW_self", _P), ("dW_self_abs", _P), ("dbias_abs", _P), ("A_max", _P)]


class _MBwdArgs(ctypes.Structure):
    """Mirror of saga_oracle_mbwd_args in saga_oracle.c."""
    _fields_ = [("n", _I64), ("col_ptr", _P), ("row_idx", _P), ("X", _P), ("F", _I64),
                ("edge_op", _I32), ("act", _I32), ("edge_w", _P), ("W_pool", _P), ("b_pool", _P), ("F_pool", _I64),
                ("W", _P), ("bias", _P), ("F_out", _I64), ("dY", _P), ("A", _P),
                ("dX", _P), ("dX_abs", _P), ("dW", _P), ("dW_abs", _P), ("dbias", _P),
                ("dW_pool", _P), ("dW_pool_abs", _P), ("db_pool", _P), ("db_pool_abs", _P),
                ("W_self", _P), ("dW_self", _P), ("dW_self_abs", _P), ("dbias_abs", _P)]


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB):
            build()
        L = ctypes.CDLL(LIB)
        L.saga_oracle_num_threads.restype = ctypes.c_int
        L.saga_oracle_hoist.restype = ctypes.c_int
        L.saga_oracle_hoist.argtypes = [_I64, _P, _I64, _P, _P, _P, _P, _P, _P, _P, _P]
        L.saga_oracle_hoist_pool.restype = ctypes.c_int
        L.saga_oracle_hoist_pool.argtypes = [_I64, _P, _I64, _P, _P, _I64, _P, _P]
        L.saga_oracle_layer.restype = ctypes.c_int
        L.saga_oracle_layer.argtypes = [ctypes.POINTER(_Args)]
        L.saga_oracle_layer_backward.restype = ctypes.c_int
        L.saga_oracle_layer_backward.argtypes = [ctypes.POINTER(_BwdArgs)]
        L.saga_oracle_max_backward.restype = ctypes.c_int
        L.saga_oracle_max_backward.argtypes = [ctypes.POINTER(_MBwdArgs)]
        L.saga_oracle_gated_backward.restype = ctypes.c_int
        L.saga_oracle_gated_backward.argtypes = [ctypes.POINTER(_GBwdArgs)]
        L.saga_oracle_gated_backward_sample.restype = ctypes.c_int
        L.saga_oracle_gated_backward_sample.argtypes = [ctypes.POINTER(_GBwdArgs), _I64, _P, _P, _P]
        L.saga_oracle_max_backward_sample.restype = ctypes.c_int
        L.saga_oracle_max_backward_sample.argtypes = [ctypes.POINTER(_MBwdArgs), _I64, _P, _P, _P]
        L.saga_oracle_backward_sample.restype = ctypes.c_int
        L.saga_oracle_backward_sample.argtypes = [ctypes.POINTER(_BwdArgs), _I64, _P, _P, _P, _I64, _P, _P, _P, _P]
        _lib = L
    return _lib


def num_threads() -> int:
    return int(lib().saga_oracle_num_threads())


def _f32(a):
    return None if a is None else np.ascontiguousarray(np.asarray(a, dtype=np.float32))


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def hoist(X, W_gate, W_msg=None):
    """Per-vertex products of Section 3.2 as fp64 arrays n x F: (Ps, Pd, M, Ps_abs, Pd_abs, M_abs),
    the last three being the absolute-term sums of the first three."""
    X = _f32(X)
    n, F = X.shape
    Wg, Wm = _f32(W_gate), _f32(W_msg)
    assert Wg.shape == (F, 2 * F) and (Wm is None or Wm.shape == (F, F))
    out = tuple(np.empty((n, F), np.float64) for _ in range(6))
    rc = lib().saga_oracle_hoist(n, _ptr(X), F, _ptr(Wg), _ptr(Wm), *[_ptr(a) for a in out])
    assert rc == 0
    return out


def hoist_pool(X, W_pool, b_pool=None):
    """H = sigmoid(X W_pool^T + b) per vertex (Figure 11's ApplyEdge, hoisted) and its error scale."""
    X = _f32(X)
    n, F = X.shape
    Wp, bp = _f32(W_pool), _f32(b_pool)
    Fp = Wp.shape[0]
    assert Wp.shape == (Fp, F) and (bp is None or bp.shape == (Fp,))
    H, Ha = np.empty((n, Fp), np.float64), np.empty((n, Fp), np.float64)
    rc = lib().saga_oracle_hoist_pool(n, _ptr(X), F, _ptr(Wp), _ptr(bp), Fp, _ptr(H), _ptr(Ha))
    assert rc == 0
    return H, Ha


def layer(col_ptr, row_idx, X, edge_op="copy", edge_weight=None, W_gate=None, b_gate=None, W_msg=None,
          W_pool=None, b_pool=None, agg="sum", W=None, bias=None, W_self=None, act="none", vlist=None,
          hoisted=None, want_abs=True):
    """Run one layer on the CPU oracle.

    Returns a dict with fp64 arrays: "A" (Gather output, nv x Fm), "A_abs" (its error scale),
    and, when W is given, "Y" (nv x F_out) and "Y_abs". vlist selects the destination vertices
    (default: all, in order). hoisted = the tuple from hoist() (gated) or hoist_pool() (pool)
    switches the message to its hoisted form.
    """
    col_ptr = np.ascontiguousarray(np.asarray(col_ptr, dtype=np.int64))
    row_idx = np.ascontiguousarray(np.asarray(row_idx, dtype=np.int32))
    X = _f32(X)
    n, F = X.shape
    assert col_ptr.shape == (n + 1,) and int(col_ptr[-1]) == row_idx.shape[0]
    w = _f32(edge_weight)
    Wg, bg, Wm = _f32(W_gate), _f32(b_gate), _f32(W_msg)
    Wp, bp = _f32(W_pool), _f32(b_pool)
    if Wg is not None:
        assert Wg.shape == (F, 2 * F)
    if Wm is not None:
        assert Wm.shape == (F, F)
    if bg is not None:
        assert bg.shape == (F,)
    if w is not None:
        assert w.shape == (row_idx.shape[0],)
    Fm, Fp = F, 0
    if edge_op == "pool":
        if hoisted is not None:
            Fp = np.asarray(hoisted[0]).shape[1]
        else:
            Fp = Wp.shape[0]
            assert Wp.shape == (Fp, F) and (bp is None or bp.shape == (Fp,))
        Fm = Fp
    Wv, bv, Ws = _f32(W), _f32(bias), _f32(W_self)
    F_out = 0
    if Wv is not None:
        assert Wv.shape[0] == Fm
        F_out = Wv.shape[1]
        if bv is not None:
            assert bv.shape == (F_out,)
        if Ws is not None:
            assert Ws.shape == (F, F_out)
    if vlist is None:
        vl, nv = None, n
    else:
        vl = np.ascontiguousarray(np.asarray(vlist, dtype=np.int64))
        nv = vl.shape[0]
    G = [None] * 6
    H = [None] * 2
    if hoisted is not None:
        hs = [np.ascontiguousarray(a, dtype=np.float64) for a in hoisted]
        if edge_op == "pool":
            assert len(hs) == 2
            H = hs
        else:
            assert len(hs) == 6
            G = hs
    out = {"A": np.empty((nv, Fm), np.float64)}
    if want_abs:
        out["A_abs"] = np.empty((nv, Fm), np.float64)
    if Wv is not None:
        out["Y"] = np.empty((nv, F_out), np.float64)
        if want_abs:
            out["Y_abs"] = np.empty((nv, F_out), np.float64)
    a = _Args(n, _ptr(col_ptr), _ptr(row_idx), _ptr(X), F, EDGE_OPS[edge_op], AGGS[agg], _ptr(w),
              _ptr(Wg), _ptr(bg), _ptr(Wm), _ptr(Wp), _ptr(bp), Fp,
              *[_ptr(x) for x in G], *[_ptr(x) for x in H],
              _ptr(Wv), _ptr(bv), _ptr(Ws), F_out, ACTS[act], 0,
              _ptr(vl), nv, _ptr(out["A"]), _ptr(out.get("A_abs")), _ptr(out.get("Y")), _ptr(out.get("Y_abs")))
    rc = lib().saga_oracle_layer(ctypes.byref(a))
    if rc != 0:
        raise ValueError("saga_oracle_layer rejected its arguments")
    return out


def layer_backward(col_ptr, row_idx, X, A, dY, W, edge_op="copy", edge_weight=None, bias=None, W_self=None, act="none"):
    """Gradients of one sum-accumulator layer with a linear ApplyEdge (Section 2.2's backward stages).

    A is the forward Gather output (fp64, from layer()); dY the gradient of the layer's output.
    Returns fp64 arrays: dX, dX_abs, dW, dW_abs, dbias, dbias_abs, dA, and dW_self, dW_self_abs when W_self is given.
    """
    col_ptr = np.ascontiguousarray(np.asarray(col_ptr, dtype=np.int64))
    row_idx = np.ascontiguousarray(np.asarray(row_idx, dtype=np.int32))
    X, Wv, dYv = _f32(X), _f32(W), _f32(dY)
    A = np.ascontiguousarray(np.asarray(A, dtype=np.float64))
    n, F = X.shape
    F_out = Wv.shape[1]
    assert A.shape == (n, F) and Wv.shape == (F, F_out) and dYv.shape == (n, F_out)
    w, bv, Ws = _f32(edge_weight), _f32(bias), _f32(W_self)
    out = {"dX": np.empty((n, F)), "dX_abs": np.empty((n, F)), "dW": np.empty((F, F_out)), "dW_abs": np.empty((F, F_out)),
           "dbias": np.empty(F_out), "dbias_abs": np.empty(F_out), "dA": np.empty((n, F))}
    if Ws is not None:
        assert Ws.shape == (F, F_out)
        out["dW_self"] = np.empty((F, F_out))
        out["dW_self_abs"] = np.empty((F, F_out))
    a = _BwdArgs(n, _ptr(col_ptr), _ptr(row_idx), _ptr(X), F, EDGE_OPS[edge_op], ACTS[act], _ptr(w), _ptr(A),
                 _ptr(Wv), _ptr(bv), _ptr(Ws), F_out, _ptr(dYv), _ptr(out["dX"]), _ptr(out["dX_abs"]), _ptr(out["dW"]),
                 _ptr(out["dW_abs"]), _ptr(out.get("dW_self")), _ptr(out["dbias"]), _ptr(out["dA"]),
                 _ptr(out.get("dW_self_abs")), _ptr(out["dbias_abs"]))
    rc = lib().saga_oracle_layer_backward(ctypes.byref(a))
    if rc != 0:
        raise ValueError("saga_oracle_layer_backward rejected its arguments")
    return out


def backward_sample(col_ptr, row_idx, X, A, dY, W, ulist, w_entries, edge_op="copy", edge_weight=None, bias=None, W_self=None,
                    act="none", want_dbias=False):
    """layer_backward's definitions evaluated only for the rows dX[ulist] and the entries dW[f, o] in w_entries
    (a list of (f, o) pairs), for graphs too large to do whole. A may be fp32 or fp64 (it is read as fp64).
    Returns dict: dX, dX_abs (len(ulist) x F), dW, dW_abs (len(w_entries)), and dbias, dbias_abs when asked for."""
    col_ptr = np.ascontiguousarray(np.asarray(col_ptr, dtype=np.int64))
    row_idx = np.ascontiguousarray(np.asarray(row_idx, dtype=np.int32))
    Wv, dYv = _f32(W), _f32(dY)
    A = np.ascontiguousarray(np.asarray(A, dtype=np.float64))
    n, F = A.shape
    F_out = Wv.shape[1]
    Xv = _f32(X)
    assert Wv.shape == (F, F_out) and dYv.shape == (n, F_out) and (Xv is None or Xv.shape == (n, F))
    w, bv, Ws = _f32(edge_weight), _f32(bias), _f32(W_self)
    ul = np.ascontiguousarray(np.asarray(ulist, dtype=np.int64))
    wf = np.ascontiguousarray(np.asarray([f for f, _ in w_entries], dtype=np.int64))
    wo = np.ascontiguousarray(np.asarray([o for _, o in w_entries], dtype=np.int64))
    assert ((wf >= 0) & (wf < F)).all() and ((wo >= 0) & (wo < F_out)).all()
    out = {"dX": np.zeros((len(ul), F)), "dX_abs": np.zeros((len(ul), F)), "dW": np.zeros(len(wf)), "dW_abs": np.zeros(len(wf))}
    if want_dbias:
        out["dbias"] = np.empty(F_out)
        out["dbias_abs"] = np.empty(F_out)
    a = _BwdArgs(n, _ptr(col_ptr), _ptr(row_idx), _ptr(Xv), F, EDGE_OPS[edge_op], ACTS[act], _ptr(w), _ptr(A),
                 _ptr(Wv), _ptr(bv), _ptr(Ws), F_out, _ptr(dYv), None, None, None, None, None, _ptr(out.get("dbias")), None,
                 None, _ptr(out.get("dbias_abs")))
    rc = lib().saga_oracle_backward_sample(ctypes.byref(a), len(ul), _ptr(ul), _ptr(out["dX"]), _ptr(out["dX_abs"]),
                                           len(wf), _ptr(wf), _ptr(wo), _ptr(out["dW"]), _ptr(out["dW_abs"]))
    if rc != 0:
        raise ValueError("saga_oracle_backward_sample rejected its arguments")
    return out


def gated_backward(col_ptr, row_idx, X, A, dY, W, W_gate, b_gate=None, W_msg=None, bias=None, act="none", W_self=None, agg="sum"):
    """Gradients of one gated layer (Example 2.1 / Figure 2, Section 2.2's backward stages).

    agg "sum": A is the forward Gather output (fp64). agg "max": A is not read (pass None); the Gather output is
    recomputed and returned as "A", and only the edges that supplied a maximum carry gradient. Returns fp64 arrays dX,
    dW, dbias, dW_gate (F x 2F), db_gate, dW_msg (with respect to an explicit identity when W_msg is None), dW_self
    when W_self is given, and their *_abs error scales."""
    col_ptr = np.ascontiguousarray(np.asarray(col_ptr, dtype=np.int64))
    row_idx = np.ascontiguousarray(np.asarray(row_idx, dtype=np.int32))
    Xv, Wv, dYv, Wg = _f32(X), _f32(W), _f32(dY), _f32(W_gate)
    n, F = Xv.shape
    F_out = Wv.shape[1]
    if agg == "sum":
        A = np.ascontiguousarray(np.asarray(A, dtype=np.float64))
        assert A.shape == (n, F)
    else:
        assert agg == "max" and A is None
    assert Wv.shape == (F, F_out) and dYv.shape == (n, F_out) and Wg.shape == (F, 2 * F)
    bg, Wm, bv, Ws = _f32(b_gate), _f32(W_msg), _f32(bias), _f32(W_self)
    assert Wm is None or Wm.shape == (F, F)
    out = {"dX": np.empty((n, F)), "dX_abs": np.empty((n, F)), "dW": np.empty((F, F_out)), "dW_abs": np.empty((F, F_out)),
           "dbias": np.empty(F_out), "dbias_abs": np.empty(F_out), "dW_gate": np.empty((F, 2 * F)), "dW_gate_abs": np.empty((F, 2 * F)),
           "db_gate": np.empty(F), "db_gate_abs": np.empty(F), "dW_msg": np.empty((F, F)), "dW_msg_abs": np.empty((F, F))}
    if Ws is not None:
        assert Ws.shape == (F, F_out)
        out.update(dW_self=np.empty((F, F_out)), dW_self_abs=np.empty((F, F_out)))
    if agg == "max":
        out["A"] = np.empty((n, F))
    a = _GBwdArgs(n, _ptr(col_ptr), _ptr(row_idx), _ptr(Xv), F, _ptr(Wg), _ptr(bg), _ptr(Wm), _ptr(A), _ptr(Wv), _ptr(bv),
                  F_out, ACTS[act], AGGS[agg], _ptr(dYv), _ptr(out["dX"]), _ptr(out["dX_abs"]), _ptr(out["dW"]), _ptr(out["dW_abs"]),
                  _ptr(out["dbias"]), _ptr(out["dW_gate"]), _ptr(out["dW_gate_abs"]), _ptr(out["db_gate"]),
                  _ptr(out["db_gate_abs"]), _ptr(out["dW_msg"]), _ptr(out["dW_msg_abs"]),
                  _ptr(Ws), _ptr(out.get("dW_self")), _ptr(out.get("dW_self_abs")), _ptr(out["dbias_abs"]), _ptr(out.get("A")))
    rc = lib().saga_oracle_gated_backward(ctypes.byref(a))
    if rc != 0:
        raise ValueError("saga_oracle_gated_backward rejected its arguments")
    return out


def gated_backward_sample(col_ptr, row_idx, X, dZ, W, W_gate, ulist, b_gate=None, W_msg=None):
    """gated_backward's definitions (no activation: dZ is given) evaluated only for the rows dX[ulist], from the in- and
    out-edges of those vertices, for graphs too large to do whole. Returns dict dX, dX_abs (len(ulist) x F)."""
    col_ptr = np.ascontiguousarray(np.asarray(col_ptr, dtype=np.int64))
    row_idx = np.ascontiguousarray(np.asarray(row_idx, dtype=np.int32))
    Xv, Wv, dZv, Wg = _f32(X), _f32(W), _f32(dZ), _f32(W_gate)
    n, F = Xv.shape
    F_out = Wv.shape[1]
    assert Wv.shape == (F, F_out) and dZv.shape == (n, F_out) and Wg.shape == (F, 2 * F)
    bg, Wm = _f32(b_gate), _f32(W_msg)
    ul = np.ascontiguousarray(np.asarray(ulist, dtype=np.int64))
    assert len(set(ul.tolist())) == len(ul)
    out = {"dX": np.zeros((len(ul), F)), "dX_abs": np.zeros((len(ul), F))}
    a = _GBwdArgs(n, _ptr(col_ptr), _ptr(row_idx), _ptr(Xv), F, _ptr(Wg), _ptr(bg), _ptr(Wm), None, _ptr(Wv), None,
                  F_out, ACTS["none"], AGGS["sum"], _ptr(dZv), *([None] * 11), None, None, None, None, None)
    rc = lib().saga_oracle_gated_backward_sample(ctypes.byref(a), len(ul), _ptr(ul), _ptr(out["dX"]), _ptr(out["dX_abs"]))
    if rc != 0:
        raise ValueError("saga_oracle_gated_backward_sample rejected its arguments")
    return out


def max_backward(col_ptr, row_idx, X, dY, W, edge_op="copy", edge_weight=None, W_pool=None, b_pool=None, bias=None, act="none",
                 W_self=None):
    """Gradients of one max-accumulator layer (COPY, MUL_WEIGHT or POOL messages; Figure 11 and Section 2.2's backward
    stages). Returns fp64 arrays A (the recomputed Gather output), dX, dW, dbias and, for POOL, dW_pool, db_pool, with
    W_self dW_self, plus *_abs error scales."""
    col_ptr = np.ascontiguousarray(np.asarray(col_ptr, dtype=np.int64))
    row_idx = np.ascontiguousarray(np.asarray(row_idx, dtype=np.int32))
    Xv, Wv, dYv = _f32(X), _f32(W), _f32(dY)
    n, F = Xv.shape
    Wp, bp, w, bv, Ws = _f32(W_pool), _f32(b_pool), _f32(edge_weight), _f32(bias), _f32(W_self)
    Fp = Wp.shape[0] if edge_op == "pool" else 0
    Fm = Fp if edge_op == "pool" else F
    F_out = Wv.shape[1]
    assert Wv.shape == (Fm, F_out) and dYv.shape == (n, F_out)
    out = {"A": np.empty((n, Fm)), "dX": np.empty((n, F)), "dX_abs": np.empty((n, F)), "dW": np.empty((Fm, F_out)),
           "dW_abs": np.empty((Fm, F_out)), "dbias": np.empty(F_out), "dbias_abs": np.empty(F_out)}
    if Ws is not None:
        assert Ws.shape == (F, F_out)
        out.update(dW_self=np.empty((F, F_out)), dW_self_abs=np.empty((F, F_out)))
    if edge_op == "pool":
        assert Wp.shape == (Fp, F)
        out.update(dW_pool=np.empty((Fp, F)), dW_pool_abs=np.empty((Fp, F)), db_pool=np.empty(Fp), db_pool_abs=np.empty(Fp))
    a = _MBwdArgs(n, _ptr(col_ptr), _ptr(row_idx), _ptr(Xv), F, EDGE_OPS[edge_op], ACTS[act], _ptr(w), _ptr(Wp), _ptr(bp), Fp,
                  _ptr(Wv), _ptr(bv), F_out, _ptr(dYv), _ptr(out["A"]), _ptr(out["dX"]), _ptr(out["dX_abs"]), _ptr(out["dW"]),
                  _ptr(out["dW_abs"]), _ptr(out["dbias"]), _ptr(out.get("dW_pool")), _ptr(out.get("dW_pool_abs")),
                  _ptr(out.get("db_pool")), _ptr(out.get("db_pool_abs")),
                  _ptr(Ws), _ptr(out.get("dW_self")), _ptr(out.get("dW_self_abs")), _ptr(out["dbias_abs"]))
    rc = lib().saga_oracle_max_backward(ctypes.byref(a))
    if rc != 0:
        raise ValueError("saga_oracle_max_backward rejected its arguments")
    return out


def max_backward_sample(col_ptr, row_idx, X, dY, W, ulist, edge_op="copy", edge_weight=None, W_pool=None, b_pool=None, bias=None,
                        act="none", W_self=None):
    """max_backward's definitions evaluated only for the rows dX[ulist] (distinct source vertices), from those vertices'
    out-edges and the whole columns of the destinations they reach, for graphs too large to do whole. Returns dict dX,
    dX_abs (len(ulist) x F)."""
    col_ptr = np.ascontiguousarray(np.asarray(col_ptr, dtype=np.int64))
    row_idx = np.ascontiguousarray(np.asarray(row_idx, dtype=np.int32))
    Xv, Wv, dYv = _f32(X), _f32(W), _f32(dY)
    n, F = Xv.shape
    Wp, bp, w, bv, Ws = _f32(W_pool), _f32(b_pool), _f32(edge_weight), _f32(bias), _f32(W_self)
    Fp = Wp.shape[0] if edge_op == "pool" else 0
    Fm = Fp if edge_op == "pool" else F
    F_out = Wv.shape[1]
    assert Wv.shape == (Fm, F_out) and dYv.shape == (n, F_out)
    assert Ws is None or Ws.shape == (F, F_out)
    assert edge_op != "pool" or Wp.shape == (Fp, F)
    ul = np.ascontiguousarray(np.asarray(ulist, dtype=np.int64))
    assert len(set(ul.tolist())) == len(ul)
    out = {"dX": np.zeros((len(ul), F)), "dX_abs": np.zeros((len(ul), F))}
    a = _MBwdArgs(n, _ptr(col_ptr), _ptr(row_idx), _ptr(Xv), F, EDGE_OPS[edge_op], ACTS[act], _ptr(w), _ptr(Wp), _ptr(bp), Fp,
                  _ptr(Wv), _ptr(bv), F_out, _ptr(dYv), None, None, None, None, None, None, None, None, None, None,
                  _ptr(Ws), None, None, None)
    rc = lib().saga_oracle_max_backward_sample(ctypes.byref(a), len(ul), _ptr(ul), _ptr(out["dX"]), _ptr(out["dX_abs"]))
    if rc != 0:
        raise ValueError("saga_oracle_max_backward_sample rejected its arguments")
    return out

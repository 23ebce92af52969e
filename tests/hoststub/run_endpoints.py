"""The per-vertex products of gated and pooled layers taken over the graph's endpoint lists (vertices with out-edges, vertices
with in-edges) on the CPU stand-in: a directed power-law graph with many vertices of neither kind, rows of 128 features (the
width at which the product kernel takes lists), forwards and backwards against the oracle, and the call that must not
allocate after an ordinary one.

  python tests/hoststub/run_endpoints.py <library>"""
import ctypes
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
TESTS = os.path.dirname(HERE)
sys.path[:0] = [os.path.dirname(TESTS), TESTS, HERE]

import numpy as np
import torch

import oracle
import saga_inputs as si
from helpers import TOL_F32, assert_sum_close
from stub_binding import StubContext, dev


def main():
    lib = sys.argv[1]
    F, Fo = 128, 8
    wl = si.workload(4, scale=11, f_in=F, f_out=Fo)
    g = wl.graph
    n = g.n
    cp, ri = g.col_ptr.numpy(), g.row_idx.numpy()
    indeg, outdeg = np.diff(cp), np.bincount(ri, minlength=n)
    assert (indeg == 0).sum() > n // 8 and (outdeg == 0).sum() > n // 8 and (indeg > 0).sum() >= 64 and (outdeg > 0).sum() >= 64
    okw = dict(W_gate=wl.W_gate.numpy(), b_gate=wl.b_gate.numpy(), W_msg=wl.W_msg.numpy())
    bias = si.uniform_pm(Fo, 0.3, 5)
    dY = si.normal_features(n, Fo, 99)
    fwd = oracle.layer(cp, ri, wl.X.numpy(), "gated", W=wl.W.numpy(), bias=bias.numpy(), act="relu", **okw)
    bwd = oracle.gated_backward(cp, ri, wl.X.numpy(), fwd["A"], dY.numpy(), wl.W.numpy(), bias=bias.numpy(), act="relu", **okw)
    Wp, bp = si.glorot_uniform(F, F, 7).T.contiguous(), si.uniform_pm(F, 0.2, 8)
    pool = oracle.layer(cp, ri, wl.X.numpy(), "pool", agg="sum", W=wl.W.numpy(), act="none", W_pool=Wp.numpy(), b_pool=bp.numpy())
    for mode in (0, 2):
        ctx = StubContext(lib)
        ctx.lib.stub_row_list_launches.restype = ctypes.c_int64
        ctx.set_mode(mode, 5)
        h = ctx.graph_create_csc(n, dev(g.col_ptr), dev(g.row_idx))
        X, W, b = dev(wl.X), dev(wl.W), dev(bias)
        gate = dict(edge_op="gated", W_gate=dev(wl.W_gate), b_gate=dev(wl.b_gate), W_msg=dev(wl.W_msg))
        before = ctx.lib.stub_row_list_launches()
        Y, A = dev(torch.full((n, Fo), float("nan"))), dev(torch.full((n, F), float("nan")))
        ctx.layer_forward(h, X, Y, W=W, bias=b, act="relu", accum_out=A, **gate)
        ctx.synchronize()
        assert ctx.lib.stub_row_list_launches() == before + 2, "the gated products did not go over the two lists"
        assert_sum_close(Y.t.numpy(), fwd["Y"], fwd["Y_abs"], TOL_F32, f"gated layer, mode {mode}")
        Y2 = dev(torch.full((n, Fo), float("nan")))
        ctx.layer_forward(h, X, Y2, W=W, bias=b, act="relu", no_alloc=True, **gate)
        ctx.synchronize()
        assert ctx.lib.stub_row_list_launches() == before + 4
        assert torch.equal(Y2.t, Y.t), "the call that must not allocate gives other bits"
        full = lambda *s: dev(torch.full(s, float("nan")))
        out = dict(dW=full(F, Fo), dX=full(n, F), dbias=full(Fo), dW_gate=full(F, 2 * F), db_gate=full(F), dW_msg=full(F, F))
        ctx.layer_backward(h, A, dev(dY), W, out["dW"], X=X, Y=Y, act="relu", bias=b, dX=out["dX"], dbias=out["dbias"],
                           dW_gate=out["dW_gate"], db_gate=out["db_gate"], dW_msg=out["dW_msg"], **gate)
        ctx.synchronize()
        assert ctx.lib.stub_row_list_launches() == before + 6
        for name, t in out.items():
            assert_sum_close(t.t.numpy(), bwd[name], np.maximum(bwd[name + "_abs"], 1e-30), TOL_F32, f"gated backward {name}, mode {mode}")
        Yp = dev(torch.full((n, Fo), float("nan")))
        ctx.layer_forward(h, X, Yp, edge_op="pool", agg="sum", W=W, act="none", W_pool=dev(Wp), b_pool=dev(bp))
        ctx.synchronize()
        assert ctx.lib.stub_row_list_launches() == before + 7, "the pooled rows did not go over the source list"
        assert_sum_close(Yp.t.numpy(), pool["Y"], pool["Y_abs"], TOL_F32, f"pooled layer, mode {mode}")
        h.destroy()
        ctx.destroy()
    # a graph in which every vertex is both: no list is used
    sym = si.workload(1)
    ctx = StubContext(lib)
    ctx.lib.stub_row_list_launches.restype = ctypes.c_int64
    n1 = sym.graph.n
    X1 = si.normal_features(n1, F, 3)
    W1 = si.glorot_uniform(F, Fo, 4)
    Wg1, bg1 = si.glorot_uniform(2 * F, F, 5).T.contiguous(), si.uniform_pm(F, 0.1, 6)
    ref = oracle.layer(sym.graph.col_ptr.numpy(), sym.graph.row_idx.numpy(), X1.numpy(), "gated", W=W1.numpy(), act="none",
                       W_gate=Wg1.numpy(), b_gate=bg1.numpy())
    h = ctx.graph_create_csc(n1, dev(sym.graph.col_ptr), dev(sym.graph.row_idx))
    before = ctx.lib.stub_row_list_launches()
    Y1 = dev(torch.full((n1, Fo), float("nan")))
    ctx.layer_forward(h, dev(X1), Y1, edge_op="gated", W_gate=dev(Wg1), b_gate=dev(bg1), W=dev(W1), act="none")
    ctx.synchronize()
    assert ctx.lib.stub_row_list_launches() == before
    assert_sum_close(Y1.t.numpy(), ref["Y"], ref["Y_abs"], TOL_F32, "gated layer on a graph with self-loops")
    h.destroy()
    ctx.destroy()
    print("ok: products over endpoint lists match the oracle", flush=True)


if __name__ == "__main__":
    main()

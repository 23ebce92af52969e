"""Max over gated messages from host memory, forwards (with the Gather output kept through accum_out) and backwards, on
the CPU stand-in: the chunk schedules with a third row per vertex (the kept maxima beside [Pd | gradient of accum]),
against the oracle, for several tilings and in the three legal orders of the deferred stream operations.

  python tests/hoststub/run_gated_max.py <library>"""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
TESTS = os.path.dirname(HERE)
sys.path[:0] = [os.path.dirname(TESTS), TESTS, HERE]

import numpy as np
import torch

import oracle
import saga_inputs as si
from helpers import TOL_F32, assert_sum_close, coarse_gated_workload
from stub_binding import StubContext, dev


def main():
    lib = sys.argv[1]
    checked = 0
    for F, Fo, act, with_b, with_msg, with_self, Q, P, mode in ((8, 6, "relu", True, True, False, 2, 3, 0),
                                                               (12, 4, "none", False, False, False, 1, 4, 1),
                                                               (16, 8, "relu", True, True, True, 3, 2, 2),
                                                               (5, 3, "relu", True, False, False, 2, 2, 2)):
        wl = coarse_gated_workload(8, F, Fo)
        g = wl.graph
        n = g.n
        cp, ri = g.col_ptr.numpy(), g.row_idx.numpy()
        Ws = si.glorot_uniform(F, Fo, 41) if with_self else None
        bg = wl.b_gate if with_b else None
        Wm = wl.W_msg if with_msg else None
        dY = si.normal_features(n, Fo, 99)
        Y_in = si.normal_features(n, Fo, 98)
        slope = {"none": torch.ones_like(Y_in.double()), "relu": (Y_in > 0).double()}[act]
        dZ = (dY.double() * slope).float()
        opt = lambda t: None if t is None else t.numpy()
        bwd = oracle.gated_backward(cp, ri, wl.X.numpy(), None, dZ.numpy(), wl.W.numpy(), act="none", agg="max",
                                    W_gate=wl.W_gate.numpy(), b_gate=opt(bg), W_msg=opt(Wm), W_self=opt(Ws))
        ctx = StubContext(lib)
        ctx.set_mode(mode, 17)
        for name, val in (("dst_intervals", Q), ("src_intervals", P), ("bwd_tile_rows", 100), ("cut_degree", 16), ("split", 16)):
            ctx.set_option(name, val)
        h = ctx.graph_create_csc(n, g.col_ptr, g.row_idx)
        gate = dict(edge_op="gated", agg="max", W_gate=dev(wl.W_gate), b_gate=dev(bg), W_msg=dev(Wm), W_self=dev(Ws))
        Wd = dev(wl.W)
        X_h = wl.X.clone()
        A_h = torch.full((n, F + 3), float("nan"))[:, :F]           # rows further apart than they are wide
        Yf = torch.full((n, Fo), float("nan"))
        ctx.layer_forward(h, X_h, Yf, W=Wd, act="none", accum_out=A_h, **gate)
        what = f"gated max {F}->{Fo} {act} {Q}x{P} mode {mode}"
        assert_sum_close(A_h.numpy(), bwd["A"], np.maximum(np.abs(bwd["A"]), 1e-30), TOL_F32, what + " A")
        full = lambda *s: dev(torch.full(s, float("nan")))
        out = dict(dW=full(F, Fo), dbias=full(Fo), dW_gate=full(F, 2 * F), db_gate=full(F) if with_b else None,
                   dW_msg=full(F, F) if with_msg else None, dW_self=full(F, Fo) if with_self else None)
        dX_h = torch.full((n, F), float("nan"))
        for rep in range(2):
            ctx.layer_backward(h, A_h, dY, Wd, out["dW"], X=X_h, Y=Y_in, act=act, dX=dX_h, dbias=out["dbias"], dW_gate=out["dW_gate"],
                               db_gate=out["db_gate"], dW_msg=out["dW_msg"], dW_self=out["dW_self"], **gate)
            for name, t in out.items():
                if t is not None:
                    assert np.abs(bwd[name]).max() > 0, name
                    assert_sum_close(t.t.numpy(), bwd[name], np.maximum(bwd[name + "_abs"], 1e-30), TOL_F32, f"{what} call {rep} {name}")
            assert_sum_close(dX_h.numpy(), bwd["dX"], bwd["dX_abs"], TOL_F32, f"{what} call {rep} dX")
        h.destroy()
        ctx.destroy()
        checked += 1
    print(f"ok: {checked} layers of max over gated messages match the oracle forwards and backwards", flush=True)


if __name__ == "__main__":
    main()

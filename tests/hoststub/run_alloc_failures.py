"""Error paths of the streamed calls on the CPU stand-in of the HIP runtime: the n-th device or pinned allocation of a
call fails, for n = 1, 2, ... until a call gets through. Every failed call must come back with an error status (never
a crash, never a half-built tiling that a later call trips over), and the same call repeated without the failure must
give the oracle's result.

  python tests/hoststub/run_alloc_failures.py <library>"""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
TESTS = os.path.dirname(HERE)
sys.path[:0] = [os.path.dirname(TESTS), TESTS, HERE]

import numpy as np
import torch

import oracle
import saga_inputs as si
from helpers import assert_sum_close
from paper_1810_08403_amd import binding as B
from stub_binding import StubContext, dev


def main():
    lib = sys.argv[1]
    rng = np.random.default_rng(5)
    n, m = 300, 2500
    g = si.csc_from_lists(n, sorted(set(zip(rng.integers(n, size=m).tolist(), rng.integers(n, size=m).tolist()))))
    t = lambda *shape, s=1.0: torch.as_tensor((rng.standard_normal(shape) * s).astype(np.float32))
    cp, ri = g.col_ptr.numpy(), g.row_idx.numpy()
    failures = 0
    for op, F, Fo in (("mul_weight", 16, 8), ("gated", 8, 4), ("pool", 12, 4)):
        X, W, bias, w = t(n, F), t(F, Fo, s=0.3), t(Fo, s=0.2), t(g.nnz)
        kw, okw = {}, {}
        if op == "gated":
            Wg, bg = t(F, 2 * F, s=0.3), t(F, s=0.2)
            kw, okw = dict(W_gate=dev(Wg), b_gate=dev(bg)), dict(W_gate=Wg.numpy(), b_gate=bg.numpy())
        if op == "pool":
            Wp, bp = t(F, F, s=0.3), t(F, s=0.2)
            kw, okw = dict(W_pool=dev(Wp), b_pool=dev(bp)), dict(W_pool=Wp.numpy(), b_pool=bp.numpy())
        ref = oracle.layer(cp, ri, X.numpy(), op, w.numpy() if op == "mul_weight" else None, agg="sum", W=W.numpy(), bias=bias.numpy(),
                           act="relu", **okw)
        for mode in (0, 1, 2):
            ctx = StubContext(lib)
            ctx.set_mode(mode, 3)
            ctx.set_option("dst_intervals", 2)
            ctx.set_option("src_intervals", 3)
            h = ctx.graph_create_csc(n, g.col_ptr, g.row_idx)
            h.set_edge_data(w)
            nth = 1
            while True:
                Y = torch.full((n, Fo), float("nan"))
                ctx.lib.stub_fail_allocation(nth)
                try:
                    ctx.layer_forward(h, X.clone(), Y, edge_op=op, agg="sum", W=dev(W), bias=dev(bias), act="relu", **kw)
                    ok = True
                except B.SagaError as e:
                    assert e.status in (5, 6), f"{op} mode {mode} allocation {nth}: status {e.status}"
                    ok = False
                    failures += 1
                ctx.lib.stub_fail_allocation(0)
                if ok:
                    assert_sum_close(Y.numpy(), ref["Y"], ref["Y_abs"], 1e-4, f"{op} mode {mode} after {nth - 1} failed calls")
                    break
                nth += 1
                assert nth < 200
            if op == "mul_weight":         # and the backward pass, whose first call also builds the edge order by source
                dY = t(n, Fo)
                bwd = oracle.layer_backward(cp, ri, X.numpy(), ref["A"], dY.numpy(), W.numpy(), op, w.numpy(), bias=bias.numpy(), act="relu")
                f32 = lambda a: torch.as_tensor(np.ascontiguousarray(a), dtype=torch.float32).clone()
                nth = 1
                while True:
                    dX, dW, db = torch.full((n, F), float("nan")), dev(torch.full((F, Fo), float("nan"))), dev(torch.full((Fo,), float("nan")))
                    ctx.lib.stub_fail_allocation(nth)
                    try:
                        ctx.layer_backward(h, f32(ref["A"]), dY.clone(), dev(W), dW, X=X.clone(), Y=f32(ref["Y"]), edge_op=op, bias=dev(bias),
                                           act="relu", dX=dX, dbias=db)
                        ok = True
                    except B.SagaError as e:
                        assert e.status in (5, 6), f"backward mode {mode} allocation {nth}: status {e.status}"
                        ok = False
                        failures += 1
                    ctx.lib.stub_fail_allocation(0)
                    if ok:
                        assert_sum_close(dX.numpy(), bwd["dX"], bwd["dX_abs"], 1e-4, f"backward mode {mode} dX after {nth - 1} failed calls")
                        assert_sum_close(dW.t.numpy(), bwd["dW"], bwd["dW_abs"], 1e-4, f"backward mode {mode} dW")
                        break
                    nth += 1
                    assert nth < 200
            h.destroy()
            ctx.destroy()
            live = ctx.live_counts()
            assert live["allocations"] == 0 and live["streams"] == 0 and live["events"] == 0, f"left behind {live}"
    print(f"ok: {failures} calls failed on purpose, every one with an error status", flush=True)


if __name__ == "__main__":
    main()

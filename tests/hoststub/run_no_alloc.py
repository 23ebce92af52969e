"""saga_layer_forward_noalloc on the CPU stand-in of the HIP runtime: the call must reach no allocator (the stand-in
counts hipMalloc / hipFree / hipHostMalloc / hipHostFree and stream and event creations), must give the bits of the
ordinary call, must refuse a row width whose work list has not been built and a layer that does not fit the scratch array.

  python tests/hoststub/run_no_alloc.py <library>"""
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
TESTS = os.path.dirname(HERE)
sys.path[:0] = [os.path.dirname(TESTS), TESTS, HERE]

import numpy as np
import torch

import saga_inputs as si
from paper_1810_08403_amd import binding as B
from stub_binding import StubContext, dev


def main():
    lib = sys.argv[1]
    rng = np.random.default_rng(11)
    t = lambda *shape, s=1.0: torch.as_tensor((rng.standard_normal(shape) * s).astype(np.float32))
    ctx = StubContext(lib)
    ctx.set_mode(2, 5)
    checked = 0
    for n, m, hub in ((700, 9000, True), (150, 900, False)):          # the second graph is smaller: stale scratch contents must not show
        edges = set(zip(rng.integers(n, size=m).tolist(), rng.integers(n, size=m).tolist()))
        if hub:
            edges |= {(u, 3) for u in range(n)}                        # a column that is cut into pieces: partial rows in the scratch
        g = si.csc_from_lists(n, sorted(edges))
        h = ctx.graph_create_csc(n, dev(g.col_ptr), dev(g.row_idx))
        w = t(g.nnz)
        for op, F, Fo, agg in (("mul_weight", 24, 8, "sum"), ("copy", 24, 5, "max"), ("gated", 8, 4, "sum"), ("pool", 12, 4, "max")):
            X, W, bias = t(n, F), t(F, Fo, s=0.3), t(Fo, s=0.2)
            kw = {}
            if op == "mul_weight":
                kw["edge_weight"] = dev(w)
            if op == "gated":
                kw.update(W_gate=dev(t(F, 2 * F, s=0.3)), b_gate=dev(t(F, s=0.2)))
            if op == "pool":
                kw.update(W_pool=dev(t(F, F, s=0.3)), b_pool=dev(t(F, s=0.2)))
            args = dict(edge_op=op, agg=agg, W=dev(W), bias=dev(bias), act="relu", **kw)
            Y0, A0 = dev(torch.full((n, Fo), float("nan"))), dev(torch.full((n, F), float("nan")))
            Y1, A1 = dev(torch.full((n, Fo), float("nan"))), dev(torch.full((n, F), float("nan")))
            ctx.layer_forward(h, dev(X), Y0, accum_out=A0, **args)                # builds the work list for this row width
            before = ctx.lib.stub_allocator_calls()
            ctx.layer_forward(h, dev(X), Y1, accum_out=A1, no_alloc=True, **args)
            assert ctx.lib.stub_allocator_calls() == before, f"{op}: the no-allocation call reached an allocator"
            ctx.synchronize()                                                       # resident calls return after enqueueing
            assert torch.equal(Y0.t, Y1.t) and torch.equal(A0.t, A1.t), f"{op} n={n}: results differ from the ordinary call"
            assert not torch.isnan(Y1.t).any()
            checked += 1
        # a row width nobody has run yet: refused, not built
        try:
            ctx.layer_forward(h, dev(t(n, 200)), dev(torch.empty(n, 200)), edge_op="copy", no_alloc=True)
            raise AssertionError("a missing work list was accepted")
        except B.SagaError as e:
            assert e.status == 3, e
        h.destroy()
    # a layer that does not fit the 64 MiB: refused with SAGA_ERR_BUDGET, and the next call still works
    n, F = 9000, 2048
    g = si.csc_from_lists(n, [(i, (i * 7) % n) for i in range(n)])
    h = ctx.graph_create_csc(n, dev(g.col_ptr), dev(g.row_idx))
    X, W = torch.zeros(n, F), torch.zeros(F, 4)
    Y = dev(torch.empty(n, 4))
    ctx.layer_forward(h, dev(X), Y, edge_op="copy", W=dev(W))
    try:
        ctx.layer_forward(h, dev(X), Y, edge_op="copy", W=dev(W), no_alloc=True)
        raise AssertionError("a layer beyond the scratch size was accepted")
    except B.SagaError as e:
        assert e.status == 4, e
    ctx.layer_forward(h, dev(X), Y, edge_op="copy", W=dev(W))
    h.destroy()
    ctx.destroy()
    print(f"ok: {checked} layers, no allocator reached", flush=True)


if __name__ == "__main__":
    main()

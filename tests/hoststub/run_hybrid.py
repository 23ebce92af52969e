"""The dense-block path of bf16 sum layers (well-filled blocks of the adjacency matrix as dense products, the rest as a
remainder for the sparse kernel) on the CPU stand-in: the host-side plan (ranks, blocks, chunks, partial-row slots, the
remainder CSC, weight packing) against the oracle, for several thresholds, chunk lengths and graphs.

  python tests/hoststub/run_hybrid.py <library>"""
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
from stub_binding import StubContext, dev


def main():
    lib = sys.argv[1]
    rng = np.random.default_rng(31)
    t = lambda *shape, s=1.0: torch.as_tensor((rng.standard_normal(shape) * s).astype(np.float32))
    checked = 0
    for scale, ef, sym in ((9, 40, True), (10, 12, False), (8, 100, True)):
        src, dst = si.rmat_edges(scale, ef << scale, 900 + scale)
        g = si.build_csc(1 << scale, src, dst, symmetrise=sym, self_loops=sym)
        n = g.n
        cp, ri = g.col_ptr.numpy(), g.row_idx.numpy()
        for F, Fo, op, opts in ((128, 16, "mul_weight", dict(dense_min_edges=8, dense_tile_gain=0, dense_chunk=3)),
                                (256, 8, "copy", dict(dense_min_edges=24, dense_tile_gain=64)),
                                (128, 0, "mul_weight", dict(dense_min_edges=4, dense_tile_gain=0, dense_chunk=1, split=16, cut_degree=16)),
                                (128, 8, "mul_weight", dict())):
            X = si.round_to_bf16(t(n, F))
            w = t(g.nnz)
            W = si.round_to_bf16(t(F, Fo, s=0.3)) if Fo else None
            ref = oracle.layer(cp, ri, X.numpy(), op, w.numpy() if op == "mul_weight" else None, agg="sum",
                               W=None if W is None else W.numpy(), act="relu" if Fo else "none")
            for mode, attach in ((0, True), (2, False)):
                ctx = StubContext(lib)
                ctx.set_mode(mode, 9)
                for k, v in opts.items():
                    ctx.set_option(k, v)
                h = ctx.graph_create_csc(n, dev(g.col_ptr), dev(g.row_idx))
                kw = {}
                if op == "mul_weight":
                    if attach:
                        h.set_edge_data(dev(w))
                    else:
                        kw["edge_weight"] = dev(w)
                if W is not None:
                    kw.update(W=dev(W.to(torch.bfloat16)), act="relu")
                Xb = dev(X.to(torch.bfloat16))        # kept alive: resident calls return after enqueueing
                Y = dev(torch.full((n, Fo or F), float("nan"), dtype=torch.bfloat16))
                A = dev(torch.full((n, F), float("nan")))
                ctx.set_profiling(True)
                for rep in range(2):     # the second call finds the plan (and attached weights already packed)
                    ctx.reset_timings()
                    ctx.layer_forward(h, Xb, Y, edge_op=op, agg="sum", accum_out=A, **kw)
                    ctx.synchronize()
                    if opts:             # thresholds chosen so that these graphs do have dense blocks: two propagation launches
                        assert ctx.get_timings()["n_gather_launches"] == 2, "the dense-block path was not taken"
                    what = f"rmat {scale} F={F}->{Fo} {op} {opts} mode {mode} attach={attach} call {rep}"
                    assert_sum_close(A.t.numpy(), ref["A"], ref["A_abs"], 2e-5, what + " Gather")
                    ykey = "Y" if Fo else "A"     # without ApplyVertex the layer's output is the Gather output, rounded to bf16
                    assert_sum_close(Y.t.float().numpy(), ref[ykey], ref[ykey + "_abs"], 1e-2, what + " layer")
                if op == "mul_weight" and attach:   # new edge data on the handle: packed again at the next call
                    w2 = t(g.nnz)
                    w2d = dev(w2)
                    h.set_edge_data(w2d)
                    ctx.layer_forward(h, Xb, Y, edge_op=op, agg="sum", accum_out=A, **kw)
                    ctx.synchronize()
                    ref2 = oracle.layer(cp, ri, X.numpy(), op, w2.numpy(), agg="sum", W=None if W is None else W.numpy(), act="relu" if Fo else "none")
                    assert_sum_close(A.t.numpy(), ref2["A"], ref2["A_abs"], 2e-5, what + " Gather after new edge data")
                # and the same bits as without the dense blocks, up to the two-part weights: compare through the oracle only
                h.destroy()
                ctx.destroy()
                checked += 1
    print(f"ok: {checked} dense-block layers match the oracle", flush=True)


if __name__ == "__main__":
    main()

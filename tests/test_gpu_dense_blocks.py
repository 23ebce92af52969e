"""The dense-block path of bf16 sum layers (well-filled 64 x 32 blocks of the degree-ranked adjacency matrix on the matrix
cores, the remainder through the sparse propagation kernel; the fused Scatter-ApplyEdge-Gather of Sections 3.2 / 3.3)
against the oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import saga_inputs as si
from helpers import TOL_BF16, assert_sum_close

pytestmark = pytest.mark.gpu


def _rmat(scale, ef, sym):
    src, dst = si.rmat_edges(scale, ef << scale, 900 + scale)
    return si.build_csc(1 << scale, src, dst, symmetrise=sym, self_loops=sym)


@pytest.mark.parametrize("scale,ef,sym", [(9, 40, True), (11, 24, False), (8, 100, True)])
@pytest.mark.parametrize("F,Fo,op,opts", [(128, 16, "mul_weight", dict(dense_min_edges=8, dense_tile_gain=0, dense_chunk=3)),
                                          (256, 8, "copy", dict(dense_min_edges=24, dense_tile_gain=64)),
                                          (640, 0, "mul_weight", dict(dense_min_edges=4, dense_tile_gain=0, dense_chunk=1, split=16, cut_degree=16)),
                                          (512, 64, "mul_weight", dict())])
def test_dense_blocks_match_the_oracle(scale, ef, sym, F, Fo, op, opts):
    import paper_1810_08403_amd as saga
    g = _rmat(scale, ef, sym)
    n = g.n
    rng = np.random.default_rng(41)
    t = lambda *shape, s=1.0: torch.as_tensor((rng.standard_normal(shape) * s).astype(np.float32))
    X, w = si.round_to_bf16(t(n, F)), t(g.nnz)
    W = si.round_to_bf16(t(F, Fo, s=0.3)) if Fo else None
    cp, ri = g.col_ptr.numpy(), g.row_idx.numpy()
    ref = oracle.layer(cp, ri, X.numpy(), op, w.numpy() if op == "mul_weight" else None, agg="sum", W=None if W is None else W.numpy(),
                       act="relu" if Fo else "none")
    ctx = saga.Context(0)
    for k, v in opts.items():
        ctx.set_option(k, v)
    h = ctx.graph_create_csc(n, g.col_ptr.cuda(), g.row_idx.cuda())
    kw = {}
    if op == "mul_weight":
        h.set_edge_data(w.cuda())
    if W is not None:
        kw.update(W=W.cuda().to(torch.bfloat16), act="relu")
    Xd = X.cuda().to(torch.bfloat16)
    Y = torch.full((n, Fo or F), float("nan"), device="cuda", dtype=torch.bfloat16)
    A = torch.full((n, F), float("nan"), device="cuda")
    ctx.set_profiling(True)
    outs = []
    for rep in range(2):
        ctx.reset_timings()
        ctx.layer_forward(h, Xd, Y, edge_op=op, agg="sum", accum_out=A, **kw)
        torch.cuda.synchronize()
        if opts:
            assert ctx.get_timings()["n_gather_launches"] == 2, "the dense-block path was not taken"
        what = f"rmat {scale} F={F}->{Fo} {op} {opts} call {rep}"
        # the Gather output is fp32 sums of exact bf16 products with two-part bf16 weights (2^-17 relative): well inside the bf16 bar
        assert_sum_close(A.cpu().numpy(), ref["A"], ref["A_abs"], 2e-5, what + " Gather")
        ykey = "Y" if Fo else "A"
        assert_sum_close(Y.float().cpu().numpy(), ref[ykey], ref[ykey + "_abs"], TOL_BF16, what + " layer")
        outs.append((A.clone(), Y.clone()))
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1]), "not reproducible run to run"
    if op == "mul_weight":      # weights passed with the call are packed per call; new attached data are packed at the next call
        w2 = t(g.nnz)
        ref2 = oracle.layer(cp, ri, X.numpy(), op, w2.numpy(), agg="sum", W=None if W is None else W.numpy(), act="relu" if Fo else "none")
        ctx.layer_forward(h, Xd, Y, edge_op=op, edge_weight=w2.cuda(), agg="sum", accum_out=A, **kw)
        torch.cuda.synchronize()
        assert_sum_close(A.cpu().numpy(), ref2["A"], ref2["A_abs"], 2e-5, "per-call weights")
        ctx.layer_forward(h, Xd, Y, edge_op=op, agg="sum", accum_out=A, **kw)
        torch.cuda.synchronize()
        assert_sum_close(A.cpu().numpy(), ref["A"], ref["A_abs"], 2e-5, "attached weights after a call with per-call weights")
        h.set_edge_data(w2.cuda())
        ctx.layer_forward(h, Xd, Y, edge_op=op, agg="sum", accum_out=A, **kw)
        torch.cuda.synchronize()
        assert_sum_close(A.cpu().numpy(), ref2["A"], ref2["A_abs"], 2e-5, "new attached weights")
    # the same layer without the dense blocks gives the same sums up to the rounding of the two-part weights
    ctx.set_option("dense_blocks", 0)
    A0 = torch.full((n, F), float("nan"), device="cuda")
    ctx.layer_forward(h, Xd, Y, edge_op=op, agg="sum", accum_out=A0, **kw)
    torch.cuda.synchronize()
    refk = ref2 if op == "mul_weight" else ref
    assert_sum_close(A0.cpu().numpy(), refk["A"], refk["A_abs"], 2e-5, "sparse path")
    h.destroy()
    ctx.destroy()


@pytest.mark.parametrize("scale,ef,sym", [(9, 40, True), (11, 24, False)])
@pytest.mark.parametrize("F,Fo,op,attach,opts", [(256, 128, "mul_weight", True, dict(dense_min_edges=8, dense_tile_gain=0, dense_chunk=3)),
                                                 (128, 384, "mul_weight", False, dict(dense_min_edges=16, dense_tile_gain=0)),
                                                 (512, 256, "copy", False, dict(dense_min_edges=4, dense_tile_gain=0, dense_chunk=1, split=16, cut_degree=16))])
def test_dense_blocks_in_the_bf16_backward_pass(scale, ef, sym, F, Fo, op, attach, opts):
    """The backward propagation of a bf16 layer runs over the edges grouped by source: the same dense-block form on the
    transposed adjacency matrix (rows of min(F, F_out) values travel: 128, 128 and 256 here). Against the oracle's whole-graph
    backward pass; the same call without dense blocks must agree with the same reference and differ in bits where the
    edges carry weights (two-part bf16 weights round differently), which shows that the dense kernel ran."""
    import paper_1810_08403_amd as saga
    g = _rmat(scale, ef, sym)
    n = g.n
    rng = np.random.default_rng(43)
    t = lambda *shape, s=1.0: torch.as_tensor((rng.standard_normal(shape) * s).astype(np.float32))
    X, w = si.round_to_bf16(t(n, F)), t(g.nnz)
    W = si.round_to_bf16(t(F, Fo, s=0.3))
    dY = si.round_to_bf16(t(n, Fo))
    cp, ri = g.col_ptr.numpy(), g.row_idx.numpy()
    wn = w.numpy() if op == "mul_weight" else None
    fwd = oracle.layer(cp, ri, X.numpy(), op, wn, agg="sum", W=W.numpy(), act="relu")
    bwd = oracle.layer_backward(cp, ri, X.numpy(), fwd["A"], dY.numpy(), W.numpy(), op, wn, act="relu")
    bf = torch.bfloat16
    results = []
    for dense in (1, 0):
        ctx = saga.Context(0)
        for k, v in opts.items():
            ctx.set_option(k, v)
        ctx.set_option("dense_blocks", dense)
        h = ctx.graph_create_csc(n, g.col_ptr.cuda(), g.row_idx.cuda())
        kw = {}
        if op == "mul_weight":
            if attach:
                h.set_edge_data(w.cuda())
            else:
                kw["edge_weight"] = w.cuda()
        A = torch.as_tensor(fwd["A"], dtype=torch.float32).cuda()
        Y16 = torch.as_tensor(fwd["Y"], dtype=torch.float32).cuda().to(bf)
        dW = torch.full((F, Fo), float("nan"), device="cuda")
        for rep in range(2):     # the second call finds the plan, and attached weights already packed
            dX = torch.full((n, F), float("nan"), device="cuda", dtype=bf)
            ctx.layer_backward(h, A, dY.cuda().to(bf), W.cuda().to(bf), dW, Y=Y16, edge_op=op, act="relu", dX=dX, **kw)
            torch.cuda.synchronize()
            what = f"bf16 backward rmat {scale} {F}->{Fo} {op} dense_blocks={dense} call {rep}"
            assert_sum_close(dX.float().cpu().numpy(), bwd["dX"], bwd["dX_abs"], TOL_BF16, what + " dX")
            assert_sum_close(dW.cpu().numpy(), bwd["dW"], bwd["dW_abs"], 1e-5, what + " dW")
        if op == "mul_weight" and attach:   # new attached data reach the transposed order and its packed blocks
            w2 = t(g.nnz)
            h.set_edge_data(w2.cuda())
            bwd2 = oracle.layer_backward(cp, ri, X.numpy(), fwd["A"], dY.numpy(), W.numpy(), op, w2.numpy(), act="relu")
            dX2 = torch.full((n, F), float("nan"), device="cuda", dtype=bf)
            ctx.layer_backward(h, A, dY.cuda().to(bf), W.cuda().to(bf), dW, Y=Y16, edge_op=op, act="relu", dX=dX2)
            torch.cuda.synchronize()
            assert_sum_close(dX2.float().cpu().numpy(), bwd2["dX"], bwd2["dX_abs"], TOL_BF16, "new attached weights, dX")
        results.append(dX.clone())
        h.destroy()
        ctx.destroy()
    if op == "mul_weight":
        assert not torch.equal(results[0], results[1]), "the dense-block path was not taken in the backward pass"

"""The other layer programs of the paper on the same kernels: CommNet (Figure 9) and
max-pooling GCN (Figure 11), through the C ABI against the oracle."""
import numpy as np
import pytest
import torch

import saga_inputs as si
from helpers import TOL_BF16, TOL_F32, assert_sum_close, make_graph, run_gpu, run_oracle

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    import paper_1810_08403_amd as saga
    c = saga.Context(0)
    yield c
    c.destroy()


@pytest.mark.parametrize("f_in,f_out", [(64, 64), (128, 48), (20, 7), (500, 16)])
def test_commnet_layer(ctx, f_in, f_out):
    wl = si.commnet_workload(scale=12, f_in=f_in, f_out=f_out)
    graph = make_graph(ctx, wl.graph)
    bias = si.uniform_pm(f_out, 0.3, 77)
    Y, A = run_gpu(ctx, wl, graph, bias=bias)
    ref = run_oracle(wl, bias=bias)
    assert_sum_close(A, ref["A"], ref["A_abs"], TOL_F32, "CommNet Gather")
    assert_sum_close(Y, ref["Y"], ref["Y_abs"], TOL_F32, "CommNet layer")
    # the self term really is there: without it the result differs
    wl2 = si.commnet_workload(scale=12, f_in=f_in, f_out=f_out)
    wl2.W_self = None
    Y2, _ = run_gpu(ctx, wl2, graph, bias=bias)
    assert np.abs(Y - Y2).max() > 1e-3
    graph.destroy()


def test_commnet_layer_bf16(ctx):
    wl = si.commnet_workload(scale=12, f_in=128, f_out=64)
    wl.dtype = "bf16"
    wl.X, wl.W, wl.W_self = si.round_to_bf16(wl.X), si.round_to_bf16(wl.W), si.round_to_bf16(wl.W_self)
    graph = make_graph(ctx, wl.graph)
    Y, A = run_gpu(ctx, wl, graph)
    ref = run_oracle(wl)
    assert_sum_close(A, ref["A"], ref["A_abs"], TOL_F32, "CommNet bf16 Gather")
    assert_sum_close(Y, ref["Y"], ref["Y_abs"], TOL_BF16, "CommNet bf16 layer")
    graph.destroy()


@pytest.mark.parametrize("f_in,f_pool,f_out", [(64, 32, 16), (128, 128, 128), (30, 9, 5), (16, 256, 8)])
def test_max_pooling_gcn_layer(ctx, f_in, f_pool, f_out):
    wl = si.mpgcn_workload(scale=12, f_in=f_in, f_pool=f_pool, f_out=f_out)
    deg = wl.graph.in_degree()
    assert (deg == 0).any() and deg.max().item() > 128          # empty columns and cut columns
    graph = make_graph(ctx, wl.graph)
    Y, A = run_gpu(ctx, wl, graph, agg="max")
    ref = run_oracle(wl, agg="max", hoisted=True)
    assert A.shape == (wl.graph.n, f_pool)
    # the messages are sigmoids evaluated in fp32, so the maximum is compared to tolerance, not bit for bit
    assert_sum_close(A, ref["A"], ref["A_abs"], TOL_F32, "MP-GCN max Gather")
    assert_sum_close(Y, ref["Y"], ref["Y_abs"], TOL_F32, "MP-GCN layer")
    assert not A[(deg == 0).numpy()].any() and (A[(deg > 0).numpy()] > 0).all()
    # naive per-edge oracle on a sample agrees too
    vl = np.arange(0, wl.graph.n, 37)
    refn = run_oracle(wl, agg="max", vlist=vl)
    assert_sum_close(Y[vl], refn["Y"], refn["Y_abs"], TOL_F32, "MP-GCN layer vs naive oracle")
    graph.destroy()


def test_pool_with_sum_and_sigmoid_vertex_activation(ctx):
    wl = si.mpgcn_workload(scale=11, f_in=32, f_pool=16, f_out=8)
    wl.act = "sigmoid"
    graph = make_graph(ctx, wl.graph)
    Y, A = run_gpu(ctx, wl, graph, agg="sum")
    ref = run_oracle(wl, agg="sum", hoisted=True)
    assert_sum_close(A, ref["A"], ref["A_abs"], TOL_F32, "pool + sum Gather")
    assert_sum_close(Y, ref["Y"], ref["Y_abs"], TOL_F32, "sigmoid ApplyVertex")
    graph.destroy()


def test_new_parameters_are_validated(ctx):
    import paper_1810_08403_amd as saga
    wl = si.mpgcn_workload(scale=9, f_in=16, f_pool=8, f_out=4)
    graph = make_graph(ctx, wl.graph)
    X = wl.X.cuda()
    n = wl.graph.n
    def status(fn):
        with pytest.raises(saga.SagaError) as e:
            fn()
        return e.value.status
    Y8 = torch.empty(n, 8, device="cuda")
    assert status(lambda: ctx.layer_forward(graph, X, Y8, edge_op="pool")) == 1                       # no W_pool
    assert status(lambda: ctx.layer_forward(graph, X, Y8, edge_op="pool", W_pool=torch.zeros(8, 15, device="cuda"))) == 1
    assert status(lambda: ctx.layer_forward(graph, X, torch.empty(n, 16, device="cuda"), edge_op="pool",
                                            W_pool=wl.W_pool.cuda())) == 1                              # Y must be n x F_pool
    Y4 = torch.empty(n, 4, device="cuda")
    assert status(lambda: ctx.layer_forward(graph, X, Y4, edge_op="copy", W=torch.zeros(16, 4, device="cuda"),
                                            W_self=torch.zeros(15, 4, device="cuda"))) == 1
    assert status(lambda: ctx.layer_forward(graph, X, torch.empty(n, 16, device="cuda"), edge_op="copy",
                                            W_self=torch.zeros(16, 16, device="cuda"))) == 3            # W_self without W
    graph.destroy()


@pytest.mark.parametrize("dtype,f_in,f_out,edge_op,act", [("f32", 500, 16, "mul_weight", "relu"), ("f32", 64, 3, "copy", "sigmoid"),
                                                          ("bf16", 512, 64, "mul_weight", "relu"), ("bf16", 96, 40, "copy", "none"),
                                                          ("f32", 37, 5, "mul_weight", "relu")])
def test_transform_first_gives_the_same_layer(dtype, f_in, f_out, edge_op, act):
    """Option transform_first: the product runs before the propagation when the layer narrows the rows. Same function as
    the paper's order (the oracle's), different rounding order."""
    from helpers import new_context
    wl = si.workload(2, scale=12, f_in=f_in, f_out=f_out)
    wl.edge_op, wl.act, wl.dtype = edge_op, act, dtype
    if edge_op == "copy":
        wl.edge_weight = None
    if dtype == "bf16":
        wl.X, wl.W = si.round_to_bf16(wl.X), si.round_to_bf16(wl.W)
    bias = si.uniform_pm(f_out, 0.3, 77)
    ref = run_oracle(wl, bias=bias)
    tol = TOL_BF16 if dtype == "bf16" else TOL_F32
    with new_context(transform_first=1) as c:
        graph = make_graph(c, wl.graph)
        Y, _ = run_gpu(c, wl, graph, bias=bias, want_accum=False)
        assert_sum_close(Y, ref["Y"], ref["Y_abs"], tol, f"transform-first {dtype} {f_in}->{f_out}")
        info = graph.info()
        # with accum_out the paper's order runs (the Gather output has to exist) and gives its usual result
        Y2, A = run_gpu(c, wl, graph, bias=bias, want_accum=True)
        assert_sum_close(A, ref["A"], ref["A_abs"], TOL_F32, "Gather with accum_out")
        assert_sum_close(Y2, ref["Y"], ref["Y_abs"], tol, "layer with accum_out")
        graph.destroy()
    assert info["n_work_items"] > 0


@pytest.mark.parametrize("dtype,edge_op,agg", [("f32", "mul_weight", "sum"), ("f32", "copy", "max"), ("f32", "mul_weight", "max"),
                                               ("bf16", "mul_weight", "sum"), ("bf16", "copy", "max")])
def test_stage_by_stage_propagation_equals_the_fused_operator(dtype, edge_op, agg):
    """Option fused = 0 runs Scatter, ApplyEdge and Gather one after the other through a materialised per-edge tensor
    (the baseline of the paper's Section 6.2). Fusion preserves the layer (Section 3.2): max results are the same
    bits, sums agree with the oracle like the fused ones do; gated and pooled messages are refused in this mode."""
    import paper_1810_08403_amd as saga
    from helpers import assert_bit_equal, new_context
    wl = si.workload(3 if dtype == "bf16" else 2, scale=11, edge_factor=24, f_in=72, f_out=40)
    wl.edge_op = edge_op
    if edge_op == "copy":
        wl.edge_weight = None
    tol = TOL_BF16 if dtype == "bf16" else TOL_F32
    ref = run_oracle(wl, agg=agg)
    with new_context() as c1, new_context(fused=0) as c0:
        res = {}
        for name, c in (("fused", c1), ("staged", c0)):
            graph = make_graph(c, wl.graph)
            res[name] = run_gpu(c, wl, graph, agg=agg)
            graph.destroy()
        for name in res:
            assert_sum_close(res[name][0], ref["Y"], ref["Y_abs"], tol, f"{name} {dtype} {edge_op} {agg}")
        if agg == "max":
            assert_bit_equal(res["staged"][1], res["fused"][1], "stage-by-stage max Gather vs fused")
            assert_bit_equal(res["staged"][1], ref["A"], "stage-by-stage max Gather vs oracle")
        wg = si.workload(4, scale=9, f_in=16, f_out=8)
        gg = make_graph(c0, wg.graph)
        with pytest.raises(saga.SagaError) as e:
            run_gpu(c0, wg, gg)
        assert e.value.status == 3
        gg.destroy()


@pytest.mark.parametrize("op", ["gated", "pool"])
def test_per_vertex_products_over_the_edge_endpoints_only(ctx, op):
    """Configuration 4's directed graph at R-MAT 16 with rows of 128 features: a third of the vertices have no out-edge,
    a third no in-edge, and the per-vertex products of the gated and of the pooled ApplyEdge (Section 3.2) are formed for
    edge endpoints only (the two lists end in ragged tiles). The whole layer against the oracle, the number of products
    formed against the degree counts, and a second call on the same handle gives the same bits."""
    import oracle
    wl = si.workload(4, scale=16)
    g = wl.graph
    n, F = wl.X.shape
    cp, ri = g.col_ptr.numpy(), g.row_idx.numpy()
    n_dst, n_src = int((np.diff(cp) > 0).sum()), int((np.bincount(ri, minlength=n) > 0).sum())
    assert n_dst % 64 and n_src % 64 and 16384 <= n_dst <= n * 7 // 8 and 16384 <= n_src <= n * 7 // 8
    if op == "gated":
        kw = dict(edge_op="gated", W_gate=wl.W_gate.cuda(), b_gate=wl.b_gate.cuda(), W_msg=wl.W_msg.cuda())
        ref = oracle.layer(cp, ri, wl.X.numpy(), "gated", W=wl.W.numpy(), act="relu", b_gate=wl.b_gate.numpy(),
                           hoisted=oracle.hoist(wl.X.numpy(), wl.W_gate.numpy(), wl.W_msg.numpy()))
        formed = n_src * 2 * F + n_dst * F
    else:
        Wp, bp = si.glorot_uniform(F, F, 71).T.contiguous(), si.uniform_pm(F, 0.2, 72)
        kw = dict(edge_op="pool", W_pool=Wp.cuda(), b_pool=bp.cuda())
        ref = oracle.layer(cp, ri, wl.X.numpy(), "pool", agg="sum", W=wl.W.numpy(), act="relu", W_pool=Wp.numpy(), b_pool=bp.numpy())
        formed = n_src * F
    graph = make_graph(ctx, g)
    X, W = wl.X.cuda(), wl.W.cuda()
    Y = torch.full((n, wl.W.shape[1]), float("nan"), device="cuda")
    ctx.layer_forward(graph, X, Y, W=W, act="relu", **kw)
    torch.cuda.synchronize()
    assert ctx.get_timings()["n_hoist_row_cols"] == formed
    assert_sum_close(Y.cpu().numpy(), ref["Y"], ref["Y_abs"], TOL_F32, f"{op} layer at R-MAT 16")
    Y2 = torch.full_like(Y, float("nan"))
    ctx.layer_forward(graph, X, Y2, W=W, act="relu", **kw)
    torch.cuda.synchronize()
    assert torch.equal(Y, Y2)
    graph.destroy()

"""Streamed (chunked) layer on the GPU: vertex intervals x edge chunks from host memory
must give what the oracle gives, for any tiling."""
import numpy as np
import pytest
import torch

import saga_inputs as si
from helpers import TOL_F32, assert_bit_equal, assert_sum_close, coarse_gated_workload, new_context, run_oracle

pytestmark = pytest.mark.gpu


def _streamed(ctx, wl, graph, agg, with_vertex=True, bias=None):
    n, F = wl.X.shape
    X = wl.X.clone().pin_memory()
    kw = dict(edge_op=wl.edge_op, agg=agg)
    if with_vertex:
        kw.update(W=wl.W.cuda(), act=wl.act, bias=None if bias is None else bias.cuda())
        Y = torch.empty(n, wl.W.shape[1]).pin_memory()
    else:
        Y = torch.empty(n, F).pin_memory()
    Y.fill_(float("nan"))
    ctx.layer_forward(graph, X, Y, **kw)
    return Y.numpy().copy()


@pytest.fixture(scope="module")
def wl():
    w = si.workload(5, scale=13, edge_factor=24, f_in=48, f_out=40)
    return w


@pytest.mark.parametrize("Q,P", [(1, 1), (1, 2), (2, 3), (3, 3), (4, 7), (1, 16), (2, 2)])
def test_any_tiling_gives_the_oracle_result(wl, Q, P):
    import paper_1810_08403_amd as saga
    ctx = saga.Context(0)
    ctx.set_option("dst_intervals", Q)
    ctx.set_option("src_intervals", P)
    graph = ctx.graph_create_csc(wl.graph.n, wl.graph.col_ptr, wl.graph.row_idx)   # host graph
    graph.set_edge_data(wl.edge_weight)
    ref_max = run_oracle(wl, agg="max", with_vertex=False)
    A = _streamed(ctx, wl, graph, "max", with_vertex=False)
    assert_bit_equal(A, ref_max["A"], f"max Gather, {Q} x {P}")
    ref = run_oracle(wl, agg="sum")
    Y = _streamed(ctx, wl, graph, "sum")
    assert_sum_close(Y, ref["Y"], ref["Y_abs"], TOL_F32, f"sum layer, {Q} x {P}")
    refm = run_oracle(wl, agg="max")
    Y = _streamed(ctx, wl, graph, "max")
    assert_sum_close(Y, refm["Y"], refm["Y_abs"], TOL_F32, f"max layer, {Q} x {P}")
    t = ctx.get_timings()
    assert t["plan_dst_intervals"] == Q and t["plan_src_intervals"] == P
    assert t["bytes_d2h"] > 0 and t["bytes_h2d"] >= Q * wl.X.numel() * 4 * 0  # counted
    ctx.destroy()


def test_copy_edge_op_and_empty_columns_streamed():
    import paper_1810_08403_amd as saga
    w = si.workload(4, scale=12, f_in=24, f_out=8)          # directed, empty columns
    w.edge_op, w.edge_weight = "copy", None
    ctx = saga.Context(0)
    ctx.set_option("dst_intervals", 2)
    ctx.set_option("src_intervals", 5)
    graph = ctx.graph_create_csc(w.graph.n, w.graph.col_ptr, w.graph.row_idx)
    for agg in ("sum", "max"):
        ref = run_oracle(w, agg=agg, with_vertex=False)
        A = _streamed(ctx, w, graph, agg, with_vertex=False)
        if agg == "max":
            assert_bit_equal(A, ref["A"])
        else:
            assert_sum_close(A, ref["A"], ref["A_abs"], TOL_F32)
    ctx.destroy()


def test_budget_drives_the_plan_and_is_respected(wl):
    import paper_1810_08403_amd as saga
    n, F = wl.X.shape
    x_bytes = n * F * 4
    # a budget of about half of |X| + slack: the accumulator cannot hold every destination row at once
    budget = x_bytes // 2 + (4 << 20)
    ctx = saga.Context(0, hbm_budget_bytes=budget)
    graph = ctx.graph_create_csc(wl.graph.n, wl.graph.col_ptr, wl.graph.row_idx)
    graph.set_edge_data(wl.edge_weight)
    ref = run_oracle(wl, agg="sum")
    Y = _streamed(ctx, wl, graph, "sum")
    assert_sum_close(Y, ref["Y"], ref["Y_abs"], TOL_F32, "budgeted plan")
    t = ctx.get_timings()
    assert t["plan_dst_intervals"] >= 2 and t["plan_src_intervals"] >= t["plan_dst_intervals"]
    assert ctx.peak_device_bytes() <= budget
    ctx.destroy()
    # a budget no plan can meet
    ctx = saga.Context(0, hbm_budget_bytes=1 << 16)
    graph = ctx.graph_create_csc(wl.graph.n, wl.graph.col_ptr, wl.graph.row_idx)
    graph.set_edge_data(wl.edge_weight)
    with pytest.raises(saga.SagaError) as e:
        _streamed(ctx, wl, graph, "sum")
    assert e.value.status == 4      # SAGA_ERR_BUDGET
    ctx.destroy()


def test_streamed_needs_attached_edge_data_and_rejects_mixed_placement(wl):
    import paper_1810_08403_amd as saga
    ctx = saga.Context(0)
    graph = ctx.graph_create_csc(wl.graph.n, wl.graph.col_ptr, wl.graph.row_idx)
    X = wl.X.clone().pin_memory()
    Y = torch.empty_like(X).pin_memory()
    with pytest.raises(saga.SagaError) as e:
        ctx.layer_forward(graph, X, Y, edge_op="mul_weight")
    assert e.value.status == 1
    with pytest.raises(saga.SagaError) as e:
        ctx.layer_forward(graph, X.cuda(), Y, edge_op="copy")
    assert e.value.status == 1
    bad = wl.graph.row_idx.clone()
    bad[5] = wl.graph.n + 3
    with pytest.raises(saga.SagaError) as e:
        ctx.graph_create_csc(wl.graph.n, wl.graph.col_ptr, bad)
    assert e.value.status == 2
    ctx.destroy()


@pytest.mark.parametrize("schedule,overlap", [(0, 0), (1, 1), (1, 0), (2, 1), (2, 0)])
def test_baseline_schedules_give_the_same_result(wl, schedule, overlap):
    """Stage-by-stage and destination-order schedules and streaming off (the baselines of the
    paper's Section 6.2) move data differently but must compute the same layer."""
    from helpers import new_context
    with new_context(dst_intervals=3, src_intervals=4, schedule=schedule, overlap=overlap) as ctx:
        graph = ctx.graph_create_csc(wl.graph.n, wl.graph.col_ptr, wl.graph.row_idx)
        graph.set_edge_data(wl.edge_weight)
        ref_max = run_oracle(wl, agg="max", with_vertex=False)
        A = _streamed(ctx, wl, graph, "max", with_vertex=False)
        assert_bit_equal(A, ref_max["A"], f"max Gather, schedule {schedule}")
        ref = run_oracle(wl, agg="sum")
        Y = _streamed(ctx, wl, graph, "sum")
        assert_sum_close(Y, ref["Y"], ref["Y_abs"], TOL_F32, f"sum layer, schedule {schedule}")
        refm = run_oracle(wl, agg="max")
        Y = _streamed(ctx, wl, graph, "max")
        assert_sum_close(Y, refm["Y"], refm["Y_abs"], TOL_F32, f"max layer, schedule {schedule}")
        t = ctx.get_timings()
        x_bytes = wl.X.numel() * 4
        if schedule == 0:
            assert t["bytes_h2d"] < 3 * 3 * x_bytes + 3 * 2 ** 26        # X three times per call + chunks
        if schedule == 2:
            assert t["bytes_d2h"] > 3 * x_bytes                            # accumulators swapped per chunk


def test_reencoded_graph_gives_the_permuted_oracle_result(wl):
    """Section 3.1's id re-encoding for chunk balance: the layer on the relabelled graph, features and edge data is the
    layer on the original ones with its rows renamed (max: bit for bit; sum: to tolerance), and the chunks are more even."""
    import copy
    import paper_1810_08403_amd as saga
    Q, P = 2, 8
    new_id, stats = saga.plan_reencoding(wl.graph.col_ptr, wl.graph.row_idx, Q, P, seed=4)
    assert stats["after"]["max_chunk_edges"] < stats["before"]["max_chunk_edges"]
    w2 = copy.copy(wl)
    w2.graph = si.relabel_csc(wl.graph, new_id)
    w2.X = torch.empty_like(wl.X)
    w2.X[new_id.long()] = wl.X
    w2.edge_weight = si.gcn_edge_weights(w2.graph)
    ctx = saga.Context(0)
    ctx.set_option("dst_intervals", Q)
    ctx.set_option("src_intervals", P)
    graph = ctx.graph_create_csc(w2.graph.n, w2.graph.col_ptr, w2.graph.row_idx)
    graph.set_edge_data(w2.edge_weight)
    ref_max = run_oracle(wl, agg="max", with_vertex=False)        # the oracle on the ORIGINAL ids
    A = _streamed(ctx, w2, graph, "max", with_vertex=False)
    assert_bit_equal(A[new_id.long().numpy()], ref_max["A"], "max Gather on re-encoded ids")
    ref = run_oracle(wl, agg="sum")
    Y = _streamed(ctx, w2, graph, "sum")
    assert_sum_close(Y[new_id.long().numpy()], ref["Y"], ref["Y_abs"], TOL_F32, "sum layer on re-encoded ids")
    ctx.destroy()


@pytest.mark.parametrize("act,edge_op,Q,P,tile", [("relu", "mul_weight", 2, 3, 1000), ("none", "mul_weight", 1, 4, 0), ("relu", "copy", 3, 3, 4096),
                                                  ("none", "copy", 1, 1, 777), ("sigmoid", "mul_weight", 2, 2, 1500)])
def test_streamed_backward_matches_oracle(wl, act, edge_op, Q, P, tile):
    """Backward pass with everything but the parameters in host memory: tiles of backward-ApplyVertex, then the chunk
    schedule over the edges clustered by source."""
    import oracle
    import paper_1810_08403_amd as saga
    g = wl.graph
    n, F = wl.X.shape
    Fo = wl.W.shape[1]
    cp, ri = g.col_ptr.numpy(), g.row_idx.numpy()
    w = wl.edge_weight.numpy() if edge_op == "mul_weight" else None
    dY = si.normal_features(n, Fo, 21)
    bias = si.uniform_pm(Fo, 0.3, 3)
    fwd = oracle.layer(cp, ri, wl.X.numpy(), edge_op, w, W=wl.W.numpy(), bias=bias.numpy(), act=act)
    bwd = oracle.layer_backward(cp, ri, wl.X.numpy(), fwd["A"], dY.numpy(), wl.W.numpy(), edge_op, w, bias=bias.numpy(), act=act)
    ctx = saga.Context(0)
    for name, val in (("dst_intervals", Q), ("src_intervals", P), ("bwd_tile_rows", tile)):
        ctx.set_option(name, val)
    graph = ctx.graph_create_csc(n, g.col_ptr, g.row_idx)        # host graph
    if edge_op == "mul_weight":
        graph.set_edge_data(wl.edge_weight)
    pin = lambda a: torch.as_tensor(np.ascontiguousarray(a), dtype=torch.float32).pin_memory()
    A_h, Y_h, dY_h = pin(fwd["A"]), pin(fwd["Y"]), pin(dY.numpy())
    dX_h = torch.full((n, F), float("nan")).pin_memory()
    dW, db = torch.full((F, Fo), float("nan"), device="cuda"), torch.full((Fo,), float("nan"), device="cuda")
    for rep in range(2):                                           # the second call reuses the transposed chunk grid
        ctx.layer_backward(graph, A_h, dY_h, wl.W.cuda(), dW, Y=Y_h, edge_op=edge_op, bias=bias.cuda(), act=act, dX=dX_h, dbias=db)
        torch.cuda.synchronize()
        what = f"streamed backward {act} {edge_op} {Q}x{P} tile {tile} call {rep}"
        assert_sum_close(dW.cpu().numpy(), bwd["dW"], bwd["dW_abs"], TOL_F32, what + " dW")
        assert_sum_close(dX_h.numpy(), bwd["dX"], bwd["dX_abs"], TOL_F32, what + " dX")
        assert_sum_close(db.cpu().numpy(), bwd["dbias"], np.maximum(bwd["dbias_abs"], 1e-30), TOL_F32, what + " dbias")
        dX_h.fill_(float("nan"))
    # without dX only backward-ApplyVertex runs, over tiles of rows
    dW.fill_(float("nan"))
    db.fill_(float("nan"))
    ctx.layer_backward(graph, A_h, dY_h, wl.W.cuda(), dW, Y=Y_h, edge_op=edge_op, bias=bias.cuda(), act=act, dbias=db)
    torch.cuda.synchronize()
    assert_sum_close(dW.cpu().numpy(), bwd["dW"], bwd["dW_abs"], TOL_F32, "parameter gradients only: dW")
    assert_sum_close(db.cpu().numpy(), bwd["dbias"], np.maximum(bwd["dbias_abs"], 1e-30), TOL_F32, "parameter gradients only: dbias")
    # a forward call on the same graph still works afterwards (its own chunk grid is untouched)
    Yf = torch.empty(n, Fo).pin_memory()
    kw = dict(edge_op=edge_op, W=wl.W.cuda(), act=act, bias=bias.cuda())
    ctx.layer_forward(graph, wl.X.clone().pin_memory(), Yf, **kw)
    assert_sum_close(Yf.numpy(), fwd["Y"], fwd["Y_abs"], TOL_F32, "forward after backward")
    ctx.destroy()


@pytest.mark.parametrize("act,Q,P,tile", [("relu", 2, 3, 1000), ("sigmoid", 1, 4, 0), ("none", 3, 3, 700)])
def test_streamed_backward_with_own_product(act, Q, P, tile):
    """The CommNet layer (COPY messages, Y = act(A W + X W_self + b)) backwards with everything but the parameters in
    host memory: dW_self is added interval by interval from tiles of X, and the vertex's own partial gradient
    dZ W_self^T joins dX as the second operand pair of the schedule's last product, its rows of dZ formed tile by tile."""
    import oracle
    import paper_1810_08403_amd as saga
    wl = si.commnet_workload(scale=12, f_in=40, f_out=24)
    g = wl.graph
    n, F = wl.X.shape
    Fo = wl.W.shape[1]
    cp, ri = g.col_ptr.numpy(), g.row_idx.numpy()
    dY = si.normal_features(n, Fo, 21)
    bias = si.uniform_pm(Fo, 0.3, 3)
    fwd = oracle.layer(cp, ri, wl.X.numpy(), "copy", W=wl.W.numpy(), W_self=wl.W_self.numpy(), bias=bias.numpy(), act=act)
    bwd = oracle.layer_backward(cp, ri, wl.X.numpy(), fwd["A"], dY.numpy(), wl.W.numpy(), "copy", bias=bias.numpy(),
                                W_self=wl.W_self.numpy(), act=act)
    ctx = saga.Context(0)
    for name, val in (("dst_intervals", Q), ("src_intervals", P), ("bwd_tile_rows", tile)):
        ctx.set_option(name, val)
    graph = ctx.graph_create_csc(n, g.col_ptr, g.row_idx)
    pin = lambda a: torch.as_tensor(np.ascontiguousarray(a), dtype=torch.float32).pin_memory()
    X_h, A_h, Y_h, dY_h = wl.X.clone().pin_memory(), pin(fwd["A"]), pin(fwd["Y"]), pin(dY.numpy())
    dX_h = torch.full((n, F), float("nan")).pin_memory()
    nan = lambda *s: torch.full(s, float("nan"), device="cuda")
    dW, dWs, db = nan(F, Fo), nan(F, Fo), nan(Fo)
    kw = dict(X=X_h, Y=Y_h, edge_op="copy", bias=bias.cuda(), act=act, W_self=wl.W_self.cuda(), dbias=db, dW_self=dWs)
    for rep, want_dx in enumerate([True, True, False]):           # the second call reuses the grid; the third has no dX
        for t in (dW, dWs, db):
            t.fill_(float("nan"))
        dX_h.fill_(float("nan"))
        ctx.layer_backward(graph, A_h, dY_h, wl.W.cuda(), dW, dX=dX_h if want_dx else None, **kw)
        what = f"streamed backward with W_self, {act} {Q}x{P} call {rep}"
        assert_sum_close(dW.cpu().numpy(), bwd["dW"], bwd["dW_abs"], TOL_F32, what + " dW")
        assert_sum_close(dWs.cpu().numpy(), bwd["dW_self"], bwd["dW_self_abs"], TOL_F32, what + " dW_self")
        assert_sum_close(db.cpu().numpy(), bwd["dbias"], np.maximum(bwd["dbias_abs"], 1e-30), TOL_F32, what + " dbias")
        if want_dx:
            assert_sum_close(dX_h.numpy(), bwd["dX"], bwd["dX_abs"], TOL_F32, what + " dX")
    with pytest.raises(saga.SagaError) as e:                      # W_self without X
        ctx.layer_backward(graph, A_h, dY_h, wl.W.cuda(), dW, Y=Y_h, edge_op="copy", act=act, W_self=wl.W_self.cuda(), dW_self=dWs)
    assert e.value.status == 1
    ctx.destroy()


@pytest.mark.parametrize("edge_op,act,Q,P", [("copy", "relu", 2, 3), ("mul_weight", "none", 1, 4), ("pool", "relu", 2, 2), ("pool", "sigmoid", 1, 3)])
def test_streamed_max_backward_matches_oracle(edge_op, act, Q, P):
    """Backward pass of a max-accumulator layer (plain, weighted or pooled messages) from host memory: the gradient of accum
    goes out to pinned memory tile by tile, then rows [A | gradient of accum] travel over the chunks of edges clustered
    by source while the vertex's own row sits beside the accumulator; pooled layers finish per interval on the device."""
    import oracle
    import paper_1810_08403_amd as saga
    pool = edge_op == "pool"
    wl = si.mpgcn_workload(scale=12, f_in=16, f_pool=32, f_out=24) if pool else si.commnet_workload(scale=12, f_in=40, f_out=24)
    if pool:   # coarse values: the order of the sigmoids, ties included, is the same in fp32 and fp64
        wl.X = torch.round(wl.X.clamp(-1, 1) * 4) / 4
        wl.W_pool = torch.round((wl.W_pool * 4).clamp(-0.5, 0.5) * 8) / 8
        wl.b_pool = torch.round(wl.b_pool.clamp(-0.5, 0.5) * 8) / 8
    g = wl.graph
    n, F = wl.X.shape
    Fm, Fo = wl.W.shape
    cp, ri = g.col_ptr.numpy(), g.row_idx.numpy()
    w = si.uniform_pm(g.nnz, 1.0, 17) if edge_op == "mul_weight" else None     # both signs
    dY = si.normal_features(n, Fo, 23)
    bias = si.uniform_pm(Fo, 0.3, 3)
    okw = {}
    if w is not None:
        okw["edge_weight"] = w.numpy()
    if pool:
        okw.update(W_pool=wl.W_pool.numpy(), b_pool=wl.b_pool.numpy())
    ctx = saga.Context(0)
    for name, val in (("dst_intervals", Q), ("src_intervals", P), ("bwd_tile_rows", 900)):
        ctx.set_option(name, val)
    graph = ctx.graph_create_csc(n, g.col_ptr, g.row_idx)
    if w is not None:
        graph.set_edge_data(w)
    kw = dict(edge_op=edge_op, agg="max", act=act, bias=bias.cuda())
    if pool:
        kw.update(W_pool=wl.W_pool.cuda(), b_pool=wl.b_pool.cuda())
    X_h = wl.X.clone().pin_memory()
    Y_h, A_h = torch.empty(n, Fo).pin_memory(), torch.empty(n, Fm).pin_memory()
    fwd = oracle.layer(cp, ri, wl.X.numpy(), edge_op, agg="max", W=wl.W.numpy(), bias=bias.numpy(), act=act, **okw)
    bwd = oracle.max_backward(cp, ri, wl.X.numpy(), dY.numpy(), wl.W.numpy(), edge_op, bias=bias.numpy(), act=act, **okw)
    if pool:
        # a forward pass on the device supplies A and Y: its pooled rows are the ones the backward pass recomputes bit for bit
        with new_context() as c2:
            g2 = c2.graph_create_csc(n, g.col_ptr.cuda(), g.row_idx.cuda())
            Yd, Ad = torch.empty(n, Fo, device="cuda"), torch.empty(n, Fm, device="cuda")
            c2.layer_forward(g2, wl.X.cuda(), Yd, W=wl.W.cuda(), accum_out=Ad, **kw)
            torch.cuda.synchronize()
            A_h.copy_(Ad.cpu())
            Y_h.copy_(Yd.cpu())
            g2.destroy()
        assert_sum_close(A_h.numpy(), bwd["A"], np.maximum(np.abs(bwd["A"]), 1e-30), TOL_F32, "pooled Gather of the forward pass")
    else:
        A_h.copy_(torch.as_tensor(bwd["A"], dtype=torch.float32))
        Y_h.copy_(torch.as_tensor(fwd["Y"], dtype=torch.float32))
    dY_h = dY.clone().pin_memory()
    dX_h = torch.full((n, F), float("nan")).pin_memory()
    nan = lambda *s: torch.full(s, float("nan"), device="cuda")
    dW, db = nan(Fm, Fo), nan(Fo)
    gk = dict(dW_pool=nan(Fm, F), db_pool=nan(Fm)) if pool else {}
    for rep, want_dx in enumerate([True, True, False]):
        ctx.layer_backward(graph, A_h, dY_h, wl.W.cuda(), dW, X=X_h, Y=Y_h, dX=dX_h if want_dx else None, dbias=db, **kw, **gk)
        what = f"streamed max backward {edge_op} {act} {Q}x{P} call {rep}"
        assert_sum_close(dW.cpu().numpy(), bwd["dW"], bwd["dW_abs"], TOL_F32, what + " dW")
        assert_sum_close(db.cpu().numpy(), bwd["dbias"], np.maximum(bwd["dbias_abs"], 1e-30), TOL_F32, what + " dbias")
        if want_dx:
            assert_sum_close(dX_h.numpy(), bwd["dX"], bwd["dX_abs"], TOL_F32, what + " dX")
        if pool:
            assert_sum_close(gk["dW_pool"].cpu().numpy(), bwd["dW_pool"], bwd["dW_pool_abs"], TOL_F32, what + " dW_pool")
            assert_sum_close(gk["db_pool"].cpu().numpy(), bwd["db_pool"], bwd["db_pool_abs"], TOL_F32, what + " db_pool")
            for t in gk.values():
                t.fill_(float("nan"))
        dX_h.fill_(float("nan"))
        dW.fill_(float("nan"))
        db.fill_(float("nan"))
    ctx.destroy()


def test_streamed_sum_over_pooled_messages_backward():
    """Sum over pooled messages from host memory: the gradient of accum travels as plain vertex data, then the same
    per-interval finish as for the max accumulator; against autograd of the definition in fp64."""
    import paper_1810_08403_amd as saga
    wl = si.mpgcn_workload(scale=11, f_in=12, f_pool=20, f_out=8)
    g = wl.graph
    n, F = wl.X.shape
    Fm, Fo = wl.W.shape
    dY = si.normal_features(n, Fo, 7)
    Xt = wl.X.double().requires_grad_(True)
    Wpt, bpt, Wt = wl.W_pool.double().requires_grad_(True), wl.b_pool.double().requires_grad_(True), wl.W.double().requires_grad_(True)
    H = torch.sigmoid(Xt @ Wpt.T + bpt)
    deg = g.col_ptr[1:] - g.col_ptr[:-1]
    dst = torch.repeat_interleave(torch.arange(n), deg)
    Aref = torch.zeros(n, Fm, dtype=torch.float64).index_add(0, dst, H[g.row_idx.long()])
    ((Aref @ Wt) * dY.double()).sum().backward()
    ctx = saga.Context(0)
    for name, val in (("dst_intervals", 2), ("src_intervals", 3)):
        ctx.set_option(name, val)
    graph = ctx.graph_create_csc(n, g.col_ptr, g.row_idx)
    X_h, A_h, dY_h = wl.X.clone().pin_memory(), Aref.detach().float().pin_memory(), dY.clone().pin_memory()
    dX_h = torch.full((n, F), float("nan")).pin_memory()
    nan = lambda *s: torch.full(s, float("nan"), device="cuda")
    dW, dWp, dbp = nan(Fm, Fo), nan(Fm, F), nan(Fm)
    ctx.layer_backward(graph, A_h, dY_h, wl.W.cuda(), dW, X=X_h, edge_op="pool", agg="sum", W_pool=wl.W_pool.cuda(), b_pool=wl.b_pool.cuda(),
                       act="none", dX=dX_h, dW_pool=dWp, db_pool=dbp)
    for name, got, ref in [("dW", dW.cpu(), Wt.grad), ("dX", dX_h, Xt.grad), ("dW_pool", dWp.cpu(), Wpt.grad), ("db_pool", dbp.cpu(), bpt.grad)]:
        err = (got.double() - ref).abs().max().item()
        assert err <= 2e-5 * ref.abs().max().item(), (name, err)
    ctx.destroy()


@pytest.mark.parametrize("F,Fo,act,with_b,with_msg,Q,P", [(16, 12, "relu", True, True, 2, 3), (20, 8, "none", False, False, 1, 4),
                                                          (64, 32, "sigmoid", True, True, 3, 3), (7, 5, "relu", True, False, 2, 2)])
def test_streamed_gated_backward_matches_oracle(F, Fo, act, with_b, with_msg, Q, P):
    """Backward pass of a gated layer from host memory: tile pass, the chunk schedule over the in-edges (destination
    parts of the gate gradient), the chunk schedule over the edges clustered by source (source parts, both at once,
    and dX as its last product), per-vertex products and gradients passing through pinned memory in between."""
    import oracle
    import paper_1810_08403_amd as saga
    wl = si.workload(4, scale=11, f_in=F, f_out=Fo)
    g = wl.graph
    n = g.n
    cp, ri = g.col_ptr.numpy(), g.row_idx.numpy()
    bias = si.uniform_pm(Fo, 0.3, 5)
    dY = si.normal_features(n, Fo, 99)
    okw = dict(W_gate=wl.W_gate.numpy(), b_gate=wl.b_gate.numpy() if with_b else None, W_msg=wl.W_msg.numpy() if with_msg else None)
    fwd = oracle.layer(cp, ri, wl.X.numpy(), "gated", W=wl.W.numpy(), bias=bias.numpy(), act=act, **okw)
    bwd = oracle.gated_backward(cp, ri, wl.X.numpy(), fwd["A"], dY.numpy(), wl.W.numpy(), bias=bias.numpy(), act=act, **okw)
    ctx = saga.Context(0)
    for name, val in (("dst_intervals", Q), ("src_intervals", P), ("bwd_tile_rows", 700)):
        ctx.set_option(name, val)
    graph = ctx.graph_create_csc(n, g.col_ptr, g.row_idx)
    pin = lambda a: torch.as_tensor(np.ascontiguousarray(a), dtype=torch.float32).pin_memory()
    X_h, A_h, Y_h, dY_h = wl.X.clone().pin_memory(), pin(fwd["A"]), pin(fwd["Y"]), dY.clone().pin_memory()
    dX_h = torch.full((n, F), float("nan")).pin_memory()
    nan = lambda *s: torch.full(s, float("nan"), device="cuda")
    out = dict(dW=nan(F, Fo), dbias=nan(Fo), dW_gate=nan(F, 2 * F), db_gate=nan(F) if with_b else None, dW_msg=nan(F, F) if with_msg else None)
    kw = dict(X=X_h, Y=Y_h, edge_op="gated", act=act, bias=bias.cuda(), W_gate=wl.W_gate.cuda(),
              b_gate=wl.b_gate.cuda() if with_b else None, W_msg=wl.W_msg.cuda() if with_msg else None)
    for rep, want_dx in enumerate([True, True, False]):            # the second call reuses both grids; the third has no dX
        for t in out.values():
            if t is not None:
                t.fill_(float("nan"))
        dX_h.fill_(float("nan"))
        ctx.layer_backward(graph, A_h, dY_h, wl.W.cuda(), out["dW"], dX=dX_h if want_dx else None, dbias=out["dbias"],
                           dW_gate=out["dW_gate"], db_gate=out["db_gate"], dW_msg=out["dW_msg"], **kw)
        what = f"streamed gated backward {F}->{Fo} {act} {Q}x{P} call {rep}"
        for name in ("dW", "dbias", "dW_gate", "db_gate", "dW_msg"):
            if out[name] is not None:
                assert_sum_close(out[name].cpu().numpy(), bwd[name], np.maximum(bwd[name + "_abs"], 1e-30), TOL_F32, what + " " + name)
        if want_dx:
            assert_sum_close(dX_h.numpy(), bwd["dX"], bwd["dX_abs"], TOL_F32, what + " dX")
    # a forward call on the same graph still works afterwards
    Yf = torch.empty(n, Fo).pin_memory()
    ctx.layer_forward(graph, X_h, Yf, W=wl.W.cuda(), **{k: v for k, v in kw.items() if k not in ("X", "Y")})
    assert_sum_close(Yf.numpy(), fwd["Y"], fwd["Y_abs"], TOL_F32, "forward after backward")
    ctx.destroy()


@pytest.mark.parametrize("F,Fo,act,with_b,with_msg,with_self,Q,P", [(16, 12, "relu", True, True, False, 2, 3), (20, 8, "none", False, False, False, 1, 4),
                                                                    (64, 32, "sigmoid", True, True, True, 3, 3), (7, 5, "relu", True, False, False, 2, 2),
                                                                    (128, 16, "relu", True, True, False, 2, 5)])
def test_streamed_gated_max_backward_matches_oracle(F, Fo, act, with_b, with_msg, with_self, Q, P):
    """Max over gated messages backwards from host memory. The Gather output handed to the backward call is the one the
    streamed forward call kept (its maxima are compared bit for bit with the messages the backward pass forms again from
    the rows of X, in intervals of its own); the stored output is synthetic, only the activation's derivative is taken
    from it, and the oracle is given the same dZ."""
    import oracle
    import paper_1810_08403_amd as saga
    wl = coarse_gated_workload(10, F, Fo)
    g = wl.graph
    n = g.n
    cp, ri = g.col_ptr.numpy(), g.row_idx.numpy()
    deg = np.diff(cp)
    assert deg.max() > 128 and (deg == 0).any()
    Ws = si.glorot_uniform(F, Fo, 41) if with_self else None
    bg = wl.b_gate if with_b else None
    Wm = wl.W_msg if with_msg else None
    opt = lambda t: None if t is None else t.cuda()
    dY = si.normal_features(n, Fo, 99)
    Y_in = si.normal_features(n, Fo, 98)
    if act == "sigmoid":
        Y_in = torch.sigmoid(Y_in)
    slope = {"none": torch.ones_like(Y_in.double()), "relu": (Y_in > 0).double(), "sigmoid": Y_in.double() * (1 - Y_in.double())}[act]
    dZ = (dY.double() * slope).float()
    okw = dict(W_gate=wl.W_gate.numpy(), b_gate=None if bg is None else bg.numpy(), W_msg=None if Wm is None else Wm.numpy(),
               W_self=None if Ws is None else Ws.numpy())
    bwd = oracle.gated_backward(cp, ri, wl.X.numpy(), None, dZ.numpy(), wl.W.numpy(), act="none", agg="max", **okw)
    ctx = saga.Context(0)
    for name, val in (("dst_intervals", Q), ("src_intervals", P), ("bwd_tile_rows", 300)):
        ctx.set_option(name, val)
    graph = ctx.graph_create_csc(n, g.col_ptr, g.row_idx)
    X_h, dY_h, Y_h = wl.X.clone().pin_memory(), dY.clone().pin_memory(), Y_in.clone().pin_memory()
    A_h = torch.full((n, F), float("nan")).pin_memory()
    Yf = torch.empty(n, Fo).pin_memory()
    gate = dict(edge_op="gated", agg="max", W_gate=wl.W_gate.cuda(), b_gate=opt(bg), W_msg=opt(Wm), W_self=opt(Ws))
    ctx.layer_forward(graph, X_h, Yf, W=wl.W.cuda(), act="none", accum_out=A_h, **gate)
    what = f"streamed gated max {F}->{Fo} {act} {Q}x{P}"
    assert_sum_close(A_h.numpy(), bwd["A"], np.maximum(np.abs(bwd["A"]), 1e-30), TOL_F32, what + " A")
    nan = lambda *s: torch.full(s, float("nan"), device="cuda")
    out = dict(dW=nan(F, Fo), dbias=nan(Fo), dW_gate=nan(F, 2 * F), db_gate=nan(F) if with_b else None,
               dW_msg=nan(F, F) if with_msg else None, dW_self=nan(F, Fo) if with_self else None)
    dX_h = torch.full((n, F), float("nan")).pin_memory()
    first = None
    for rep, want_dx in enumerate([True, True, False]):            # the second call reuses both grids; the third has no dX
        for t in out.values():
            if t is not None:
                t.fill_(float("nan"))
        dX_h.fill_(float("nan"))
        ctx.layer_backward(graph, A_h, dY_h, wl.W.cuda(), out["dW"], X=X_h, Y=Y_h, act=act, dX=dX_h if want_dx else None,
                           dbias=out["dbias"], dW_gate=out["dW_gate"], db_gate=out["db_gate"], dW_msg=out["dW_msg"],
                           dW_self=out["dW_self"], **gate)
        for name, t in out.items():
            if t is not None:
                assert np.abs(bwd[name]).max() > 0, name
                assert_sum_close(t.cpu().numpy(), bwd[name], np.maximum(bwd[name + "_abs"], 1e-30), TOL_F32, f"{what} call {rep} {name}")
        if want_dx:
            assert_sum_close(dX_h.numpy(), bwd["dX"], bwd["dX_abs"], TOL_F32, f"{what} call {rep} dX")
            if not with_self:   # a source that supplied no maximum and has no in-edges gets exactly nothing
                assert ((bwd["dX_abs"] == 0) <= (dX_h.numpy() == 0)).all()
        if first is None:
            first = {k: v.clone() for k, v in out.items() if v is not None}
        else:
            assert all(torch.equal(first[k], out[k]) for k in first), "the same call twice gives other bits"
    ctx.destroy()


def test_streamed_gated_max_backward_forms_the_forward_calls_bits_again():
    """Configuration 4's widths on R-MAT 16 with continuous data, one destination interval and eight source intervals: the
    forward call forms the destination parts of the gate for all 65,536 rows at once, the out-edge pass of the backward
    call forms them again in intervals of 8,192 rows (a size at which a product on the resident path would pick another
    kernel), and the messages made from them must still be the kept maxima bit for bit, or the edges carry no gradient.
    With continuous data fp32 and fp64 rank a few near-tied messages differently (a relative gap near 1e-7 among some
    thirty candidates for each of 8.4 M maxima), which moves one edge's share each: at most one element in 10,000 of dX may
    miss the element-wise bar, and the parameter gradients, in which every such edge moves one term of order one, are held
    to 2e-3 of their largest entry (measured: 4e-4; were the bits not the forward call's, most terms would be missing)."""
    import oracle
    import paper_1810_08403_amd as saga
    F, Fo = 128, 128
    wl = si.workload(4, scale=16, f_in=F, f_out=Fo)
    g = wl.graph
    n = g.n
    cp, ri = g.col_ptr.numpy(), g.row_idx.numpy()
    dZ = si.normal_features(n, Fo, 99)
    okw = dict(W_gate=wl.W_gate.numpy(), b_gate=wl.b_gate.numpy(), W_msg=wl.W_msg.numpy())
    bwd = oracle.gated_backward(cp, ri, wl.X.numpy(), None, dZ.numpy(), wl.W.numpy(), act="none", agg="max", **okw)
    with new_context(dst_intervals=1, src_intervals=8, bwd_tile_rows=5000) as ctx:
        graph = ctx.graph_create_csc(n, g.col_ptr, g.row_idx)
        X_h, dY_h = wl.X.clone().pin_memory(), dZ.clone().pin_memory()
        A_h, Yf = torch.full((n, F), float("nan")).pin_memory(), torch.empty(n, Fo).pin_memory()
        gate = dict(edge_op="gated", agg="max", W_gate=wl.W_gate.cuda(), b_gate=wl.b_gate.cuda(), W_msg=wl.W_msg.cuda())
        ctx.layer_forward(graph, X_h, Yf, W=wl.W.cuda(), act="none", accum_out=A_h, **gate)
        assert np.abs(A_h.numpy().astype(np.float64) - bwd["A"]).max() <= TOL_F32 * np.abs(bwd["A"]).max()
        nan = lambda *s: torch.full(s, float("nan"), device="cuda")
        out = dict(dW=nan(F, Fo), dbias=nan(Fo), dW_gate=nan(F, 2 * F), db_gate=nan(F), dW_msg=nan(F, F))
        dX_h = torch.full((n, F), float("nan")).pin_memory()
        ctx.layer_backward(graph, A_h, dY_h, wl.W.cuda(), out["dW"], X=X_h, act="none", dX=dX_h, dbias=out["dbias"],
                           dW_gate=out["dW_gate"], db_gate=out["db_gate"], dW_msg=out["dW_msg"], **gate)
        err = np.abs(dX_h.numpy().astype(np.float64) - bwd["dX"])
        assert np.isfinite(err).all()
        missed = (err > TOL_F32 * np.maximum(bwd["dX_abs"], 1e-30)).sum()
        print(f"{missed} of {err.size} elements of dX miss the bar")
        assert missed <= err.size // 10000, f"{missed} of {err.size} elements of dX miss the bar"
        for name, t in out.items():
            e = np.abs(t.cpu().numpy().astype(np.float64) - bwd[name]).max()
            assert e <= 2e-3 * np.abs(bwd[name]).max(), (name, e, np.abs(bwd[name]).max())
        graph.destroy()


@pytest.mark.parametrize("Q,P", [(1, 3), (2, 2), (3, 5)])
@pytest.mark.parametrize("agg", ["sum", "max"])
def test_streamed_gated_layer(Q, P, agg):
    """Configuration 4's layer from host memory: hoisted rows through pinned host memory, [Ps | M] streamed, Pd resident."""
    import paper_1810_08403_amd as saga
    w = si.workload(4, scale=12, f_in=40, f_out=24)
    g = w.graph
    n = g.n
    ctx = saga.Context(0)
    ctx.set_option("dst_intervals", Q)
    ctx.set_option("src_intervals", P)
    graph = ctx.graph_create_csc(n, g.col_ptr, g.row_idx)
    bias = si.uniform_pm(24, 0.3, 4)
    ref = run_oracle(w, agg=agg, bias=bias, hoisted=True)
    Y = torch.full((n, 24), float("nan")).pin_memory()
    ctx.layer_forward(graph, w.X.clone().pin_memory(), Y, edge_op="gated", agg=agg, W_gate=w.W_gate.cuda(), b_gate=w.b_gate.cuda(),
                      W_msg=w.W_msg.cuda(), W=w.W.cuda(), bias=bias.cuda(), act=w.act)
    assert_sum_close(Y.numpy(), ref["Y"], ref["Y_abs"], TOL_F32, f"streamed gated {agg} {Q}x{P}")
    # the same call on a device-resident copy gives the same layer
    with_dev = saga.Context(0)
    gd = with_dev.graph_create_csc(n, g.col_ptr.cuda(), g.row_idx.cuda())
    Yd = torch.empty(n, 24, device="cuda")
    with_dev.layer_forward(gd, w.X.cuda(), Yd, edge_op="gated", agg=agg, W_gate=w.W_gate.cuda(), b_gate=w.b_gate.cuda(),
                           W_msg=w.W_msg.cuda(), W=w.W.cuda(), bias=bias.cuda(), act=w.act)
    assert_sum_close(Yd.cpu().numpy(), ref["Y"], ref["Y_abs"], TOL_F32, "resident gated")
    with_dev.destroy()
    ctx.destroy()


@pytest.mark.parametrize("agg", ["max", "sum"])
def test_streamed_max_pooling_and_commnet_layers(agg):
    import paper_1810_08403_amd as saga
    ctx = saga.Context(0)
    ctx.set_option("dst_intervals", 2)
    ctx.set_option("src_intervals", 3)
    # Figure 11: pooled messages, hoisted through host memory, then max (or sum) over them
    w = si.mpgcn_workload(scale=12, f_in=24, f_pool=40, f_out=16)
    g = w.graph
    graph = ctx.graph_create_csc(g.n, g.col_ptr, g.row_idx)
    ref = run_oracle(w, agg=agg, hoisted=True)
    Y = torch.full((g.n, 16), float("nan")).pin_memory()
    ctx.layer_forward(graph, w.X.clone().pin_memory(), Y, edge_op="pool", agg=agg, W_pool=w.W_pool.cuda(), b_pool=w.b_pool.cuda(),
                      W=w.W.cuda(), act=w.act)
    assert_sum_close(Y.numpy(), ref["Y"], ref["Y_abs"], TOL_F32, f"streamed pooled layer, {agg}")
    # Figure 9: the two-term ApplyVertex needs the interval's own rows
    c = si.commnet_workload(scale=12, f_in=48, f_out=20)
    gc = c.graph
    graph2 = ctx.graph_create_csc(gc.n, gc.col_ptr, gc.row_idx)
    refc = run_oracle(c, agg=agg)
    Yc = torch.full((gc.n, 20), float("nan")).pin_memory()
    ctx.layer_forward(graph2, c.X.clone().pin_memory(), Yc, edge_op="copy", agg=agg, W=c.W.cuda(), W_self=c.W_self.cuda(), act=c.act)
    assert_sum_close(Yc.numpy(), refc["Y"], refc["Y_abs"], TOL_F32, f"streamed CommNet layer, {agg}")
    ctx.destroy()


def test_streamed_apps_respect_the_budget_over_repeated_calls():
    """The per-vertex products of gated and pooled layers are formed on the device inside the chunk schedule, through
    buffers of their own; together with the schedule's buffers they have to stay under the budget, call after call."""
    import paper_1810_08403_amd as saga
    budget = 8 << 20
    ctx = saga.Context(0, hbm_budget_bytes=budget)
    w = si.mpgcn_workload(scale=13, f_in=64, f_pool=96, f_out=32)
    g = w.graph
    graph = ctx.graph_create_csc(g.n, g.col_ptr, g.row_idx)
    ref = run_oracle(w, agg="max", hoisted=True)
    X = w.X.clone().pin_memory()
    for rep in range(3):
        Y = torch.full((g.n, 32), float("nan")).pin_memory()
        ctx.layer_forward(graph, X, Y, edge_op="pool", agg="max", W_pool=w.W_pool.cuda(), b_pool=w.b_pool.cuda(), W=w.W.cuda(), act=w.act)
        assert_sum_close(Y.numpy(), ref["Y"], ref["Y_abs"], TOL_F32, f"pooled layer under {budget >> 20} MiB, call {rep}")
        assert ctx.peak_device_bytes() <= budget, (ctx.peak_device_bytes(), budget)
    wg = si.workload(4, scale=13, f_in=64, f_out=32)
    gg = wg.graph
    graph2 = ctx.graph_create_csc(gg.n, gg.col_ptr, gg.row_idx)
    refg = run_oracle(wg, agg="sum", hoisted=True)
    Xg = wg.X.clone().pin_memory()
    for rep in range(2):
        Yg = torch.full((gg.n, 32), float("nan")).pin_memory()
        ctx.layer_forward(graph2, Xg, Yg, edge_op="gated", W_gate=wg.W_gate.cuda(), b_gate=wg.b_gate.cuda(), W_msg=wg.W_msg.cuda(),
                          W=wg.W.cuda(), act=wg.act)
        assert_sum_close(Yg.numpy(), refg["Y"], refg["Y_abs"], TOL_F32, f"gated layer under {budget >> 20} MiB, call {rep}")
        assert ctx.peak_device_bytes() <= budget, (ctx.peak_device_bytes(), budget)
    t = ctx.get_timings()
    assert t["plan_dst_intervals"] * t["plan_src_intervals"] > 1
    ctx.destroy()


def test_forward_and_backward_alternate_under_one_budget():
    """A training step calls the forward and the backward pass on the same context: the backward pass needs more room
    per vertex than the forward pass, so the tiling and the buffers the forward call left behind may not simply be
    kept. Both results stay right and the allocation high-water mark stays under the budget."""
    import oracle
    import paper_1810_08403_amd as saga
    wl = si.commnet_workload(scale=13, f_in=48, f_out=40)
    g = wl.graph
    n, F = wl.X.shape
    Fo = wl.W.shape[1]
    cp, ri = g.col_ptr.numpy(), g.row_idx.numpy()
    dY = si.normal_features(n, Fo, 5)
    fwd = oracle.layer(cp, ri, wl.X.numpy(), "copy", W=wl.W.numpy(), W_self=wl.W_self.numpy(), act="relu")
    bwd = oracle.layer_backward(cp, ri, wl.X.numpy(), fwd["A"], dY.numpy(), wl.W.numpy(), "copy", W_self=wl.W_self.numpy(), act="relu")
    budget = 6 << 20
    ctx = saga.Context(0, hbm_budget_bytes=budget)
    graph = ctx.graph_create_csc(n, g.col_ptr, g.row_idx)
    pin = lambda a: torch.as_tensor(np.ascontiguousarray(a), dtype=torch.float32).pin_memory()
    X_h, A_h, Y_ref_h, dY_h = wl.X.clone().pin_memory(), pin(fwd["A"]), pin(fwd["Y"]), pin(dY.numpy())
    W, Ws = wl.W.cuda(), wl.W_self.cuda()
    plans = []
    for rep in range(2):
        Y_h = torch.full((n, Fo), float("nan")).pin_memory()
        ctx.layer_forward(graph, X_h, Y_h, edge_op="copy", W=W, W_self=Ws, act="relu")
        t = ctx.get_timings()
        plans.append((t["plan_dst_intervals"], t["plan_src_intervals"]))
        assert_sum_close(Y_h.numpy(), fwd["Y"], fwd["Y_abs"], TOL_F32, f"forward, call {rep}")
        assert ctx.peak_device_bytes() <= budget, ("forward", rep, ctx.peak_device_bytes(), budget)
        dX_h = torch.full((n, F), float("nan")).pin_memory()
        dW, dWs = torch.full((F, Fo), float("nan"), device="cuda"), torch.full((F, Fo), float("nan"), device="cuda")
        ctx.layer_backward(graph, A_h, dY_h, W, dW, dX=dX_h, X=X_h, Y=Y_ref_h, edge_op="copy", act="relu", W_self=Ws, dW_self=dWs)
        t = ctx.get_timings()
        plans.append((t["plan_dst_intervals"], t["plan_src_intervals"]))
        assert_sum_close(dX_h.numpy(), bwd["dX"], bwd["dX_abs"], TOL_F32, f"backward dX, call {rep}")
        assert_sum_close(dW.cpu().numpy(), bwd["dW"], bwd["dW_abs"], TOL_F32, f"backward dW, call {rep}")
        assert_sum_close(dWs.cpu().numpy(), bwd["dW_self"], bwd["dW_self_abs"], TOL_F32, f"backward dW_self, call {rep}")
        assert ctx.peak_device_bytes() <= budget, ("backward", rep, ctx.peak_device_bytes(), budget, plans)
    assert all(q * p > 1 for q, p in plans), plans
    ctx.destroy()


@pytest.mark.parametrize("schedule", [0, 1, 2])
def test_source_intervals_without_out_edges(schedule):
    """Whole source intervals may have no out-edges (the schedule then skips them). With the destination order
    innermost a source buffer is then reused one step after the kernels that last read it, not two."""
    import dataclasses
    wl0 = si.workload(5, scale=12, edge_factor=24, f_in=32, f_out=24)
    g0 = wl0.graph
    n, P = g0.n, 8
    Sp = (n + P - 1) // P
    dst = g0.dst_of_edges()
    src = g0.row_idx.long()
    keep = ~torch.isin(torch.div(src, Sp, rounding_mode="floor"), torch.tensor([2, 4, 7]))
    g = si.build_csc(n, src[keep], dst[keep])
    wl = dataclasses.replace(wl0, graph=g, edge_weight=si.gcn_edge_weights(g0)[keep].contiguous())
    assert g.nnz == int(keep.sum())
    with new_context(dst_intervals=2, src_intervals=P, schedule=schedule) as ctx:
        graph = ctx.graph_create_csc(n, g.col_ptr, g.row_idx)
        graph.set_edge_data(wl.edge_weight)
        for rep in range(2):
            ref_max = run_oracle(wl, agg="max", with_vertex=False)
            A = _streamed(ctx, wl, graph, "max", with_vertex=False)
            assert_bit_equal(A, ref_max["A"], f"max Gather, schedule {schedule}, call {rep}")
            ref = run_oracle(wl, agg="sum")
            Y = _streamed(ctx, wl, graph, "sum")
            assert_sum_close(Y, ref["Y"], ref["Y_abs"], TOL_F32, f"sum layer, schedule {schedule}, call {rep}")


@pytest.mark.parametrize("edge_op,agg,act,Q,P", [("copy", "max", "relu", 2, 3), ("mul_weight", "max", "sigmoid", 1, 4),
                                                 ("pool", "max", "relu", 2, 2), ("gated", "sum", "relu", 2, 3),
                                                 ("gated", "sum", "sigmoid", 1, 2)])
def test_streamed_backward_own_product_in_every_layer_program(edge_op, agg, act, Q, P):
    """Y = act(A W + X W_self + b) with a max Gather, pooled or gated messages, backwards from host memory: dW_self is
    added tile by tile with the other ApplyVertex gradients, and dZ W_self^T joins dX inside the schedule's last
    product (beside the identity for a plain max Gather, W_pool for pooled rows, [W_gs; W_m] and W_gd for gated ones)."""
    import oracle
    import paper_1810_08403_amd as saga
    pool, gated = edge_op == "pool", edge_op == "gated"
    if pool:
        wl = si.mpgcn_workload(scale=11, f_in=16, f_pool=32, f_out=24)
        wl.X = torch.round(wl.X.clamp(-1, 1) * 4) / 4          # coarse values, see the pooled max test above
        wl.W_pool = torch.round((wl.W_pool * 4).clamp(-0.5, 0.5) * 8) / 8
        wl.b_pool = torch.round(wl.b_pool.clamp(-0.5, 0.5) * 8) / 8
    elif gated:
        wl = si.workload(4, scale=11, f_in=20, f_out=12)
    else:
        wl = si.commnet_workload(scale=11, f_in=40, f_out=24)
    g = wl.graph
    n, F = wl.X.shape
    Fm, Fo = wl.W.shape
    cp, ri = g.col_ptr.numpy(), g.row_idx.numpy()
    W_self = si.glorot_uniform(F, Fo, 77)
    w = si.uniform_pm(g.nnz, 1.0, 17) if edge_op == "mul_weight" else None
    dY = si.normal_features(n, Fo, 31)
    bias = si.uniform_pm(Fo, 0.3, 3)
    okw, kw = {}, dict(edge_op=edge_op, agg=agg, act=act, bias=bias.cuda(), W_self=W_self.cuda())
    if w is not None:
        okw["edge_weight"] = w.numpy()
    if pool:
        okw.update(W_pool=wl.W_pool.numpy(), b_pool=wl.b_pool.numpy())
        kw.update(W_pool=wl.W_pool.cuda(), b_pool=wl.b_pool.cuda())
    if gated:
        okw.update(W_gate=wl.W_gate.numpy(), b_gate=wl.b_gate.numpy(), W_msg=wl.W_msg.numpy())
        kw.update(W_gate=wl.W_gate.cuda(), b_gate=wl.b_gate.cuda(), W_msg=wl.W_msg.cuda())
    fwd = oracle.layer(cp, ri, wl.X.numpy(), edge_op, agg=agg, W=wl.W.numpy(), W_self=W_self.numpy(), bias=bias.numpy(), act=act, **okw)
    if gated:
        bwd = oracle.gated_backward(cp, ri, wl.X.numpy(), fwd["A"], dY.numpy(), wl.W.numpy(), bias=bias.numpy(), act=act,
                                    W_self=W_self.numpy(), **okw)
    else:
        bwd = oracle.max_backward(cp, ri, wl.X.numpy(), dY.numpy(), wl.W.numpy(), edge_op, bias=bias.numpy(), act=act,
                                  W_self=W_self.numpy(), **okw)
    ctx = saga.Context(0)
    for name, val in (("dst_intervals", Q), ("src_intervals", P), ("bwd_tile_rows", 600)):
        ctx.set_option(name, val)
    graph = ctx.graph_create_csc(n, g.col_ptr, g.row_idx)
    if w is not None:
        graph.set_edge_data(w)
    X_h = wl.X.clone().pin_memory()
    Y_h, A_h = torch.empty(n, Fo).pin_memory(), torch.empty(n, Fm).pin_memory()
    if pool:   # the device's own pooled rows decide the maxima (see the pooled max test above)
        with new_context() as c2:
            g2 = c2.graph_create_csc(n, g.col_ptr.cuda(), g.row_idx.cuda())
            Yd, Ad = torch.empty(n, Fo, device="cuda"), torch.empty(n, Fm, device="cuda")
            c2.layer_forward(g2, wl.X.cuda(), Yd, W=wl.W.cuda(), accum_out=Ad, **kw)
            torch.cuda.synchronize()
            A_h.copy_(Ad.cpu())
            Y_h.copy_(Yd.cpu())
            g2.destroy()
    else:
        A_h.copy_(torch.as_tensor(fwd["A"], dtype=torch.float32))
        Y_h.copy_(torch.as_tensor(fwd["Y"], dtype=torch.float32))
    dY_h = dY.clone().pin_memory()
    dX_h = torch.full((n, F), float("nan")).pin_memory()
    nan = lambda *s: torch.full(s, float("nan"), device="cuda")
    out = dict(dW=nan(Fm, Fo), dbias=nan(Fo), dW_self=nan(F, Fo))
    if pool:
        out.update(dW_pool=nan(Fm, F), db_pool=nan(Fm))
    if gated:
        out.update(dW_gate=nan(F, 2 * F), db_gate=nan(F), dW_msg=nan(F, F))
    for rep, want_dx in enumerate([True, False, True]):
        for t in out.values():
            t.fill_(float("nan"))
        dX_h.fill_(float("nan"))
        rest = {k: v for k, v in out.items() if k != "dW"}
        ctx.layer_backward(graph, A_h, dY_h, wl.W.cuda(), out["dW"], X=X_h, Y=Y_h, dX=dX_h if want_dx else None, **rest, **kw)
        what = f"streamed backward with W_self, {edge_op} {agg} {act} {Q}x{P} call {rep}"
        for name, got in out.items():
            assert_sum_close(got.cpu().numpy(), bwd[name], np.maximum(bwd[name + "_abs"], 1e-30), TOL_F32, what + " " + name)
        if want_dx:
            assert_sum_close(dX_h.numpy(), bwd["dX"], bwd["dX_abs"], TOL_F32, what + " dX")
    ctx.destroy()


@pytest.mark.parametrize("app", ["gated", "pool"])
def test_streamed_products_never_cross_the_host_link(app):
    """Gated and pooled layers from host memory: the per-vertex products are formed on the device from the rows of X,
    so what crosses the link is X once per destination interval (plus, for a gated layer, once more for the
    destination parts), the edge chunks and Y: not the two to three times wider products."""
    import paper_1810_08403_amd as saga
    Q, P = 2, 3
    if app == "gated":
        wl = si.workload(4, scale=12, f_in=32, f_out=24)
        kw = dict(edge_op="gated", W_gate=wl.W_gate.cuda(), b_gate=wl.b_gate.cuda(), W_msg=wl.W_msg.cuda())
        ref = run_oracle(wl, agg="sum", hoisted=True)
        x_passes = Q + 1
    else:
        wl = si.mpgcn_workload(scale=12, f_in=32, f_pool=96, f_out=24)
        kw = dict(edge_op="pool", agg="max", W_pool=wl.W_pool.cuda(), b_pool=wl.b_pool.cuda())
        ref = run_oracle(wl, agg="max", hoisted=True)
        x_passes = Q
    g = wl.graph
    n, F = wl.X.shape
    with new_context(dst_intervals=Q, src_intervals=P) as ctx:
        graph = ctx.graph_create_csc(n, g.col_ptr, g.row_idx)
        Y = torch.full((n, 24), float("nan")).pin_memory()
        ctx.reset_timings()
        ctx.layer_forward(graph, wl.X.clone().pin_memory(), Y, W=wl.W.cuda(), act=wl.act, **kw)
        t = ctx.get_timings()
        assert_sum_close(Y.numpy(), ref["Y"], ref["Y_abs"], TOL_F32, f"streamed {app} layer")
        x_bytes = n * F * 4
        chunk_bytes = g.nnz * 4 + 64 * (g.nnz // 16 + n) + Q * P * 4096     # ids, a generous bound on work items, padding
        assert t["bytes_d2h"] == n * 24 * 4, t
        assert x_passes * x_bytes <= t["bytes_h2d"] <= x_passes * x_bytes + chunk_bytes, (t["bytes_h2d"], x_bytes, chunk_bytes)

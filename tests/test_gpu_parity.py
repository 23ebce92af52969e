"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by element."""
import numpy as np
import pytest
import torch

import saga_inputs as si
from helpers import (TOL_BF16, TOL_F32, assert_bit_equal, assert_sum_close, make_graph, new_context, run_gpu,
                     run_oracle)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    import paper_1810_08403_amd as saga
    c = saga.Context(0)
    yield c
    c.destroy()


def _check_layer(ctx, wl, agg="sum", bias=None, tol=None, hoisted=False):
    tol = tol or (TOL_BF16 if wl.dtype == "bf16" else TOL_F32)
    graph = make_graph(ctx, wl.graph)
    Y, A = run_gpu(ctx, wl, graph, agg=agg, bias=bias)
    ref = run_oracle(wl, agg=agg, bias=bias, hoisted=hoisted)
    if agg == "max" and wl.edge_op != "gated":
        assert_bit_equal(A, ref["A"], f"{wl.name} max Gather")
    else:
        assert_sum_close(A, ref["A"], ref["A_abs"], TOL_F32, f"{wl.name} Gather")
    assert_sum_close(Y, ref["Y"], ref["Y_abs"], tol, f"{wl.name} layer")
    graph.destroy()
    return Y, A


def test_config1_uniform_gcn(ctx):
    wl = si.workload(1)
    Y, _ = _check_layer(ctx, wl)
    assert (Y >= 0).all()


def test_config1_with_bias_and_no_activation(ctx):
    wl = si.workload(1)
    wl.act = "none"
    _check_layer(ctx, wl, bias=si.uniform_pm(64, 0.5, 9))


def test_config2_two_layers_scaled(ctx):
    wl = si.workload(2, scale=13)
    graph = make_graph(ctx, wl.graph)
    Y1, A1 = run_gpu(ctx, wl, graph)
    ref1 = run_oracle(wl)
    assert_sum_close(A1, ref1["A"], ref1["A_abs"], TOL_F32, "layer 1 Gather (F = 500)")
    assert_sum_close(Y1, ref1["Y"], ref1["Y_abs"], TOL_F32, "layer 1")
    # layer 2 takes the GPU's layer-1 output on both sides, so only layer 2 is compared
    H = torch.from_numpy(Y1)
    Y2, A2 = run_gpu(ctx, wl, graph, X=H, W=wl.extra["W2"], act="none")
    ref2 = run_oracle(wl, X=H, W=wl.extra["W2"], act="none")
    assert Y2.shape[1] == 3
    assert_sum_close(A2, ref2["A"], ref2["A_abs"], TOL_F32, "layer 2 Gather (F = 16)")
    assert_sum_close(Y2, ref2["Y"], ref2["Y_abs"], TOL_F32, "layer 2 (16 -> 3)")
    graph.destroy()


def test_config3_bf16_scaled_with_heavy_columns(ctx):
    wl = si.workload(3, scale=12, edge_factor=100)
    assert wl.graph.in_degree().max().item() > 1024      # some columns are split into sub-groups
    _check_layer(ctx, wl)


def test_config3_bf16_ragged_widths(ctx):
    wl = si.workload(3, scale=10, edge_factor=30, f_in=136, f_out=40)
    _check_layer(ctx, wl)
    wl = si.workload(3, scale=10, edge_factor=30, f_in=37, f_out=5)   # rows not 16-byte multiples
    _check_layer(ctx, wl)


@pytest.mark.parametrize("b,wm", [(True, True), (False, False), (True, False), (False, True)])
def test_config4_gated_scaled(ctx, b, wm):
    wl = si.workload(4, scale=12)
    if not b:
        wl.b_gate = None
    if not wm:
        wl.W_msg = None
    _check_layer(ctx, wl, hoisted=True)


def test_gated_small_widths_against_naive_oracle(ctx):
    for F in (4, 8, 20, 7):
        wl = si.workload(4, scale=9, f_in=F, f_out=6)
        _check_layer(ctx, wl, hoisted=False)


@pytest.mark.parametrize("F", [1, 3, 4, 16, 17, 64, 100, 128, 256, 500, 1028])
@pytest.mark.parametrize("agg", ["sum", "max"])
def test_gather_widths_and_both_accumulators(ctx, F, agg):
    wl = si.workload(5, scale=10, edge_factor=24, f_in=F, f_out=8)   # directed R-MAT, heavy column 0
    graph = make_graph(ctx, wl.graph)
    Y, A = run_gpu(ctx, wl, graph, agg=agg)
    ref = run_oracle(wl, agg=agg)
    if agg == "max":
        assert_bit_equal(A, ref["A"], f"max F={F}")
    else:
        assert_sum_close(A, ref["A"], ref["A_abs"], TOL_F32, f"sum F={F}")
    assert_sum_close(Y, ref["Y"], ref["Y_abs"], TOL_F32, f"layer F={F}")
    graph.destroy()


@pytest.mark.parametrize("F", [72, 128, 136, 200, 256, 264, 384, 512])
@pytest.mark.parametrize("op", ["copy", "mul_weight"])
def test_bf16_sums_on_the_matrix_unit_and_on_the_vector_alus(F, op):
    """bf16 rows of 9..64 fragments (4 or 2 edges side by side in a wavefront, or one): the propagation kernel that accumulates with MFMA (option mma = 1) and the
    one that accumulates with FMAs (mma = 0), both against the oracle at the fp32 bar (edge weights enter the MFMA
    as two bf16 parts, 2^-18 relative). Empty columns, cut columns and item tails of every length 1..7 occur."""
    wl = si.workload(4, scale=12, edge_factor=48, f_in=F, f_out=16)      # no self-loops: empty columns
    wl.edge_op, wl.dtype = op, "bf16"
    wl.edge_weight = si.normal(5, 8, wl.graph.nnz) if op == "mul_weight" else None   # signed weights
    wl.X, wl.W = si.round_to_bf16(wl.X), si.round_to_bf16(wl.W)
    deg = wl.graph.in_degree()
    assert (deg == 0).any() and deg.max().item() > 1024 and len(set((deg % 8).tolist())) == 8
    ref = run_oracle(wl, with_vertex=False)
    for mma in (1, 0):
        with new_context(mma=mma) as c:
            graph = make_graph(c, wl.graph)
            _, A = run_gpu(c, wl, graph, with_vertex=False)
            assert_sum_close(A, ref["A"], ref["A_abs"], TOL_F32, f"bf16 sum F={F} {op} mma={mma}")
            assert not A[(deg == 0).numpy()].any()
            graph.destroy()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("op", ["copy", "mul_weight"])
def test_max_gather_is_bit_exact_with_split_and_empty_columns(ctx, dtype, op):
    wl = si.workload(4, scale=12, edge_factor=48, f_in=64, f_out=16)      # no self-loops: empty columns
    wl.edge_op, wl.dtype = op, dtype
    wl.edge_weight = si.normal(5, 8, wl.graph.nnz) if op == "mul_weight" else None   # signed weights
    if dtype == "bf16":
        wl.X, wl.W = si.round_to_bf16(wl.X), si.round_to_bf16(wl.W)
    deg = wl.graph.in_degree()
    assert (deg == 0).any() and deg.max().item() > 1024
    graph = make_graph(ctx, wl.graph)
    _, A = run_gpu(ctx, wl, graph, agg="max")
    ref = run_oracle(wl, agg="max", with_vertex=False)
    assert_bit_equal(A, ref["A"], f"max {op} {dtype}")
    assert not A[(deg == 0).numpy()].any()
    graph.destroy()


def test_in_degree_invariant(ctx):
    for k, kw in ((1, {}), (4, dict(scale=14)), (3, dict(scale=11, edge_factor=200))):
        wl = si.workload(k, **kw)
        wl.edge_op, wl.dtype = "copy", "f32"
        graph = make_graph(ctx, wl.graph)
        ones = torch.ones(wl.graph.n, 8)
        _, A = run_gpu(ctx, wl, graph, X=ones, with_vertex=False)
        deg = wl.graph.in_degree().numpy().astype(np.float32)
        assert np.array_equal(A, np.repeat(deg[:, None], 8, 1))
        graph.destroy()


def test_runs_are_bitwise_reproducible(ctx):
    wl = si.workload(3, scale=12, edge_factor=100)
    graph = make_graph(ctx, wl.graph)
    Y1, A1 = run_gpu(ctx, wl, graph)
    Y2, A2 = run_gpu(ctx, wl, graph)
    assert np.array_equal(A1.view(np.uint32), A2.view(np.uint32)) and np.array_equal(Y1, Y2)
    graph.destroy()


def test_split_threshold_and_xcd_remap_do_not_change_max(ctx):
    wl = si.workload(5, scale=11, edge_factor=32, f_in=32, f_out=8)
    ref = run_oracle(wl, agg="max", with_vertex=False)
    refs = run_oracle(wl, agg="sum", with_vertex=False)
    for split, remap, team, stripe, order in ((64, 1, 1, 1024, 1), (300, 0, 0, 0, 1), (1 << 20, 1, 1, 64, 0), (16, 1, 1, 16, 1), (32, 0, 0, 256, 0),
                                              (16, 1, 0, 1024, 1), (16, 1, 0, 16, 0)):
        with new_context(split=split, xcd_remap=remap, team=team, stripe_kb=stripe, piece_order=order) as c:
            graph = make_graph(c, wl.graph)
            _, A = run_gpu(c, wl, graph, agg="max", with_vertex=False)
            assert_bit_equal(A, ref["A"], f"split={split}")
            _, A = run_gpu(c, wl, graph, agg="sum", with_vertex=False)
            assert_sum_close(A, refs["A"], refs["A_abs"], TOL_F32, f"split={split}")


def test_degenerate_graphs(ctx):
    base = si.workload(1)
    def wl_for(g, F=5, Fo=3, op="copy"):
        import copy
        w = copy.copy(base)
        w.graph, w.edge_op = g, op
        w.X = si.normal_features(g.n, F, 11)
        w.W = si.glorot_uniform(F, Fo, 12)
        w.edge_weight = si.normal(13, 1, g.nnz) if op == "mul_weight" else None
        return w
    # no edges: Gather gives zeros, the layer gives act(bias)
    wl = wl_for(si.csc_from_lists(7, []))
    graph = make_graph(ctx, wl.graph)
    bias = torch.tensor([0.25, -1.0, 2.0])
    Y, A = run_gpu(ctx, wl, graph, bias=bias)
    assert not A.any() and np.array_equal(Y, np.tile([0.25, 0.0, 2.0], (7, 1)).astype(np.float32))
    graph.destroy()
    # one vertex, one self-loop
    wl = wl_for(si.csc_from_lists(1, [(0, 0)]))
    graph = make_graph(ctx, wl.graph)
    _, A = run_gpu(ctx, wl, graph)
    assert np.array_equal(A, wl.X.numpy())
    graph.destroy()
    # star into vertex 0 (one column of 5000 edges, split), and a path
    for g in (si.csc_from_lists(5000, [(u, 0) for u in range(5000)]),
              si.csc_from_lists(300, [(v, v + 1) for v in range(299)])):
        for op in ("copy", "mul_weight"):
            wl = wl_for(g, F=24, Fo=4, op=op)
            graph = make_graph(ctx, g)
            for agg in ("sum", "max"):
                Y, A = run_gpu(ctx, wl, graph, agg=agg)
                ref = run_oracle(wl, agg=agg)
                if agg == "max":
                    assert_bit_equal(A, ref["A"])
                else:
                    assert_sum_close(A, ref["A"], ref["A_abs"], TOL_F32)
                assert_sum_close(Y, ref["Y"], ref["Y_abs"], TOL_F32)
            graph.destroy()


def test_strided_tensors(ctx):
    wl = si.workload(1)
    graph = make_graph(ctx, wl.graph)
    n = wl.graph.n
    big = torch.zeros(n, 80, device="cuda")
    big[:, :64] = wl.X.cuda()
    Xv = big[:, :64]                                  # ld = 80
    Yb = torch.zeros(n, 72, device="cuda")
    Yv = Yb[:, :64]
    ctx.layer_forward(graph, Xv, Yv, edge_op="mul_weight", edge_weight=wl.edge_weight.cuda(), W=wl.W.cuda(), act="relu")
    torch.cuda.synchronize()
    ref = run_oracle(wl)
    assert_sum_close(Yv.cpu().numpy(), ref["Y"], ref["Y_abs"], TOL_F32)
    assert not Yb[:, 64:].any()
    graph.destroy()


def test_attached_edge_data_equals_passed_edge_weight(ctx):
    wl = si.workload(1)
    graph = make_graph(ctx, wl.graph)
    Y1, _ = run_gpu(ctx, wl, graph)
    graph.set_edge_data(wl.edge_weight.cuda())
    Xd, Wd = wl.X.cuda(), wl.W.cuda()
    Y2 = torch.empty(wl.graph.n, 64, device="cuda")
    ctx.layer_forward(graph, Xd, Y2, edge_op="mul_weight", W=Wd, act="relu")
    torch.cuda.synchronize()
    assert np.array_equal(Y1, Y2.cpu().numpy())
    graph.destroy()


def test_malformed_graphs_and_arguments_are_rejected(ctx):
    import paper_1810_08403_amd as saga
    cp = torch.tensor([0, 2, 3], dtype=torch.int64, device="cuda")
    def status(fn):
        with pytest.raises(saga.SagaError) as e:
            fn()
        return e.value.status
    BAD_GRAPH, INVALID = 2, 1
    assert status(lambda: ctx.graph_create_csc(2, cp, torch.tensor([1, 0, 1], dtype=torch.int32, device="cuda"))) == BAD_GRAPH   # unsorted column
    assert status(lambda: ctx.graph_create_csc(2, cp, torch.tensor([0, 0, 1], dtype=torch.int32, device="cuda"))) == BAD_GRAPH   # duplicate edge
    assert status(lambda: ctx.graph_create_csc(2, cp, torch.tensor([0, 2, 1], dtype=torch.int32, device="cuda"))) == BAD_GRAPH   # id out of range
    assert status(lambda: ctx.graph_create_csc(2, cp, torch.tensor([0, -1, 1], dtype=torch.int32, device="cuda"))) == BAD_GRAPH
    assert status(lambda: ctx.graph_create_csc(2, torch.tensor([0, 3, 2], dtype=torch.int64, device="cuda"),
                                               torch.tensor([0, 1, 1], dtype=torch.int32, device="cuda"))) == BAD_GRAPH          # col_ptr decreases
    assert status(lambda: ctx.graph_create_csc(2, torch.tensor([1, 2, 3], dtype=torch.int64, device="cuda"),
                                               torch.tensor([0, 1, 1], dtype=torch.int32, device="cuda"))) == BAD_GRAPH          # col_ptr[0] != 0
    g = ctx.graph_create_csc(2, cp, torch.tensor([0, 1, 1], dtype=torch.int32, device="cuda"))
    X = torch.zeros(2, 4, device="cuda")
    assert status(lambda: ctx.layer_forward(g, X, torch.zeros(3, 4, device="cuda"))) == INVALID        # row count
    assert status(lambda: ctx.layer_forward(g, X, torch.zeros(2, 5, device="cuda"))) == INVALID        # width without W
    assert status(lambda: ctx.layer_forward(g, X, torch.zeros(2, 4, device="cuda"), edge_op="mul_weight")) == INVALID   # no weights
    assert status(lambda: ctx.layer_forward(g, X, torch.zeros(2, 4, device="cuda"), W=torch.zeros(5, 4, device="cuda"))) == INVALID
    assert status(lambda: ctx.layer_forward(g, X, torch.zeros(2, 4, device="cuda", dtype=torch.bfloat16))) == INVALID
    g.destroy()


@pytest.mark.parametrize("density", [1e-4, 1e-3, 1e-2, 1e-1])
def test_spmm_microbenchmark_shapes(ctx, density):
    """Section 6.1: 10,000 x 10,000 sparse (density 0.01 % .. 10 %) times 10,000 x 128 dense."""
    wl = si.spmm_workload(density)
    assert wl.graph.n == 10000 and wl.X.shape == (10000, 128)
    assert abs(wl.graph.nnz / 1e8 - density) < 0.05 * density + 2e-6
    graph = make_graph(ctx, wl.graph)
    Y, _ = run_gpu(ctx, wl, graph, with_vertex=False, want_accum=False)
    ref = run_oracle(wl, with_vertex=False)
    assert_sum_close(Y, ref["A"], ref["A_abs"], TOL_F32, f"SpMM density {density}")
    graph.destroy()


@pytest.mark.parametrize("F,dtype", [(512, "bf16"), (64, "f32"), (500, "f32"), (1028, "f32"), (3, "f32"), (2056, "bf16")])
def test_team_mode_matches_the_oracle(F, dtype):
    """Option "team": pieces of cut columns worked by whole workgroups (LDS reduction)."""
    wl = si.workload(5, scale=11, edge_factor=32, f_in=F, f_out=8)
    wl.dtype = dtype
    if dtype == "bf16":
        wl.X, wl.W = si.round_to_bf16(wl.X), si.round_to_bf16(wl.W)
    with new_context(team=1, split=16, stripe_kb=16) as c:      # narrow bands, so that columns really are cut
        graph = make_graph(c, wl.graph)
        for agg in ("sum", "max"):
            _, A = run_gpu(c, wl, graph, agg=agg)
            ref = run_oracle(wl, agg=agg, with_vertex=False)
            if agg == "max":
                assert_bit_equal(A, ref["A"], f"team max F={F}")
            else:
                assert_sum_close(A, ref["A"], ref["A_abs"], TOL_F32, f"team sum F={F}")
        assert graph.info()["n_split_vertices"] > 0


def test_team_mode_gated():
    with new_context(team=1, split=16) as c:
        for F in (128, 256, 20):
            wl = si.workload(4, scale=11, edge_factor=48, f_in=F, f_out=8)
            graph = make_graph(c, wl.graph)
            Y, A = run_gpu(c, wl, graph)
            ref = run_oracle(wl, hoisted=True)
            assert_sum_close(A, ref["A"], ref["A_abs"], TOL_F32, f"team gated F={F}")
            assert_sum_close(Y, ref["Y"], ref["Y_abs"], TOL_F32, f"team gated layer F={F}")
            graph.destroy()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_apply_vertex_product_at_ragged_shapes(ctx, dtype):
    """ApplyVertex alone: on a graph of self-loops the Gather output is X, so Y = act(X W + b) is the dense product
    kernel by itself. Row counts that end in the middle of a tile, K below, at and just above the K-tile width (odd
    and even numbers of K tiles: an odd one is padded with a zero tile), N on both sides of every tile-shape switch."""
    import paper_1810_08403_amd as saga
    n = 3 * 128 + 77
    idx = torch.arange(n, dtype=torch.int64)
    g = si.build_csc(n, idx, idx)
    graph = make_graph(ctx, g)
    tol = TOL_BF16 if dtype == "bf16" else TOL_F32
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    for K, N in [(1, 1), (15, 33), (16, 32), (17, 31), (33, 65), (48, 64), (64, 128), (100, 129), (129, 200), (300, 7), (512, 256), (520, 24)]:
        X = si.normal_features(n, K, 100 + K)
        W = si.glorot_uniform(K, N, 200 + N)
        b = si.uniform_pm(N, 0.5, 300 + N)
        if dtype == "bf16":
            X, W = si.round_to_bf16(X), si.round_to_bf16(W)
        Y = torch.full((n, N), float("nan"), device="cuda", dtype=tdt)
        ctx.layer_forward(graph, X.cuda().to(tdt), Y, edge_op="copy", W=W.cuda().to(tdt), bias=b.cuda(), act="relu")
        torch.cuda.synchronize()
        Zabs = X.double().abs() @ W.double().abs() + b.double().abs()
        ref = torch.relu(X.double() @ W.double() + b.double())
        assert_sum_close(Y.float().cpu().numpy(), ref.numpy(), Zabs.numpy(), tol, f"product {n} x {K} x {N} {dtype}")
    graph.destroy()


def test_bf16_product_at_wide_layer_widths_over_many_rows(ctx):
    """bf16 products with K = 256 and 512 over some 37,000 rows (ApplyVertex of the wide GCN layers: every workgroup walks
    several 32-row tiles with the weights held in registers). ApplyVertex alone on a graph of self-loops: a row count that
    ends inside a tile, N one wavefront's 16 columns, part of a 256-column group, a whole one and two, with and without
    bias, all three activations; K = 128 and N = 40 take the general kernel over the same rows."""
    n = 32768 + 4096 + 19
    idx = torch.arange(n, dtype=torch.int64)
    g = si.build_csc(n, idx, idx)
    graph = make_graph(ctx, g)
    cases = [(512, 256, "relu", True), (256, 512, "none", False), (512, 16, "sigmoid", True), (256, 48, "relu", True),
             (512, 272, "none", True), (256, 256, "relu", False), (512, 40, "relu", True), (128, 256, "relu", True)]
    for K, N, act, with_b in cases:
        X = si.round_to_bf16(si.normal_features(n, K, 100 + K))
        W = si.round_to_bf16(si.glorot_uniform(K, N, 200 + N))
        b = si.uniform_pm(N, 0.5, 300 + N) if with_b else None
        pad = 8 if (K, N) in ((256, 48), (512, 272)) else 0      # two cases write into a view of a wider tensor (ld = N + 8)
        Yb = torch.full((n, N + pad), float("nan"), device="cuda", dtype=torch.bfloat16)
        Y = Yb[:, :N]
        ctx.layer_forward(graph, X.cuda().to(torch.bfloat16), Y, edge_op="copy", W=W.cuda().to(torch.bfloat16),
                          bias=None if b is None else b.cuda(), act=act)
        torch.cuda.synchronize()
        assert torch.isnan(Yb[:, N:]).all()
        Z = X.double() @ W.double() + (0 if b is None else b.double())
        Zabs = X.double().abs() @ W.double().abs() + (0 if b is None else b.double().abs())
        ref = {"relu": torch.relu, "sigmoid": torch.sigmoid, "none": lambda t: t}[act](Z)
        assert_sum_close(Y.float().cpu().numpy(), ref.numpy(), Zabs.numpy(), TOL_BF16, f"bf16 product {n} x {K} x {N} {act}")
    graph.destroy()


def test_apply_vertex_product_at_layer_widths_over_many_rows(ctx):
    """fp32 products with K = 32 ... 128 over some 37,000 rows (the shapes of the hoisted products and of ApplyVertex in the
    128-wide applications: every workgroup walks several output tiles). ApplyVertex alone on a graph of self-loops, as
    above: a row count that ends inside a tile, N below, at and above the 32-column slices and 128-column tiles, with and
    without bias, all three activations."""
    n = 32768 + 4096 + 19
    idx = torch.arange(n, dtype=torch.int64)
    g = si.build_csc(n, idx, idx)
    graph = make_graph(ctx, g)
    cases = [(32, 1, "relu", True), (64, 40, "none", False), (96, 128, "sigmoid", True), (128, 129, "relu", True), (128, 384, "none", True),
             (128, 200, "relu", False), (64, 32, "relu", True), (128, 512, "relu", True), (100, 128, "relu", True)]
    for K, N, act, with_b in cases:
        X = si.normal_features(n, K, 100 + K)
        W = si.glorot_uniform(K, N, 200 + N)
        b = si.uniform_pm(N, 0.5, 300 + N) if with_b else None
        Y = torch.full((n, N), float("nan"), device="cuda")
        ctx.layer_forward(graph, X.cuda(), Y, edge_op="copy", W=W.cuda(), bias=None if b is None else b.cuda(), act=act)
        torch.cuda.synchronize()
        Z = X.double() @ W.double() + (0 if b is None else b.double())
        Zabs = X.double().abs() @ W.double().abs() + (0 if b is None else b.double().abs())
        ref = {"relu": torch.relu, "sigmoid": torch.sigmoid, "none": lambda t: t}[act](Z)
        assert_sum_close(Y.cpu().numpy(), ref.numpy(), Zabs.numpy(), TOL_F32, f"product {n} x {K} x {N} {act}")
    graph.destroy()

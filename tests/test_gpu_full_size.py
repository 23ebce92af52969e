"""Parity at the full sizes of the five configurations, in the launch configuration bench.py
times (default tunables), on sampled destination vertices the oracle computes one by one."""
import numpy as np
import pytest
import torch

import oracle
import saga_inputs as si
from helpers import TOL_BF16, TOL_F32, assert_bit_equal, assert_sum_close

pytestmark = pytest.mark.gpu


def _sample(g, count, seed):
    """Random destination vertices plus the heaviest, an empty (if any) and the last one."""
    rng = np.random.default_rng(seed)
    deg = g.in_degree().cpu().numpy()
    picks = set(rng.choice(g.n, size=count, replace=False).tolist())
    picks.update([int(deg.argmax()), g.n - 1, 0])
    zero = np.nonzero(deg == 0)[0]
    if len(zero):
        picks.add(int(zero[0]))
    return np.array(sorted(picks), dtype=np.int64)


def _source_sample(g, count, seed):
    """Random source vertices plus the one with most out-edges, the one with most in-edges, one without out-edges, the
    first and the last."""
    n = g.n
    od = torch.bincount(g.row_idx.long(), minlength=n).cpu().numpy()
    ind = g.in_degree().cpu().numpy()
    rng = np.random.default_rng(seed)
    picks = set(rng.choice(n, size=count, replace=False).tolist()) | {int(od.argmax()), int(ind.argmax()), 0, n - 1}
    picks.add(int(np.nonzero(od == 0)[0][0]))
    assert od.max() > 10_000
    return np.array(sorted(picks), dtype=np.int64)


def _mpgcn_rmat20_exact_preactivations(device):
    """The max-pooling workload bench.py times (R-MAT 20, 128 -> pool 128 -> 128) with X, W_pool and b_pool on coarse grids
    (multiples of 1/4, 1/8, 1/8): every pooled pre-activation is then a multiple of 1/32 below 9 in magnitude, exact in
    fp32 in any order of summation, and two different ones give sigmoids 3.8e-6 apart or more, so that the fp32 sigmoids
    on the GPU and the fp64 ones in the oracle rank the messages alike, ties included (the maximum is a decision, and
    both sides have to take it on the same values)."""
    wl = si.mpgcn_workload(scale=20, edge_factor=32, f_in=128, f_pool=128, f_out=128, device=device)
    wl.X = torch.round(wl.X.clamp(-1, 1) * 4) / 4
    wl.W_pool = torch.round((wl.W_pool * 8).clamp(-1, 1)) / 8
    wl.b_pool = torch.round(wl.b_pool.clamp(-0.5, 0.5) * 8) / 8
    z = wl.X.double() @ wl.W_pool.double().T + wl.b_pool.double()
    assert z.abs().max().item() <= 9.0 and z.std().item() > 0.5
    return wl


def _oracle_rows(wl, vl, agg, W=None, act=None, X=None, with_vertex=True):
    g = wl.graph
    kw = dict(edge_op=wl.edge_op, agg=agg, vlist=vl)
    if wl.edge_op == "mul_weight":
        kw["edge_weight"] = wl.edge_weight.cpu().numpy()
    if wl.edge_op == "gated":
        kw.update(W_gate=wl.W_gate.cpu().numpy(), b_gate=wl.b_gate.cpu().numpy(), W_msg=wl.W_msg.cpu().numpy())
    if with_vertex:
        kw.update(W=(wl.W if W is None else W).float().cpu().numpy(), act=wl.act if act is None else act)
    Xh = (wl.X if X is None else X).float().cpu().numpy()
    return oracle.layer(g.col_ptr.cpu().numpy(), g.row_idx.cpu().numpy(), Xh, **kw)


def test_config2_full_two_layers():
    import paper_1810_08403_amd as saga
    wl = si.workload(2, device="cuda")
    g = wl.graph
    assert g.n == 131072 and wl.X.shape == (131072, 500)
    ctx = saga.Context(0)
    graph = ctx.graph_create_csc(g.n, g.col_ptr, g.row_idx)
    graph.set_edge_data(wl.edge_weight)
    H = torch.empty(g.n, 16, device="cuda")
    A1 = torch.empty(g.n, 500, device="cuda")
    ctx.layer_forward(graph, wl.X, H, edge_op="mul_weight", W=wl.W, act="relu", accum_out=A1)
    Y = torch.empty(g.n, 3, device="cuda")
    ctx.layer_forward(graph, H, Y, edge_op="mul_weight", W=wl.extra["W2"], act="none")
    torch.cuda.synchronize()
    vl = _sample(g, 1500, 1)
    r1 = _oracle_rows(wl, vl, "sum")
    assert_sum_close(A1[vl].cpu().numpy(), r1["A"], r1["A_abs"], TOL_F32, "layer 1 Gather")
    assert_sum_close(H[vl].cpu().numpy(), r1["Y"], r1["Y_abs"], TOL_F32, "layer 1")
    r2 = _oracle_rows(wl, vl, "sum", W=wl.extra["W2"], act="none", X=H)
    assert_sum_close(Y[vl].cpu().numpy(), r2["Y"], r2["Y_abs"], TOL_F32, "layer 2")
    # in-degree invariant at full size
    ones = torch.ones(g.n, 16, device="cuda")
    D = torch.empty(g.n, 16, device="cuda")
    ctx.layer_forward(graph, ones, D, edge_op="copy")
    torch.cuda.synchronize()
    assert torch.equal(D[:, 0].long(), g.in_degree()) and torch.equal(D[:, 15].long(), g.in_degree())
    ctx.destroy()


def test_config3_full_bf16():
    import paper_1810_08403_amd as saga
    wl = si.workload(3, device="cuda")
    g = wl.graph
    assert g.n == 262144 and g.nnz > 100_000_000
    ctx = saga.Context(0)
    graph = ctx.graph_create_csc(g.n, g.col_ptr, g.row_idx)
    graph.set_edge_data(wl.edge_weight)
    X = wl.X.to(torch.bfloat16)
    W = wl.W.to(torch.bfloat16)
    Y = torch.empty(g.n, 256, device="cuda", dtype=torch.bfloat16)
    A = torch.empty(g.n, 512, device="cuda")
    ctx.layer_forward(graph, X, Y, edge_op="mul_weight", W=W, act="relu", accum_out=A)
    torch.cuda.synchronize()
    vl = _sample(g, 600, 2)
    r = _oracle_rows(wl, vl, "sum")
    assert_sum_close(A[vl].cpu().numpy(), r["A"], r["A_abs"], TOL_F32, "Gather (fp32 accumulate of bf16 rows)")
    assert_sum_close(Y[vl].float().cpu().numpy(), r["Y"], r["Y_abs"], TOL_BF16, "layer (bf16)")
    # the timed configuration (no accum_out) must give the same Y bits
    Y2 = torch.empty_like(Y)
    ctx.layer_forward(graph, X, Y2, edge_op="mul_weight", W=W, act="relu")
    torch.cuda.synchronize()
    assert torch.equal(Y.view(torch.int16), Y2.view(torch.int16))
    # max Gather, bit for bit, on the same graph
    Am = torch.empty(g.n, 512, device="cuda")
    Ym = torch.empty(g.n, 512, device="cuda", dtype=torch.bfloat16)
    ctx.layer_forward(graph, X, Ym, edge_op="mul_weight", agg="max", accum_out=Am)
    torch.cuda.synchronize()
    rm = _oracle_rows(wl, vl[:200], "max", with_vertex=False)
    assert_bit_equal(Am[vl[:200]].cpu().numpy(), rm["A"], "max Gather")
    # the two variants bench.py times beside the headline: the product before the propagation, and the propagation
    # with its multiply-accumulate on the matrix unit
    for option in ("transform_first", "mma"):
        ctx.set_option(option, 1)
        Yv = torch.empty_like(Y)
        Av = torch.empty(g.n, 512, device="cuda") if option == "mma" else None
        ctx.layer_forward(graph, X, Yv, edge_op="mul_weight", W=W, act="relu", accum_out=Av)
        torch.cuda.synchronize()
        ctx.set_option(option, 0)
        assert_sum_close(Yv[vl].float().cpu().numpy(), r["Y"], r["Y_abs"], TOL_BF16, f"layer (bf16) with option {option}")
        if Av is not None:
            assert_sum_close(Av[vl].cpu().numpy(), r["A"], r["A_abs"], TOL_F32, "Gather on the matrix unit")
    ctx.destroy()


def test_config4_full_gated():
    import paper_1810_08403_amd as saga
    wl = si.workload(4, device="cuda")
    g = wl.graph
    assert g.n == 1 << 20 and g.nnz > 25_000_000
    ctx = saga.Context(0)
    graph = ctx.graph_create_csc(g.n, g.col_ptr, g.row_idx)
    Y = torch.empty(g.n, 128, device="cuda")
    A = torch.empty(g.n, 128, device="cuda")
    ctx.layer_forward(graph, wl.X, Y, edge_op="gated", W_gate=wl.W_gate, b_gate=wl.b_gate, W_msg=wl.W_msg,
                      W=wl.W, act="relu", accum_out=A)
    torch.cuda.synchronize()
    vl = _sample(g, 400, 3)          # naive per-edge oracle on the sample
    r = _oracle_rows(wl, vl, "sum")
    assert_sum_close(A[vl].cpu().numpy(), r["A"], r["A_abs"], TOL_F32, "gated Gather")
    assert_sum_close(Y[vl].cpu().numpy(), r["Y"], r["Y_abs"], TOL_F32, "gated layer")
    deg = g.in_degree()
    assert not A[deg == 0].any()
    ctx.destroy()


def test_config4_full_gated_backward():
    """The gated backward pass at configuration 4's full size with default tunables: rows of dX for sampled vertices (the
    one with most out-edges, the one with most in-edges, one without out-edges, random ones) from the oracle's sampled
    form, which needs only those vertices' own edges; the parameter gradients, sums over all million vertices the
    oracle cannot do in seconds, through what holds at any size: they are the same bits whether or not dX is asked for,
    and doubling dY doubles every gradient exactly."""
    import paper_1810_08403_amd as saga
    wl = si.workload(4, device="cuda")
    g = wl.graph
    n, F = wl.X.shape
    ctx = saga.Context(0)
    graph = ctx.graph_create_csc(n, g.col_ptr, g.row_idx)
    Y = torch.empty(n, 128, device="cuda")
    A = torch.empty(n, 128, device="cuda")
    kw = dict(edge_op="gated", W_gate=wl.W_gate, b_gate=wl.b_gate, W_msg=wl.W_msg, act="none")
    ctx.layer_forward(graph, wl.X, Y, W=wl.W, accum_out=A, **kw)
    dY = si.normal_features(n, 128, 31).cuda()
    z = lambda *s: torch.full(s, float("nan"), device="cuda")
    def run(dy, want_dx=True):
        out = dict(dW=z(F, 128), dX=z(n, F) if want_dx else None, dW_gate=z(F, 2 * F), db_gate=z(F), dW_msg=z(F, F))
        ctx.layer_backward(graph, A, dy, wl.W, out["dW"], X=wl.X, dX=out["dX"], dW_gate=out["dW_gate"], db_gate=out["db_gate"],
                           dW_msg=out["dW_msg"], **kw)
        torch.cuda.synchronize()
        return out
    r1 = run(dY)
    od = torch.bincount(g.row_idx.long(), minlength=n).cpu().numpy()
    ind = g.in_degree().cpu().numpy()
    rng = np.random.default_rng(12)
    picks = set(rng.choice(n, size=60, replace=False).tolist()) | {int(od.argmax()), int(ind.argmax()), 0, n - 1}
    picks.add(int(np.nonzero(od == 0)[0][0]))
    ul = np.array(sorted(picks), dtype=np.int64)
    assert od.max() > 10_000
    ref = oracle.gated_backward_sample(g.col_ptr.cpu().numpy(), g.row_idx.cpu().numpy(), wl.X.cpu().numpy(), dY.cpu().numpy(),
                                       wl.W.cpu().numpy(), wl.W_gate.cpu().numpy(), ul, b_gate=wl.b_gate.cpu().numpy(),
                                       W_msg=wl.W_msg.cpu().numpy())
    assert_sum_close(r1["dX"][ul].cpu().numpy(), ref["dX"], ref["dX_abs"], TOL_F32, "configuration 4 full size, sampled rows of dX")
    for name in ("dW", "dW_gate", "db_gate", "dW_msg"):
        assert torch.isfinite(r1[name]).all() and r1[name].abs().max().item() > 0
    r2 = run(dY, want_dx=False)
    r3 = run(dY * 2.0)
    for name in ("dW", "dW_gate", "db_gate", "dW_msg"):
        assert torch.equal(r1[name], r2[name]), name
        assert torch.equal(r3[name], r1[name] * 2.0), name
    assert torch.equal(r3["dX"], r1["dX"] * 2.0)
    ctx.destroy()


def test_config3_full_bf16_backward():
    """Configuration 3 as configured (bf16, 512 -> 256, ReLU) backwards at full size: sampled rows of dX (bf16 bar) and
    sampled entries of dW (fp32 products of values exact in fp32: fp32 bar) from the oracle's sampled form."""
    import paper_1810_08403_amd as saga
    wl = si.workload(3, device="cuda")
    g = wl.graph
    n, F, Fo = g.n, 512, 256
    cp, ri, w = g.col_ptr.cpu().numpy(), g.row_idx.cpu().numpy(), wl.edge_weight.cpu().numpy()
    bf = torch.bfloat16
    W16 = wl.W.to(bf)
    ctx = saga.Context(0)
    graph = ctx.graph_create_csc(n, g.col_ptr, g.row_idx)
    graph.set_edge_data(wl.edge_weight)
    A = si.round_to_bf16(si.normal_features(n, F, 31, device="cuda")).float()     # a synthetic Gather output, taken as given
    Y16 = torch.relu(A.double() @ W16.double()).to(bf)
    dY16 = si.normal_features(n, Fo, 32, device="cuda").to(bf)
    dX = torch.empty(n, F, device="cuda", dtype=bf)
    dW, db = torch.empty(F, Fo, device="cuda"), torch.empty(Fo, device="cuda")
    ctx.layer_backward(graph, A, dY16, W16, dW, Y=Y16, edge_op="mul_weight", act="relu", dX=dX, dbias=db)
    torch.cuda.synchronize()
    rng = np.random.default_rng(5)
    od = torch.bincount(g.row_idx.long(), minlength=n).cpu().numpy()
    ul = np.array(sorted(set(rng.choice(n, size=10, replace=False).tolist()) | {int(od.argmax()), 0, n - 1}), dtype=np.int64)
    we = [(0, 0), (511, 255), (17, 200), (300, 5)]
    # the oracle sees the same bf16-valued dZ: dY masked by the stored bf16 output, handed over as dY without activation
    dZ = (dY16.float() * (Y16.float() > 0)).cpu().numpy()
    ref = oracle.backward_sample(cp, ri, None, A.cpu().numpy(), dZ, W16.float().cpu().numpy(), ul, we, "mul_weight", w, act="none",
                                 want_dbias=True)
    assert_sum_close(dX[ul].float().cpu().numpy(), ref["dX"], ref["dX_abs"], TOL_BF16, "config 3 bf16 backward dX")
    got = np.array([dW[f, o].item() for f, o in we])
    assert_sum_close(got, ref["dW"], ref["dW_abs"], TOL_F32, "config 3 bf16 backward dW")
    assert_sum_close(db.cpu().numpy(), ref["dbias"], np.maximum(ref["dbias_abs"], 1e-30), TOL_F32, "config 3 bf16 backward dbias")
    ctx.destroy()


def test_commnet_rmat20_forward_and_backward():
    """The CommNet layer bench.py times (R-MAT 20, 128 -> 128, W_self, ReLU): sampled rows of the layer from the oracle,
    then sampled rows of dX and entries of dW of its backward pass."""
    import paper_1810_08403_amd as saga
    wl = si.commnet_workload(scale=20, edge_factor=16, f_in=128, f_out=128, device="cuda")
    g = wl.graph
    n = g.n
    cp, ri = g.col_ptr.cpu().numpy(), g.row_idx.cpu().numpy()
    ctx = saga.Context(0)
    graph = ctx.graph_create_csc(n, g.col_ptr, g.row_idx)
    Y, A = torch.empty(n, 128, device="cuda"), torch.empty(n, 128, device="cuda")
    ctx.layer_forward(graph, wl.X, Y, edge_op="copy", W=wl.W, W_self=wl.W_self, act="relu", accum_out=A)
    torch.cuda.synchronize()
    vl = _sample(g, 300, 4)
    Xh, Wh, Wsh = wl.X.cpu().numpy(), wl.W.cpu().numpy(), wl.W_self.cpu().numpy()
    r = oracle.layer(cp, ri, Xh, "copy", W=Wh, W_self=Wsh, act="relu", vlist=vl)
    assert_sum_close(A[vl].cpu().numpy(), r["A"], r["A_abs"], TOL_F32, "CommNet R-MAT 20 Gather")
    assert_sum_close(Y[vl].cpu().numpy(), r["Y"], r["Y_abs"], TOL_F32, "CommNet R-MAT 20 layer")
    dY = si.normal_features(n, 128, 77, device="cuda")
    dX, dW, dWs, db = (torch.empty(n, 128, device="cuda"), torch.empty(128, 128, device="cuda"), torch.empty(128, 128, device="cuda"),
                       torch.empty(128, device="cuda"))
    ctx.layer_backward(graph, A, dY, wl.W, dW, X=wl.X, Y=Y, edge_op="copy", W_self=wl.W_self, act="relu", dX=dX, dbias=db, dW_self=dWs)
    torch.cuda.synchronize()
    rng = np.random.default_rng(9)
    od = torch.bincount(g.row_idx.long(), minlength=n).cpu().numpy()
    ul = np.array(sorted(set(rng.choice(n, size=40, replace=False).tolist()) | {int(od.argmax()), 0, n - 1}), dtype=np.int64)
    we = [(0, 0), (127, 127), (5, 99), (64, 3)]
    # both sides differentiate the layer the GPU computed: its A and its ReLU decisions (dY masked by Y > 0, no activation)
    dZ = (dY * (Y > 0)).cpu().numpy()
    ref = oracle.backward_sample(cp, ri, Xh, A.cpu().numpy(), dZ, Wh, ul, we, "copy", W_self=Wsh, act="none", want_dbias=True)
    assert_sum_close(dX[ul].cpu().numpy(), ref["dX"], ref["dX_abs"], TOL_F32, "CommNet R-MAT 20 dX")
    assert_sum_close(np.array([dW[f, o].item() for f, o in we]), ref["dW"], ref["dW_abs"], TOL_F32, "CommNet R-MAT 20 dW")
    assert_sum_close(db.cpu().numpy(), ref["dbias"], np.maximum(ref["dbias_abs"], 1e-30), TOL_F32, "CommNet R-MAT 20 dbias")
    # dW_self = X^T dZ against the same product in fp64 on the device
    dz64 = (dY * (Y > 0)).double()
    assert_sum_close(dWs.cpu().numpy(), (wl.X.double().T @ dz64).cpu().numpy(), (wl.X.double().abs().T @ dz64.abs()).cpu().numpy(), TOL_F32,
                     "CommNet R-MAT 20 dW_self")
    ctx.destroy()


def test_mpgcn_rmat20_forward_and_backward():
    """The max-pooling GCN layer bench.py times (R-MAT 20, 128 -> pool 128 -> 128, max), with pre-activations exact in fp32:
    sampled rows of the forward pass from the oracle; backwards, sampled rows of dX from the oracle's sampled form (which
    recomputes the maxima of every destination those sources reach), dW and dbias against the same sums in fp64, and
    for dW_pool and db_pool, sums over a million vertices the oracle cannot do in seconds, what holds at any size: the
    same bits with and without dX, exact doubling. The stored output handed to the backward pass is synthetic (only its
    sign is used, for ReLU's derivative), so that the oracle can be given the same mask."""
    import paper_1810_08403_amd as saga
    wl = _mpgcn_rmat20_exact_preactivations("cuda")
    g = wl.graph
    n = g.n
    cp, ri = g.col_ptr.cpu().numpy(), g.row_idx.cpu().numpy()
    ctx = saga.Context(0)
    graph = ctx.graph_create_csc(n, g.col_ptr, g.row_idx)
    Y, A = torch.empty(n, 128, device="cuda"), torch.empty(n, 128, device="cuda")
    kw = dict(edge_op="pool", agg="max", W_pool=wl.W_pool, b_pool=wl.b_pool, act="relu")
    ctx.layer_forward(graph, wl.X, Y, W=wl.W, accum_out=A, **kw)
    torch.cuda.synchronize()
    vl = _sample(g, 300, 6)
    r = oracle.layer(cp, ri, wl.X.cpu().numpy(), "pool", agg="max", W_pool=wl.W_pool.cpu().numpy(), b_pool=wl.b_pool.cpu().numpy(),
                     W=wl.W.cpu().numpy(), act="relu", vlist=vl)
    assert_sum_close(A[vl].cpu().numpy(), r["A"], r["A_abs"], TOL_F32, "MP-GCN R-MAT 20 Gather")
    assert_sum_close(Y[vl].cpu().numpy(), r["Y"], r["Y_abs"], TOL_F32, "MP-GCN R-MAT 20 layer")
    dY = si.normal_features(n, 128, 78, device="cuda")
    Y_in = si.normal_features(n, 128, 79, device="cuda")
    z = lambda *s: torch.full(s, float("nan"), device="cuda")
    def run(dy, want_dx=True):
        out = dict(dW=z(128, 128), dX=z(n, 128) if want_dx else None, dW_pool=z(128, 128), db_pool=z(128), dbias=z(128))
        ctx.layer_backward(graph, A, dy, wl.W, out["dW"], X=wl.X, Y=Y_in, dX=out["dX"], dW_pool=out["dW_pool"], db_pool=out["db_pool"],
                           dbias=out["dbias"], **kw)
        torch.cuda.synchronize()
        return out
    r1, r2, r3 = run(dY), run(dY, want_dx=False), run(dY * 2.0)
    for name in ("dW", "dW_pool", "db_pool", "dbias"):
        assert torch.isfinite(r1[name]).all() and r1[name].abs().max().item() > 0
        assert torch.equal(r1[name], r2[name]), name
        assert torch.equal(r3[name], r1[name] * 2.0), name
    assert torch.equal(r3["dX"], r1["dX"] * 2.0)
    dZ = dY * (Y_in > 0)
    ul = _source_sample(g, 60, 12)
    ref = oracle.max_backward_sample(cp, ri, wl.X.cpu().numpy(), dZ.cpu().numpy(), wl.W.cpu().numpy(), ul, "pool",
                                     W_pool=wl.W_pool.cpu().numpy(), b_pool=wl.b_pool.cpu().numpy(), act="none")
    assert np.abs(ref["dX"]).max() > 1.0
    assert_sum_close(r1["dX"][ul].cpu().numpy(), ref["dX"], np.maximum(ref["dX_abs"], 1e-30), TOL_F32, "MP-GCN R-MAT 20, sampled rows of dX")
    # dW = A^T dZ and dbias against the same sums in fp64 on the device
    dz64 = dZ.double()
    assert_sum_close(r1["dW"].cpu().numpy(), (A.double().T @ dz64).cpu().numpy(), (A.double().abs().T @ dz64.abs()).cpu().numpy(), TOL_F32,
                     "MP-GCN R-MAT 20 dW")
    assert_sum_close(r1["dbias"].cpu().numpy(), dz64.sum(0).cpu().numpy(), dz64.abs().sum(0).cpu().numpy(), TOL_F32, "MP-GCN R-MAT 20 dbias")
    ctx.destroy()


@pytest.mark.parametrize("app", ["config4", "commnet", "mpgcn"])
def test_streamed_applications_under_one_gib_at_full_size(app):
    """The gated, CommNet and max-pooling layers at the sizes bench.py --streamed times them (R-MAT 20), from pinned host
    memory through a 1 GiB device budget: sampled rows against the oracle, and the peak stays under the budget."""
    import paper_1810_08403_amd as saga
    if app == "config4":
        wl = si.workload(4)
    elif app == "commnet":
        wl = si.commnet_workload(scale=20, edge_factor=16, f_in=128, f_out=128)
    else:
        wl = si.mpgcn_workload(scale=20, edge_factor=32, f_in=128, f_pool=128, f_out=128)
    g = wl.graph
    n = g.n
    agg = "max" if app == "mpgcn" else "sum"
    budget = 1 << 30
    ctx = saga.Context(0, hbm_budget_bytes=budget)
    graph = ctx.graph_create_csc(n, g.col_ptr, g.row_idx)
    kw = dict(edge_op=wl.edge_op, agg=agg, W=wl.W.cuda(), act=wl.act)
    okw = dict(edge_op=wl.edge_op, agg=agg, W=wl.W.numpy(), act=wl.act)
    if wl.edge_op == "gated":
        kw.update(W_gate=wl.W_gate.cuda(), b_gate=wl.b_gate.cuda(), W_msg=wl.W_msg.cuda())
        okw.update(W_gate=wl.W_gate.numpy(), b_gate=wl.b_gate.numpy(), W_msg=wl.W_msg.numpy())
    if wl.edge_op == "pool":
        kw.update(W_pool=wl.W_pool.cuda(), b_pool=wl.b_pool.cuda())
        okw.update(W_pool=wl.W_pool.numpy(), b_pool=wl.b_pool.numpy())
    if wl.W_self is not None:
        kw["W_self"] = wl.W_self.cuda()
        okw["W_self"] = wl.W_self.numpy()
    X = wl.X.pin_memory()
    Y = torch.full((n, wl.W.shape[1]), float("nan")).pin_memory()
    for _ in range(2):                      # the second call reuses the chunk grid and the buffers
        ctx.layer_forward(graph, X, Y, **kw)
    torch.cuda.synchronize()
    assert ctx.peak_device_bytes() <= budget
    vl = _sample(g, 200, 8)
    r = oracle.layer(g.col_ptr.numpy(), g.row_idx.numpy(), wl.X.numpy(), vlist=vl, **okw)
    assert_sum_close(Y[vl].numpy(), r["Y"], r["Y_abs"], TOL_F32, f"{app} streamed under 1 GiB")
    assert torch.isfinite(Y).all()
    ctx.destroy()


def test_config4_streamed_gated_backward_under_two_gib():
    """Configuration 4's gated layer backwards from host memory through a 2 GiB device budget: sampled rows of dX against
    the oracle's sampled form, element by element at the fp32 bar; the parameter gradients (sums over all million
    vertices) against the device-resident backward pass of the same layer, whose sampled rows the oracle checks above.
    The stored output handed to both passes is synthetic (only its sign is used, for ReLU's derivative), so that the
    oracle is given the same mask."""
    import paper_1810_08403_amd as saga
    wl = si.workload(4, device="cuda")
    g = wl.graph
    n, F = wl.X.shape
    kw = dict(edge_op="gated", W_gate=wl.W_gate, b_gate=wl.b_gate, W_msg=wl.W_msg, act="relu")
    z = lambda *s: torch.full(s, float("nan"), device="cuda")
    names = ("dW", "dbias", "dW_gate", "db_gate", "dW_msg")
    ctx = saga.Context(0)
    graph = ctx.graph_create_csc(n, g.col_ptr, g.row_idx)
    Y, A = torch.empty(n, 128, device="cuda"), torch.empty(n, 128, device="cuda")
    ctx.layer_forward(graph, wl.X, Y, W=wl.W, accum_out=A, **kw)
    dY = si.normal_features(n, 128, 31).cuda()
    Y_in = si.normal_features(n, 128, 32).cuda()
    ref = dict(dW=z(F, 128), dbias=z(128), dW_gate=z(F, 2 * F), db_gate=z(F), dW_msg=z(F, F), dX=z(n, F))
    ctx.layer_backward(graph, A, dY, wl.W, ref["dW"], X=wl.X, Y=Y_in, dX=ref["dX"], dbias=ref["dbias"], dW_gate=ref["dW_gate"],
                       db_gate=ref["db_gate"], dW_msg=ref["dW_msg"], **kw)
    torch.cuda.synchronize()
    host = {k: v.cpu() for k, v in dict(X=wl.X, A=A, Y=Y_in, dY=dY).items()}
    ref = {k: v.cpu() for k, v in ref.items()}
    ul = _source_sample(g, 60, 12)
    graph.destroy()
    ctx.destroy()
    del Y, A, dY, Y_in
    torch.cuda.empty_cache()
    budget = 2 << 30
    ctx = saga.Context(0, hbm_budget_bytes=budget)
    hg = ctx.graph_create_csc(n, g.col_ptr.cpu(), g.row_idx.cpu())
    pin = lambda t: t.contiguous().pin_memory()
    dX_h = torch.full((n, F), float("nan")).pin_memory()
    got = dict(dW=z(F, 128), dbias=z(128), dW_gate=z(F, 2 * F), db_gate=z(F), dW_msg=z(F, F))
    ctx.layer_backward(hg, pin(host["A"]), pin(host["dY"]), wl.W, got["dW"], X=pin(host["X"]), Y=pin(host["Y"]), dX=dX_h,
                       dbias=got["dbias"], dW_gate=got["dW_gate"], db_gate=got["db_gate"], dW_msg=got["dW_msg"], **kw)
    torch.cuda.synchronize()
    assert ctx.peak_device_bytes() <= budget
    dZ = (host["dY"] * (host["Y"] > 0)).numpy()
    smp = oracle.gated_backward_sample(g.col_ptr.cpu().numpy(), g.row_idx.cpu().numpy(), host["X"].numpy(), dZ, wl.W.cpu().numpy(),
                                       wl.W_gate.cpu().numpy(), ul, b_gate=wl.b_gate.cpu().numpy(), W_msg=wl.W_msg.cpu().numpy())
    assert_sum_close(dX_h[ul].numpy(), smp["dX"], np.maximum(smp["dX_abs"], 1e-30), TOL_F32, "configuration 4 streamed under 2 GiB, sampled rows of dX")
    assert_sum_close(ref["dX"][ul].numpy(), smp["dX"], np.maximum(smp["dX_abs"], 1e-30), TOL_F32, "configuration 4 resident with ReLU, sampled rows of dX")
    for name in names:   # the same sums in another grouping: close in the norm of each tensor
        err = (got[name].cpu().double() - ref[name].double()).abs().max().item()
        assert err <= 1e-4 * ref[name].abs().max().item(), (name, err)
    err = (dX_h.double() - ref["dX"].double()).abs().max().item()
    assert err <= 1e-4 * ref["dX"].abs().max().item(), ("dX", err)
    t = ctx.get_timings()
    print(f"streamed gated backward: {t['ms_wall_streamed']:.0f} ms in the two schedules, H2D {t['bytes_h2d'] / 1e9:.1f} GB, "
          f"D2H {t['bytes_d2h'] / 1e9:.1f} GB, peak {ctx.peak_device_bytes() / 1e9:.2f} GB")
    ctx.destroy()


def test_mpgcn_rmat20_streamed_backward_under_two_gib():
    """The max-pooling layer's backward pass from host memory through a 2 GiB device budget at R-MAT 20 (pre-activations
    exact in fp32, synthetic stored output for ReLU's mask): sampled rows of dX against the oracle's sampled form, element
    by element at the fp32 bar; dW and dbias against the same sums in fp64; dW_pool and db_pool against the
    device-resident backward pass; a vertex gets a gradient exactly where the resident pass gives it one; and the peak
    stays under the budget."""
    import paper_1810_08403_amd as saga
    wl = _mpgcn_rmat20_exact_preactivations("cuda")
    g = wl.graph
    n = g.n
    kw = dict(edge_op="pool", agg="max", W_pool=wl.W_pool, b_pool=wl.b_pool, act="relu")
    z = lambda *s: torch.full(s, float("nan"), device="cuda")
    ctx = saga.Context(0)
    graph = ctx.graph_create_csc(n, g.col_ptr, g.row_idx)
    Y, A = torch.empty(n, 128, device="cuda"), torch.empty(n, 128, device="cuda")
    ctx.layer_forward(graph, wl.X, Y, W=wl.W, accum_out=A, **kw)
    dY = si.normal_features(n, 128, 78, device="cuda")
    Y_in = si.normal_features(n, 128, 79, device="cuda")
    ref = dict(dW=z(128, 128), dX=z(n, 128), dW_pool=z(128, 128), db_pool=z(128), dbias=z(128))
    ctx.layer_backward(graph, A, dY, wl.W, ref["dW"], X=wl.X, Y=Y_in, dX=ref["dX"], dW_pool=ref["dW_pool"], db_pool=ref["db_pool"],
                       dbias=ref["dbias"], **kw)
    torch.cuda.synchronize()
    host = {k: v.cpu() for k, v in dict(X=wl.X, A=A, Y=Y_in, dY=dY).items()}
    ref = {k: v.cpu() for k, v in ref.items()}
    ul = _source_sample(g, 60, 12)
    graph.destroy()
    ctx.destroy()
    del Y, A, dY, Y_in
    torch.cuda.empty_cache()
    budget = 2 << 30
    ctx = saga.Context(0, hbm_budget_bytes=budget)
    hg = ctx.graph_create_csc(n, g.col_ptr.cpu(), g.row_idx.cpu())
    pin = lambda t: t.contiguous().pin_memory()
    dX_h = torch.full((n, 128), float("nan")).pin_memory()
    got = dict(dW=z(128, 128), dW_pool=z(128, 128), db_pool=z(128), dbias=z(128))
    ctx.layer_backward(hg, pin(host["A"]), pin(host["dY"]), wl.W, got["dW"], X=pin(host["X"]), Y=pin(host["Y"]), dX=dX_h,
                       dW_pool=got["dW_pool"], db_pool=got["db_pool"], dbias=got["dbias"], **kw)
    torch.cuda.synchronize()
    assert ctx.peak_device_bytes() <= budget
    dZ = host["dY"] * (host["Y"] > 0)
    smp = oracle.max_backward_sample(g.col_ptr.cpu().numpy(), g.row_idx.cpu().numpy(), host["X"].numpy(), dZ.numpy(), wl.W.cpu().numpy(), ul,
                                     "pool", W_pool=wl.W_pool.cpu().numpy(), b_pool=wl.b_pool.cpu().numpy(), act="none")
    assert np.abs(smp["dX"]).max() > 1.0
    assert_sum_close(dX_h[ul].numpy(), smp["dX"], np.maximum(smp["dX_abs"], 1e-30), TOL_F32, "MP-GCN streamed under 2 GiB, sampled rows of dX")
    dz64, A64 = dZ.double(), host["A"].double()
    assert_sum_close(got["dW"].cpu().numpy(), (A64.T @ dz64).numpy(), (A64.abs().T @ dz64.abs()).numpy(), TOL_F32, "MP-GCN streamed dW")
    assert_sum_close(got["dbias"].cpu().numpy(), dz64.sum(0).numpy(), dz64.abs().sum(0).numpy(), TOL_F32, "MP-GCN streamed dbias")
    # the same sums in another grouping: close in the norm of each tensor
    for name in ("dW", "dW_pool", "db_pool", "dbias"):
        err = (got[name].cpu().double() - ref[name].double()).abs().max().item()
        assert err <= 1e-4 * ref[name].abs().max().item(), (name, err)
    err = (dX_h.double() - ref["dX"].double()).abs().max().item()
    assert err <= 1e-4 * ref["dX"].abs().max().item(), ("dX", err)
    # a vertex gets a gradient exactly where the resident pass gives it one
    assert torch.equal(dX_h.abs().sum(1) > 0, ref["dX"].abs().sum(1) > 0)
    ctx.destroy()


@pytest.mark.parametrize("agg", ["sum", "max"])
def test_config5_full_streamed_under_16gb(agg):
    import paper_1810_08403_amd as saga
    if not hasattr(test_config5_full_streamed_under_16gb, "wl"):
        wl = si.workload(5, device="cuda")
        g = wl.graph
        host = si.CSC(g.n, g.col_ptr.cpu(), g.row_idx.cpu())
        test_config5_full_streamed_under_16gb.wl = (wl.X.cpu().pin_memory(), wl.W.clone(), wl.edge_weight.cpu(), host)
        del wl, g
        torch.cuda.empty_cache()
    X, W, w, g = test_config5_full_streamed_under_16gb.wl
    assert g.n == 1 << 23 and X.shape == (1 << 23, 256) and g.nnz > 400_000_000
    budget = 16 * (1 << 30)
    ctx = saga.Context(0, hbm_budget_bytes=budget)
    graph = ctx.graph_create_csc(g.n, g.col_ptr, g.row_idx)
    graph.set_edge_data(w)
    Y = torch.empty(g.n, 256).pin_memory()
    ctx.layer_forward(graph, X, Y, edge_op="mul_weight", agg=agg, W=W, act="relu")
    t = ctx.get_timings()
    assert ctx.peak_device_bytes() <= budget
    print(f"config5 {agg}: plan {t['plan_dst_intervals']} x {t['plan_src_intervals']}, "
          f"{t['ms_wall_streamed']:.0f} ms, H2D {t['bytes_h2d'] / 1e9:.1f} GB, D2H {t['bytes_d2h'] / 1e9:.1f} GB, "
          f"peak device {ctx.peak_device_bytes() / 1e9:.2f} GB")
    rng = np.random.default_rng(5)
    deg = g.in_degree().numpy()
    vl = np.unique(np.concatenate([rng.choice(g.n, 300, replace=False), [0, g.n - 1, int(deg.argmax())]])).astype(np.int64)
    r = oracle.layer(g.col_ptr.numpy(), g.row_idx.numpy(), X.numpy(), edge_op="mul_weight", edge_weight=w.numpy(),
                     agg=agg, W=W.cpu().numpy(), act="relu", vlist=vl)
    assert_sum_close(Y[vl].numpy(), r["Y"], r["Y_abs"], TOL_F32, f"config 5 {agg}")
    ctx.destroy()
    if agg == "max":
        del test_config5_full_streamed_under_16gb.wl


def test_config5_full_streamed_backward_under_16gb():
    """Configuration 5's layer backwards at full size (R-MAT 23, 515 M edges, 256 -> 256, ReLU), everything but the
    parameters in host memory, 16 GiB device budget; sampled rows of dX and entries of dW from the oracle."""
    import paper_1810_08403_amd as saga
    wl = si.workload(5, device="cuda")
    g = wl.graph
    n, F, Fo = g.n, 256, 256
    host = si.CSC(n, g.col_ptr.cpu(), g.row_idx.cpu())
    W, w = wl.W.clone(), wl.edge_weight.cpu()
    del wl, g
    torch.cuda.empty_cache()
    # a synthetic Gather output (backward takes it as given), Y = ReLU(A W) formed in fp64 so that the signs are the oracle's
    A_h = torch.empty(n, F).pin_memory()
    Y_h = torch.empty(n, Fo).pin_memory()
    dY_h = torch.empty(n, Fo).pin_memory()
    step = 1 << 20
    for r0 in range(0, n, step):
        a = si.normal(311, r0 // step, step * F, device="cuda").view(step, F)
        A_h[r0:r0 + step] = a.cpu()
        Y_h[r0:r0 + step] = torch.relu(a.double() @ W.double()).float().cpu()
        dY_h[r0:r0 + step] = si.normal(312, r0 // step, step * Fo, device="cuda").view(step, Fo).cpu()
    del a
    torch.cuda.empty_cache()
    budget = 16 * (1 << 30)
    ctx = saga.Context(0, hbm_budget_bytes=budget)
    graph = ctx.graph_create_csc(n, host.col_ptr, host.row_idx)
    graph.set_edge_data(w)
    dX_h = torch.empty(n, F).pin_memory()
    dW, db = torch.empty(F, Fo, device="cuda"), torch.empty(Fo, device="cuda")
    ctx.layer_backward(graph, A_h, dY_h, W, dW, Y=Y_h, edge_op="mul_weight", act="relu", dX=dX_h, dbias=db)
    torch.cuda.synchronize()
    t = ctx.get_timings()
    assert ctx.peak_device_bytes() <= budget
    print(f"config5 backward: plan {t['plan_dst_intervals']} x {t['plan_src_intervals']}, H2D {t['bytes_h2d'] / 1e9:.1f} GB, "
          f"D2H {t['bytes_d2h'] / 1e9:.1f} GB, peak device {ctx.peak_device_bytes() / 1e9:.2f} GB")
    rng = np.random.default_rng(6)
    ul = np.unique(np.concatenate([rng.choice(n, 120, replace=False), [0, n - 1]])).astype(np.int64)
    we = [(0, 0), (255, 0), (100, 7), (31, 7)]
    ref = oracle.backward_sample(host.col_ptr.numpy(), host.row_idx.numpy(), None, A_h.numpy(), dY_h.numpy(), W.cpu().numpy(), ul, we,
                                 "mul_weight", w.numpy(), act="relu")
    assert_sum_close(dX_h[ul].numpy(), ref["dX"], ref["dX_abs"], TOL_F32, "config 5 backward dX")
    got = np.array([dW[f, o].item() for f, o in we])
    assert_sum_close(got, ref["dW"], ref["dW_abs"], TOL_F32, "config 5 backward dW")
    dz = dY_h.double() * (Y_h > 0)
    assert_sum_close(db.cpu().numpy(), dz.sum(0).numpy(), dz.abs().sum(0).numpy(), TOL_F32, "config 5 backward dbias")
    ctx.destroy()

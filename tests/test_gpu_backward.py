"""Backward pass of a layer (Section 2.2's backward stages) through the C ABI against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import saga_inputs as si
from helpers import TOL_F32, assert_sum_close, coarse_gated_workload, make_graph, new_context

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    import paper_1810_08403_amd as saga
    c = saga.Context(0)
    yield c
    c.destroy()


def _oracle_pair(wl, act, bias, with_self, dY):
    g = wl.graph
    cp, ri = g.col_ptr.numpy(), g.row_idx.numpy()
    w = wl.edge_weight.numpy() if wl.edge_op == "mul_weight" else None
    Ws = wl.W_self.numpy() if with_self else None
    b = None if bias is None else bias.numpy()
    fwd = oracle.layer(cp, ri, wl.X.numpy(), edge_op=wl.edge_op, edge_weight=w, W=wl.W.numpy(), bias=b, W_self=Ws, act=act)
    bwd = oracle.layer_backward(cp, ri, wl.X.numpy(), fwd["A"], dY.numpy(), wl.W.numpy(), wl.edge_op, w, bias=b, W_self=Ws, act=act)
    return fwd, bwd


def _run_backward(ctx, graph, wl, A, Y, dY, act, bias, with_self, attach=False, want_dx=True, pad=0):
    """GPU backward on host arrays; returns dict of numpy gradients. pad > 0 gives every matrix a row stride
    that many elements longer than its width."""
    dev = "cuda"
    def up(a):
        t = torch.as_tensor(np.ascontiguousarray(a), dtype=torch.float32)
        if pad and t.dim() == 2:
            buf = torch.zeros(t.shape[0], t.shape[1] + pad, device=dev)
            buf[:, :t.shape[1]] = t.to(dev)
            return buf[:, :t.shape[1]]
        return t.to(dev)
    def out(r, c):
        return torch.full((r, c + pad), float("nan"), device=dev)[:, :c] if pad else torch.full((r, c), float("nan"), device=dev)
    n, F = wl.X.shape
    Fo = wl.W.shape[1]
    kw = {}
    if wl.edge_op == "mul_weight":
        if attach:
            graph.set_edge_data(wl.edge_weight.to(dev))
        else:
            kw["edge_weight"] = wl.edge_weight.to(dev)
    dW, dX = out(F, Fo), (out(n, F) if want_dx else None)
    db = torch.full((Fo,), float("nan"), device=dev)
    dWs = out(F, Fo) if with_self else None
    ctx.layer_backward(graph, up(A), up(dY), up(wl.W), dW, X=up(wl.X), Y=up(Y), edge_op=wl.edge_op, bias=None if bias is None else bias.to(dev),
                       W_self=up(wl.W_self) if with_self else None, act=act, dX=dX, dbias=db, dW_self=dWs, **kw)
    torch.cuda.synchronize()
    res = {"dW": dW.cpu().numpy(), "dbias": db.cpu().numpy()}
    if want_dx:
        res["dX"] = dX.cpu().numpy()
    if with_self:
        res["dW_self"] = dWs.cpu().numpy()
    return res


def _check(res, bwd, dY, X, with_self, what):
    assert_sum_close(res["dW"], bwd["dW"], bwd["dW_abs"], TOL_F32, what + " dW")
    assert_sum_close(res["dbias"], bwd["dbias"], np.maximum(bwd["dbias_abs"], 1e-30), TOL_F32, what + " dbias")
    if "dX" in res:
        assert_sum_close(res["dX"], bwd["dX"], bwd["dX_abs"], TOL_F32, what + " dX")
    if with_self:
        assert_sum_close(res["dW_self"], bwd["dW_self"], np.maximum(bwd["dW_self_abs"], 1e-30), TOL_F32, what + " dW_self")


CASES = [
    # f_in, f_out, edge_op, act, with_self, with_bias
    (64, 64, "mul_weight", "relu", False, True),
    (128, 48, "copy", "relu", True, True),        # F_out < F_in: propagate dZ first, two-operand product
    (48, 128, "copy", "none", True, False),       # F_out > F_in: dA first, own partial gradient accumulated into
    (500, 16, "mul_weight", "relu", False, True), # GCN layer 1 shape
    (16, 3, "mul_weight", "none", False, True),   # GCN layer 2 shape, unaligned width
    (20, 7, "copy", "relu", True, True),          # nothing aligned
    (7, 20, "mul_weight", "relu", True, False),
    (256, 256, "mul_weight", "relu", False, False),
    (64, 48, "mul_weight", "sigmoid", True, True),   # the derivative y (1 - y) from the stored output
    (20, 33, "copy", "sigmoid", False, False),
]


@pytest.mark.parametrize("f_in,f_out,edge_op,act,with_self,with_bias", CASES)
def test_backward_matches_oracle(ctx, f_in, f_out, edge_op, act, with_self, with_bias):
    wl = si.commnet_workload(scale=11, f_in=f_in, f_out=f_out)   # R-MAT: heavy sources and heavy destinations
    wl.edge_op = edge_op
    if edge_op == "mul_weight":
        wl.edge_weight = si.gcn_edge_weights(wl.graph)
    n = wl.graph.n
    out_deg = torch.bincount(wl.graph.row_idx.long(), minlength=n)
    assert out_deg.max().item() > 128 and (out_deg == 0).any()    # cut groups and empty groups in the transposed order
    bias = si.uniform_pm(f_out, 0.3, 5) if with_bias else None
    dY = si.normal_features(n, f_out, 99)
    fwd, bwd = _oracle_pair(wl, act, bias, with_self, dY)
    graph = make_graph(ctx, wl.graph)
    # the oracle's A and Y rounded to fp32 go in, so that the ReLU decisions are the same on both sides
    res = _run_backward(ctx, graph, wl, fwd["A"], fwd["Y"], dY, act, bias, with_self)
    dZ = dY * torch.as_tensor(fwd["Y"] > 0) if act == "relu" else dY
    _check(res, bwd, dZ, wl.X, with_self, f"{f_in}->{f_out} {edge_op} {act}")
    graph.destroy()


def test_backward_after_gpu_forward_with_attached_edge_data_and_strided_tensors(ctx):
    wl = si.workload(2, scale=12, f_in=96, f_out=40)
    wl.act = "none"
    n = wl.graph.n
    graph = make_graph(ctx, wl.graph)
    graph.set_edge_data(wl.edge_weight.cuda())
    Xd, Wd = wl.X.cuda(), wl.W.cuda()
    Y = torch.empty(n, 40, device="cuda")
    A = torch.empty(n, 96, device="cuda")
    ctx.layer_forward(graph, Xd, Y, edge_op="mul_weight", W=Wd, act="none", accum_out=A)
    dY = si.normal_features(n, 40, 3)
    fwd, bwd = _oracle_pair(wl, "none", None, False, dY)
    res = _run_backward(ctx, graph, wl, A.cpu().numpy(), Y.cpu().numpy(), dY, "none", None, False, attach=True, pad=4)
    _check(res, bwd, dY, wl.X, False, "after GPU forward")
    # a second call reuses the transposed edge order and gives the same bits
    res2 = _run_backward(ctx, graph, wl, A.cpu().numpy(), Y.cpu().numpy(), dY, "none", None, False, attach=True, pad=4)
    assert np.array_equal(res["dX"], res2["dX"]) and np.array_equal(res["dW"], res2["dW"])
    graph.destroy()


def test_backward_without_dx_and_on_a_graph_without_edges(ctx):
    n, F, Fo = 300, 24, 12
    g = si.csc_from_lists(n, [])
    X, W, Ws = si.normal_features(n, F, 1), si.glorot_uniform(F, Fo, 2), si.glorot_uniform(F, Fo, 4)
    dY = si.normal_features(n, Fo, 3)
    wl = si.Workload(name="empty", graph=g, X=X, edge_op="copy", edge_weight=None, W=W, act="relu", dtype="f32", W_self=Ws)
    fwd, bwd = _oracle_pair(wl, "relu", None, True, dY)
    graph = make_graph(ctx, g)
    res = _run_backward(ctx, graph, wl, fwd["A"], fwd["Y"], dY, "relu", None, True)
    dZ = dY * torch.as_tensor(fwd["Y"] > 0)
    _check(res, bwd, dZ, X, True, "no edges")
    assert not res["dW"].any()                                   # A is all zero
    res = _run_backward(ctx, graph, wl, fwd["A"], fwd["Y"], dY, "relu", None, True, want_dx=False)
    _check(res, bwd, dZ, X, True, "no dX")
    graph.destroy()


def test_backward_rejects_what_it_does_not_cover(ctx):
    import paper_1810_08403_amd as saga
    wl = si.workload(1)
    graph = make_graph(ctx, wl.graph)
    n, F = wl.X.shape
    Fo = wl.W.shape[1]
    A, dY, W, dW = (torch.zeros(n, F, device="cuda"), torch.zeros(n, Fo, device="cuda"), wl.W.cuda(), torch.zeros(F, Fo, device="cuda"))
    X = wl.X.cuda()
    with pytest.raises(saga.SagaError) as e:                      # max over gated messages without the gate's parameters
        ctx.layer_backward(graph, A, dY, W, dW, X=X, agg="max", edge_op="gated")
    assert e.value.status == 1
    with pytest.raises(saga.SagaError) as e:                      # an activation without Y
        ctx.layer_backward(graph, A, dY, W, dW, act="sigmoid")
    assert e.value.status == 1
    with pytest.raises(saga.SagaError) as e:                      # W_self without dW_self
        ctx.layer_backward(graph, A, dY, W, dW, X=X, agg="max", W_self=W)
    assert e.value.status == 1
    with pytest.raises(saga.SagaError) as e:                      # max needs X
        ctx.layer_backward(graph, A, dY, W, dW, agg="max")
    assert e.value.status == 1
    with pytest.raises(saga.SagaError) as e:                      # POOL needs W_pool and dW_pool
        ctx.layer_backward(graph, A, dY, W, dW, X=X, edge_op="pool")
    assert e.value.status == 1
    with pytest.raises(saga.SagaError) as e:                      # RELU without Y
        ctx.layer_backward(graph, A, dY, W, dW, act="relu")
    assert e.value.status == 1
    with pytest.raises(saga.SagaError) as e:                      # wrong gradient shape
        ctx.layer_backward(graph, A, dY, W, torch.zeros(F, Fo + 1, device="cuda"))
    assert e.value.status == 1
    with pytest.raises(saga.SagaError) as e:                      # MUL_WEIGHT without weights
        ctx.layer_backward(graph, A, dY, W, dW, edge_op="mul_weight")
    assert e.value.status == 1
    graph.destroy()


# --------------------------------------------------------------------------
# full sizes, default tunables, sampled rows and entries from the oracle
# --------------------------------------------------------------------------

def _sample_sources(g, count, seed):
    """Random source vertices plus the one with most out-edges, one without any (if present), the first and last."""
    rng = np.random.default_rng(seed)
    od = torch.bincount(g.row_idx.long(), minlength=g.n).cpu().numpy()
    picks = set(rng.choice(g.n, size=count, replace=False).tolist())
    picks.update([int(od.argmax()), 0, g.n - 1])
    zero = np.nonzero(od == 0)[0]
    if len(zero):
        picks.add(int(zero[0]))
    return np.array(sorted(picks), dtype=np.int64)


def test_backward_config2_full_size_both_layers():
    """The two GCN layers of configuration 2 (500 -> 16 -> 3) at full size; A of each layer comes from the oracle-checked
    forward kernel's accum_out, and is an input to both sides."""
    import paper_1810_08403_amd as saga
    wl = si.workload(2, device="cuda")
    g = wl.graph
    n = g.n
    assert n == 131072
    cp, ri, w = g.col_ptr.cpu().numpy(), g.row_idx.cpu().numpy(), wl.edge_weight.cpu().numpy()
    with new_context() as ctx:
        graph = ctx.graph_create_csc(n, g.col_ptr, g.row_idx)
        graph.set_edge_data(wl.edge_weight)
        for (F, Fo, W, act, seed) in [(500, 16, wl.W, "relu", 1), (16, 3, wl.extra["W2"], "none", 2)]:
            A = si.normal_features(n, F, 100 + seed, device="cuda")       # a synthetic Gather output: backward takes it as given
            b = si.uniform_pm(Fo, 0.3, 7, device="cuda")
            Y = torch.relu(A.double() @ W.double() + b.double()).float() if act == "relu" else None
            dY = si.normal_features(n, Fo, 200 + seed, device="cuda")
            dX, dW, db = (torch.empty(n, F, device="cuda"), torch.empty(F, Fo, device="cuda"), torch.empty(Fo, device="cuda"))
            ctx.layer_backward(graph, A, dY, W, dW, Y=Y, edge_op="mul_weight", bias=b, act=act, dX=dX, dbias=db)
            torch.cuda.synchronize()
            ul = _sample_sources(g, 200, seed)
            rng = np.random.default_rng(seed)
            we = [(int(rng.integers(F)), int(rng.integers(Fo))) for _ in range(24)] + [(0, 0), (F - 1, Fo - 1)]
            ref = oracle.backward_sample(cp, ri, None, A.cpu().numpy(), dY.cpu().numpy(), W.cpu().numpy(), ul, we, "mul_weight", w,
                                         bias=b.cpu().numpy(), act=act, want_dbias=True)
            assert_sum_close(dX[ul].cpu().numpy(), ref["dX"], ref["dX_abs"], TOL_F32, f"config 2 {F}->{Fo} dX")
            got = np.array([dW[f, o].item() for f, o in we])
            assert_sum_close(got, ref["dW"], ref["dW_abs"], TOL_F32, f"config 2 {F}->{Fo} dW")
            dz_abs = (dY.double().abs() * ((Y > 0) if act == "relu" else 1)).sum(0).cpu().numpy()
            assert_sum_close(db.cpu().numpy(), ref["dbias"], np.maximum(dz_abs, 1e-30), TOL_F32, f"config 2 {F}->{Fo} dbias")


def test_backward_config3_shape_full_size_fp32():
    """Configuration 3's graph and widths (R-MAT 18, 130 M edges, 512 -> 256) in fp32, the precision the backward pass covers."""
    wl = si.workload(3, device="cuda")
    g = wl.graph
    n, F, Fo = g.n, 512, 256
    assert n == 262144 and g.nnz > 100_000_000
    cp, ri, w = g.col_ptr.cpu().numpy(), g.row_idx.cpu().numpy(), wl.edge_weight.cpu().numpy()
    W = wl.W.float()
    with new_context() as ctx:
        graph = ctx.graph_create_csc(n, g.col_ptr, g.row_idx)
        graph.set_edge_data(wl.edge_weight)
        A = si.normal_features(n, F, 31, device="cuda")
        Y = torch.relu(A.double() @ W.double()).float()
        dY = si.normal_features(n, Fo, 32, device="cuda")
        dX, dW, db = torch.empty(n, F, device="cuda"), torch.empty(F, Fo, device="cuda"), torch.empty(Fo, device="cuda")
        ctx.layer_backward(graph, A, dY, W, dW, Y=Y, edge_op="mul_weight", act="relu", dX=dX, dbias=db)
        torch.cuda.synchronize()
        ul = _sample_sources(g, 12, 3)
        we = [(0, 0), (511, 255), (17, 200), (300, 5), (128, 128), (255, 31)]
        ref = oracle.backward_sample(cp, ri, None, A.cpu().numpy(), dY.cpu().numpy(), W.cpu().numpy(), ul, we, "mul_weight", w, act="relu")
        assert_sum_close(dX[ul].cpu().numpy(), ref["dX"], ref["dX_abs"], TOL_F32, "config 3 shape dX")
        got = np.array([dW[f, o].item() for f, o in we])
        assert_sum_close(got, ref["dW"], ref["dW_abs"], TOL_F32, "config 3 shape dW")
        # the bias gradient against its definition on the device in fp64 (the oracle's whole-column form is too slow here)
        dz = dY.double() * (Y > 0)
        assert_sum_close(db.cpu().numpy(), dz.sum(0).cpu().numpy(), dz.abs().sum(0).cpu().numpy(), TOL_F32, "config 3 shape dbias")


# --------------------------------------------------------------------------
# gated layers (Example 2.1 / Figure 2)
# --------------------------------------------------------------------------

def _gated_backward_gpu(ctx, graph, wl, A, Y, dY, act, bias, with_b, with_msg, want_dx=True, W_self=None):
    dev = "cuda"
    n, F = wl.X.shape
    Fo = wl.W.shape[1]
    nan = lambda *shape: torch.full(shape, float("nan"), device=dev)
    f32 = lambda a: torch.as_tensor(np.ascontiguousarray(a), dtype=torch.float32).to(dev)
    dW, dX, db = nan(F, Fo), (nan(n, F) if want_dx else None), nan(Fo)
    dWg, dbg, dWm = nan(F, 2 * F), (nan(F) if with_b else None), (nan(F, F) if with_msg else None)
    dWs = nan(F, Fo) if W_self is not None else None
    ctx.layer_backward(graph, f32(A), f32(dY), wl.W.to(dev), dW, X=wl.X.to(dev), Y=f32(Y), edge_op="gated", act=act,
                       bias=None if bias is None else bias.to(dev), dX=dX, dbias=db,
                       W_gate=wl.W_gate.to(dev), b_gate=wl.b_gate.to(dev) if with_b else None,
                       W_msg=wl.W_msg.to(dev) if with_msg else None, dW_gate=dWg, db_gate=dbg, dW_msg=dWm,
                       W_self=None if W_self is None else W_self.to(dev), dW_self=dWs)
    torch.cuda.synchronize()
    res = {"dW": dW, "dbias": db, "dW_gate": dWg}
    if W_self is not None:
        res["dW_self"] = dWs
    if want_dx:
        res["dX"] = dX
    if with_b:
        res["db_gate"] = dbg
    if with_msg:
        res["dW_msg"] = dWm
    return {k: v.cpu().numpy() for k, v in res.items()}


@pytest.mark.parametrize("F,Fo,act,with_b,with_msg,with_self", [
    (8, 8, "relu", True, True, False),
    (64, 32, "relu", True, True, False),
    (128, 128, "none", True, True, False),       # configuration 4's widths
    (260, 16, "relu", False, True, False),       # wide kernel, two fragments per lane
    (20, 12, "relu", True, False, False),        # Example 2.1 exactly plus a bias: identity message matrix
    (7, 5, "none", False, False, False),         # nothing aligned
    (64, 48, "sigmoid", True, True, True),       # sigmoid activation and the vertex's own product
    (20, 12, "relu", True, False, True),
])
def test_gated_backward_matches_oracle(ctx, F, Fo, act, with_b, with_msg, with_self):
    wl = si.workload(4, scale=10, f_in=F, f_out=Fo)
    g = wl.graph
    n = g.n
    cp, ri = g.col_ptr.numpy(), g.row_idx.numpy()
    bias = si.uniform_pm(Fo, 0.3, 5)
    dY = si.normal_features(n, Fo, 99)
    Ws = si.glorot_uniform(F, Fo, 41) if with_self else None
    okw = dict(W_gate=wl.W_gate.numpy(), b_gate=wl.b_gate.numpy() if with_b else None, W_msg=wl.W_msg.numpy() if with_msg else None,
               W_self=None if Ws is None else Ws.numpy())
    fwd = oracle.layer(cp, ri, wl.X.numpy(), "gated", W=wl.W.numpy(), bias=bias.numpy(), act=act, **okw)
    bwd = oracle.gated_backward(cp, ri, wl.X.numpy(), fwd["A"], dY.numpy(), wl.W.numpy(), bias=bias.numpy(), act=act, **okw)
    graph = make_graph(ctx, g)
    res = _gated_backward_gpu(ctx, graph, wl, fwd["A"], fwd["Y"], dY, act, bias, with_b, with_msg, W_self=Ws)
    what = f"gated {F}->{Fo} {act}"
    assert_sum_close(res["dW"], bwd["dW"], bwd["dW_abs"], TOL_F32, what + " dW")
    assert_sum_close(res["dX"], bwd["dX"], bwd["dX_abs"], TOL_F32, what + " dX")
    assert_sum_close(res["dbias"], bwd["dbias"], np.maximum(bwd["dbias_abs"], 1e-30), TOL_F32, what + " dbias")
    if with_self:
        assert_sum_close(res["dW_self"], bwd["dW_self"], np.maximum(bwd["dW_self_abs"], 1e-30), TOL_F32, what + " dW_self")
    assert_sum_close(res["dW_gate"], bwd["dW_gate"], bwd["dW_gate_abs"], TOL_F32, what + " dW_gate")
    if with_b:
        assert_sum_close(res["db_gate"], bwd["db_gate"], bwd["db_gate_abs"], TOL_F32, what + " db_gate")
    if with_msg:
        assert_sum_close(res["dW_msg"], bwd["dW_msg"], bwd["dW_msg_abs"], TOL_F32, what + " dW_msg")
    # without dX the parameter gradients are the same bits
    res2 = _gated_backward_gpu(ctx, graph, wl, fwd["A"], fwd["Y"], dY, act, bias, with_b, with_msg, want_dx=False, W_self=Ws)
    assert np.array_equal(res2["dW_gate"], res["dW_gate"]) and np.array_equal(res2["dW"], res["dW"])
    graph.destroy()


def test_gated_backward_rejects_what_it_does_not_cover(ctx):
    import paper_1810_08403_amd as saga
    wl = si.workload(4, scale=8, f_in=16, f_out=16)
    graph = make_graph(ctx, wl.graph)
    n, F = wl.X.shape
    z = lambda *s: torch.zeros(*s, device="cuda")
    kw = dict(X=wl.X.cuda(), edge_op="gated", W_gate=wl.W_gate.cuda(), dW_gate=z(F, 2 * F))
    with pytest.raises(saga.SagaError) as e:                      # dW_msg without W_msg
        ctx.layer_backward(graph, z(n, F), z(n, 16), wl.W.cuda(), z(F, 16), dW_msg=z(F, F), **kw)
    assert e.value.status == 1
    with pytest.raises(saga.SagaError) as e:                      # W_self of the wrong shape
        ctx.layer_backward(graph, z(n, F), z(n, 16), wl.W.cuda(), z(F, 16), W_self=z(F, 15), dW_self=z(F, 15), **kw)
    assert e.value.status == 1
    with pytest.raises(saga.SagaError) as e:                      # gate gradients on a linear layer
        ctx.layer_backward(graph, z(n, F), z(n, 16), wl.W.cuda(), z(F, 16), dW_gate=z(F, 2 * F))
    assert e.value.status == 1
    kw.pop("dW_gate")
    with pytest.raises(saga.SagaError) as e:                      # dW_gate is required
        ctx.layer_backward(graph, z(n, F), z(n, 16), wl.W.cuda(), z(F, 16), **kw)
    assert e.value.status == 1
    graph.destroy()


def test_gated_backward_configuration_4_at_scale_16(ctx):
    """Configuration 4's layer (gated, 128 -> 128, bias and message matrix, ReLU) on R-MAT 16 with default tunables: the
    largest size at which the whole-graph oracle finishes in seconds (the full R-MAT 20 graph would take it minutes)."""
    wl = si.workload(4, scale=16)
    g = wl.graph
    n, F = wl.X.shape
    cp, ri = g.col_ptr.numpy(), g.row_idx.numpy()
    dY = si.normal_features(n, 128, 5)
    okw = dict(W_gate=wl.W_gate.numpy(), b_gate=wl.b_gate.numpy(), W_msg=wl.W_msg.numpy())
    fwd = oracle.layer(cp, ri, wl.X.numpy(), "gated", W=wl.W.numpy(), act="relu", b_gate=okw["b_gate"],
                       hoisted=oracle.hoist(wl.X.numpy(), okw["W_gate"], okw["W_msg"]))
    bwd = oracle.gated_backward(cp, ri, wl.X.numpy(), fwd["A"], dY.numpy(), wl.W.numpy(), act="relu", **okw)
    graph = make_graph(ctx, g)
    res = _gated_backward_gpu(ctx, graph, wl, fwd["A"], fwd["Y"], dY, "relu", None, True, True)
    info = graph.info()
    assert info["n_split_vertices"] > 0
    for name in ["dW", "dX", "dW_gate", "db_gate", "dW_msg"]:
        assert_sum_close(res[name], bwd[name], bwd[name + "_abs"], TOL_F32, "configuration 4 at scale 16, " + name)
    graph.destroy()


@pytest.mark.parametrize("F,Fo,act,with_b,with_msg,with_self", [
    (8, 8, "relu", True, True, False),
    (64, 32, "relu", True, True, False),
    (128, 128, "none", True, True, False),       # configuration 4's widths: the narrow kernel at its widest
    (160, 24, "relu", True, True, False),        # wide kernel, one fragment per lane
    (260, 16, "relu", False, True, False),       # wide kernel, two fragments per lane
    (70, 8, "none", True, True, False),          # rows that do not allow 16-byte fragments
    (20, 12, "relu", True, False, False),        # identity message matrix
    (64, 48, "sigmoid", True, True, True),       # sigmoid activation and the vertex's own product
    (20, 12, "relu", True, False, True),
])
def test_gated_max_backward_matches_oracle(ctx, F, Fo, act, with_b, with_msg, with_self):
    """Max over gated messages backwards. The Gather output handed to the backward pass is the forward pass's own (its
    maxima are compared bit for bit with the recomputed messages); the stored output is synthetic, only the activation's
    derivative is taken from it, and the oracle is given the same dZ."""
    wl = coarse_gated_workload(10, F, Fo)
    g = wl.graph
    n = g.n
    dev = "cuda"
    cp, ri = g.col_ptr.numpy(), g.row_idx.numpy()
    deg = np.diff(cp)
    assert deg.max() > 128 and (deg == 0).any()                      # cut columns and empty ones
    Ws = si.glorot_uniform(F, Fo, 41) if with_self else None
    bg = wl.b_gate if with_b else None
    Wm = wl.W_msg if with_msg else None
    opt = lambda t: None if t is None else t.to(dev)
    graph = make_graph(ctx, g)
    A = torch.full((n, F), float("nan"), device=dev)
    Yf = torch.empty(n, Fo, device=dev)
    ctx.layer_forward(graph, wl.X.to(dev), Yf, edge_op="gated", agg="max", W_gate=wl.W_gate.to(dev), b_gate=opt(bg), W_msg=opt(Wm),
                      W=wl.W.to(dev), W_self=opt(Ws), act="none", accum_out=A)
    dY = si.normal_features(n, Fo, 99)
    Y_in = si.normal_features(n, Fo, 98)
    if act == "sigmoid":
        Y_in = torch.sigmoid(Y_in)
    slope = {"none": torch.ones_like(Y_in.double()), "relu": (Y_in > 0).double(), "sigmoid": Y_in.double() * (1 - Y_in.double())}[act]
    dZ = (dY.double() * slope).float()
    okw = dict(W_gate=wl.W_gate.numpy(), b_gate=None if bg is None else bg.numpy(), W_msg=None if Wm is None else Wm.numpy(),
               W_self=None if Ws is None else Ws.numpy())
    bwd = oracle.gated_backward(cp, ri, wl.X.numpy(), None, dZ.numpy(), wl.W.numpy(), act="none", agg="max", **okw)
    what = f"gated max {F}->{Fo} {act}"
    assert_sum_close(A.cpu().numpy(), bwd["A"], np.maximum(np.abs(bwd["A"]), 1e-30), TOL_F32, what + " A")
    nan = lambda *shape: torch.full(shape, float("nan"), device=dev)
    def run(want_dx=True):
        out = dict(dW=nan(F, Fo), dX=nan(n, F) if want_dx else None, dbias=nan(Fo), dW_gate=nan(F, 2 * F),
                   db_gate=nan(F) if with_b else None, dW_msg=nan(F, F) if with_msg else None, dW_self=nan(F, Fo) if with_self else None)
        ctx.layer_backward(graph, A, dY.to(dev), wl.W.to(dev), out["dW"], X=wl.X.to(dev), Y=Y_in.to(dev), edge_op="gated", agg="max", act=act,
                           dX=out["dX"], dbias=out["dbias"], W_gate=wl.W_gate.to(dev), b_gate=opt(bg), W_msg=opt(Wm),
                           dW_gate=out["dW_gate"], db_gate=out["db_gate"], dW_msg=out["dW_msg"], W_self=opt(Ws), dW_self=out["dW_self"])
        torch.cuda.synchronize()
        return {k: v.cpu().numpy() for k, v in out.items() if v is not None}
    res = run()
    for name in res:
        assert np.abs(bwd[name]).max() > 0, name
        assert_sum_close(res[name], bwd[name], np.maximum(bwd[name + "_abs"], 1e-30), TOL_F32, f"{what} {name}")
    # a source that supplies no maximum gets nothing through the edges: its row of [dPs | dM] is zero, and without
    # in-edges dPd as well, so dX is exactly the vertex's own partial gradient (zero without W_self)
    if not with_self:
        assert ((bwd["dX_abs"] == 0) <= (res["dX"] == 0)).all()
    res2 = run(want_dx=False)
    assert np.array_equal(res2["dW_gate"], res["dW_gate"]) and np.array_equal(res2["dW"], res["dW"])
    graph.destroy()


# --------------------------------------------------------------------------
# max accumulator and max-pooling messages (Figure 11)
# --------------------------------------------------------------------------

def _quantised_pool_workload(scale, f_in, f_pool, f_out):
    """MP-GCN workload whose pooled pre-activations are exact in fp32 (coarse X, W_pool, b_pool), so that the order of the
    sigmoid messages, ties included, is the same in fp32 on the GPU and in fp64 in the oracle."""
    wl = si.mpgcn_workload(scale=scale, f_in=f_in, f_pool=f_pool, f_out=f_out)
    wl.X = torch.round(wl.X.clamp(-1, 1) * 4) / 4
    wl.W_pool = torch.round((wl.W_pool * 4).clamp(-0.5, 0.5) * 8) / 8
    wl.b_pool = torch.round(wl.b_pool.clamp(-0.5, 0.5) * 8) / 8
    assert f_in * 0.5 + 0.5 <= 8.5
    return wl


@pytest.mark.parametrize("edge_op,F,Fo,act,with_self", [("copy", 64, 32, "relu", False), ("mul_weight", 96, 128, "none", False),
                                                         ("copy", 7, 5, "relu", False), ("mul_weight", 260, 16, "relu", False),
                                                         ("mul_weight", 64, 48, "sigmoid", True), ("copy", 20, 12, "relu", True)])
def test_max_backward_matches_oracle(ctx, edge_op, F, Fo, act, with_self):
    wl = si.commnet_workload(scale=11, f_in=F, f_out=Fo)
    Ws = wl.W_self if with_self else None
    g = wl.graph
    n = g.n
    cp, ri = g.col_ptr.numpy(), g.row_idx.numpy()
    w = None
    if edge_op == "mul_weight":
        w = si.uniform_pm(g.nnz, 1.0, 17)                           # both signs
    bias = si.uniform_pm(Fo, 0.3, 5)
    dY = si.normal_features(n, Fo, 99)
    kw = dict(edge_weight=w.numpy()) if w is not None else {}
    if with_self:
        kw["W_self"] = Ws.numpy()
    fwd = oracle.layer(cp, ri, wl.X.numpy(), edge_op, agg="max", W=wl.W.numpy(), bias=bias.numpy(), act=act, **kw)
    bwd = oracle.max_backward(cp, ri, wl.X.numpy(), dY.numpy(), wl.W.numpy(), edge_op, bias=bias.numpy(), act=act, **kw)
    graph = make_graph(ctx, g)
    dev = "cuda"
    f32 = lambda a: torch.as_tensor(np.ascontiguousarray(a), dtype=torch.float32).to(dev)
    dX, dW, db = (torch.full((n, F), float("nan"), device=dev), torch.full((F, Fo), float("nan"), device=dev),
                  torch.full((Fo,), float("nan"), device=dev))
    dWs = torch.full((F, Fo), float("nan"), device=dev) if with_self else None
    ctx.layer_backward(graph, f32(bwd["A"]), dY.to(dev), wl.W.to(dev), dW, X=wl.X.to(dev), Y=f32(fwd["Y"]), edge_op=edge_op, agg="max",
                       edge_weight=None if w is None else w.to(dev), bias=bias.to(dev), act=act, dX=dX, dbias=db,
                       W_self=Ws.to(dev) if with_self else None, dW_self=dWs)
    torch.cuda.synchronize()
    what = f"max {edge_op} {F}->{Fo}"
    assert_sum_close(dW.cpu().numpy(), bwd["dW"], bwd["dW_abs"], TOL_F32, what + " dW")
    assert_sum_close(dX.cpu().numpy(), bwd["dX"], bwd["dX_abs"], TOL_F32, what + " dX")
    assert_sum_close(db.cpu().numpy(), bwd["dbias"], np.maximum(bwd["dbias_abs"], 1e-30), TOL_F32, what + " dbias")
    if with_self:
        assert_sum_close(dWs.cpu().numpy(), bwd["dW_self"], np.maximum(bwd["dW_self_abs"], 1e-30), TOL_F32, what + " dW_self")
    else:
        # every source that never supplies a maximum gets exactly zero
        assert ((bwd["dX_abs"] == 0) <= (dX.cpu().numpy() == 0)).all()
    graph.destroy()


@pytest.mark.parametrize("agg", ["max", "sum"])
@pytest.mark.parametrize("f_in,f_pool,f_out", [(16, 32, 16), (12, 7, 5), (16, 128, 64)])
def test_pool_backward_matches_oracle(ctx, agg, f_in, f_pool, f_out):
    wl = _quantised_pool_workload(11, f_in, f_pool, f_out)
    g = wl.graph
    n = g.n
    cp, ri = g.col_ptr.numpy(), g.row_idx.numpy()
    dY = si.normal_features(n, f_out, 7)
    dev = "cuda"
    graph = make_graph(ctx, g)
    Xd, Wd, Wp, bp = wl.X.to(dev), wl.W.to(dev), wl.W_pool.to(dev), wl.b_pool.to(dev)
    # the GPU's own forward pass supplies A and Y (its pooled rows are recomputed bit for bit in the backward pass)
    Y, A = torch.empty(n, f_out, device=dev), torch.empty(n, f_pool, device=dev)
    ctx.layer_forward(graph, Xd, Y, edge_op="pool", agg=agg, W_pool=Wp, b_pool=bp, W=Wd, act="none", accum_out=A)
    nan = lambda *s: torch.full(s, float("nan"), device=dev)
    dX, dW, db, dWp, dbp = nan(n, f_in), nan(f_pool, f_out), nan(f_out), nan(f_pool, f_in), nan(f_pool)
    ctx.layer_backward(graph, A, dY.to(dev), Wd, dW, X=Xd, edge_op="pool", agg=agg, W_pool=Wp, b_pool=bp, act="none",
                       dX=dX, dbias=db, dW_pool=dWp, db_pool=dbp)
    torch.cuda.synchronize()
    if agg == "max":
        bwd = oracle.max_backward(cp, ri, wl.X.numpy(), dY.numpy(), wl.W.numpy(), "pool", W_pool=wl.W_pool.numpy(),
                                  b_pool=wl.b_pool.numpy(), act="none")
        ties = 0
        for name, got in [("dW", dW), ("dX", dX), ("dW_pool", dWp), ("db_pool", dbp)]:
            assert_sum_close(got.cpu().numpy(), bwd[name], bwd[name + "_abs"], TOL_F32, f"pool max {f_in}->{f_pool}->{f_out} {name}")
    else:
        # sum over pooled messages: the linear backward of the hoisted rows, then through the sigmoid; checked against
        # autograd of the definition in fp64 on the host
        Xt = wl.X.double().requires_grad_(True)
        Wpt, bpt, Wt = wl.W_pool.double().requires_grad_(True), wl.b_pool.double().requires_grad_(True), wl.W.double().requires_grad_(True)
        H = torch.sigmoid(Xt @ Wpt.T + bpt)
        deg = g.col_ptr[1:] - g.col_ptr[:-1]
        dst = torch.repeat_interleave(torch.arange(n), deg)
        Aref = torch.zeros(n, f_pool, dtype=torch.float64).index_add(0, dst, H[g.row_idx.long()])
        ((Aref @ Wt) * dY.double()).sum().backward()
        for name, got, ref in [("dW", dW, Wt.grad), ("dX", dX, Xt.grad), ("dW_pool", dWp, Wpt.grad), ("db_pool", dbp, bpt.grad)]:
            err = (got.cpu().double() - ref).abs().max().item()
            assert err <= 2e-5 * ref.abs().max().item(), (name, err)
    graph.destroy()


def test_pool_backward_with_own_product_and_sigmoid_activation(ctx):
    """Max over pooled messages with ApplyVertex = sigmoid(A W + X W_self + bias): the vertex's own partial gradient joins
    dX inside the last product, and the activation's derivative comes from the stored output."""
    f_in, f_pool, f_out = 16, 32, 24
    wl = _quantised_pool_workload(11, f_in, f_pool, f_out)
    g = wl.graph
    n = g.n
    cp, ri = g.col_ptr.numpy(), g.row_idx.numpy()
    dY = si.normal_features(n, f_out, 7)
    Ws, bias = si.glorot_uniform(f_in, f_out, 43), si.uniform_pm(f_out, 0.3, 5)
    dev = "cuda"
    graph = make_graph(ctx, g)
    Xd, Wd, Wp, bp = wl.X.to(dev), wl.W.to(dev), wl.W_pool.to(dev), wl.b_pool.to(dev)
    Y, A = torch.empty(n, f_out, device=dev), torch.empty(n, f_pool, device=dev)
    kw = dict(edge_op="pool", agg="max", W_pool=Wp, b_pool=bp, W_self=Ws.to(dev), bias=bias.to(dev), act="sigmoid")
    ctx.layer_forward(graph, Xd, Y, W=Wd, accum_out=A, **kw)
    nan = lambda *s: torch.full(s, float("nan"), device=dev)
    dX, dW, db, dWp, dbp, dWs = nan(n, f_in), nan(f_pool, f_out), nan(f_out), nan(f_pool, f_in), nan(f_pool), nan(f_in, f_out)
    ctx.layer_backward(graph, A, dY.to(dev), Wd, dW, X=Xd, Y=Y, dX=dX, dbias=db, dW_pool=dWp, db_pool=dbp, dW_self=dWs, **kw)
    torch.cuda.synchronize()
    bwd = oracle.max_backward(cp, ri, wl.X.numpy(), dY.numpy(), wl.W.numpy(), "pool", W_pool=wl.W_pool.numpy(), b_pool=wl.b_pool.numpy(),
                              bias=bias.numpy(), act="sigmoid", W_self=Ws.numpy())
    for name, got in [("dW", dW), ("dX", dX), ("dW_pool", dWp), ("db_pool", dbp), ("dW_self", dWs), ("dbias", db)]:
        assert_sum_close(got.cpu().numpy(), bwd[name], np.maximum(bwd[name + "_abs"], 1e-30), TOL_F32, f"pool max with W_self, sigmoid: {name}")
    graph.destroy()


# --------------------------------------------------------------------------
# bf16 layers
# --------------------------------------------------------------------------

@pytest.mark.parametrize("f_in,f_out,edge_op,act,with_self", [(128, 48, "mul_weight", "relu", False), (48, 128, "copy", "none", False),
                                                              (512, 256, "mul_weight", "relu", False), (20, 7, "copy", "relu", False),
                                                              (64, 64, "mul_weight", "none", False), (128, 48, "copy", "relu", True),
                                                              (48, 128, "mul_weight", "none", True), (20, 7, "copy", "relu", True)])
def test_bf16_backward_matches_oracle(ctx, f_in, f_out, edge_op, act, with_self):
    from helpers import TOL_BF16
    wl = si.commnet_workload(scale=11, f_in=f_in, f_out=f_out)
    wl.edge_op = edge_op
    if edge_op == "mul_weight":
        wl.edge_weight = si.gcn_edge_weights(wl.graph)
    wl.X, wl.W, wl.W_self = si.round_to_bf16(wl.X), si.round_to_bf16(wl.W), si.round_to_bf16(wl.W_self)
    n = wl.graph.n
    dY = si.round_to_bf16(si.normal_features(n, f_out, 99))
    fwd, bwd = _oracle_pair(wl, act, None, with_self, dY)
    graph = make_graph(ctx, wl.graph)
    dev = "cuda"
    b16 = lambda a: torch.as_tensor(np.ascontiguousarray(a), dtype=torch.float32).to(dev).to(torch.bfloat16)
    A = torch.as_tensor(fwd["A"], dtype=torch.float32).to(dev)
    dW, db = torch.full((f_in, f_out), float("nan"), device=dev), torch.full((f_out,), float("nan"), device=dev)
    dX = torch.full((n, f_in), float("nan"), device=dev, dtype=torch.bfloat16)
    kw = dict(edge_weight=wl.edge_weight.to(dev)) if edge_op == "mul_weight" else {}
    dWs = torch.full((f_in, f_out), float("nan"), device=dev)
    if with_self:   # Y = act(A W + X W_self): dW_self from X widened to fp32, dZ W_self^T inside the dX product
        kw.update(X=b16(wl.X), W_self=b16(wl.W_self), dW_self=dWs)
    ctx.layer_backward(graph, A, b16(dY), b16(wl.W), dW, Y=b16(fwd["Y"]), edge_op=edge_op, act=act, dX=dX, dbias=db, **kw)
    torch.cuda.synchronize()
    what = f"bf16 {f_in}->{f_out} {edge_op} {act}" + (" with W_self" if with_self else "")
    if with_self:
        assert_sum_close(dWs.cpu().numpy(), bwd["dW_self"], bwd["dW_self_abs"], TOL_F32, what + " dW_self")
    # the parameter gradients are fp32 products of exactly representable inputs: the fp32 bar applies
    assert_sum_close(dW.cpu().numpy(), bwd["dW"], bwd["dW_abs"], TOL_F32, what + " dW")
    dZ = dY * torch.as_tensor(fwd["Y"] > 0) if act == "relu" else dY
    assert_sum_close(db.cpu().numpy(), bwd["dbias"], np.maximum(np.abs(dZ.numpy().astype(np.float64)).sum(0), 1e-30), TOL_F32, what + " dbias")
    assert_sum_close(dX.float().cpu().numpy(), bwd["dX"], bwd["dX_abs"], TOL_BF16, what + " dX")
    graph.destroy()


def test_bf16_backward_rejects_mixed_dtypes(ctx):
    import paper_1810_08403_amd as saga
    wl = si.workload(1)
    graph = make_graph(ctx, wl.graph)
    n, F = wl.X.shape
    Fo = wl.W.shape[1]
    bf = torch.bfloat16
    A, W16, dW = torch.zeros(n, F, device="cuda"), wl.W.cuda().to(bf), torch.zeros(F, Fo, device="cuda")
    with pytest.raises(saga.SagaError) as e:                      # fp32 dY with bf16 W
        ctx.layer_backward(graph, A, torch.zeros(n, Fo, device="cuda"), W16, dW)
    assert e.value.status == 1
    with pytest.raises(saga.SagaError) as e:                      # fp32 dX with bf16 W
        ctx.layer_backward(graph, A, torch.zeros(n, Fo, device="cuda", dtype=bf), W16, dW, dX=torch.zeros(n, F, device="cuda"))
    assert e.value.status == 1
    with pytest.raises(saga.SagaError) as e:                      # gated layers are fp32 only
        ctx.layer_backward(graph, A, torch.zeros(n, Fo, device="cuda", dtype=bf), W16, dW, edge_op="gated")
    assert e.value.status == 3
    graph.destroy()


@pytest.mark.parametrize("F", [64, 260])
def test_backward_with_team_mode_and_other_tunables(F):
    """The optional work-list shapes (a workgroup per piece of a cut group, small pieces and bands) under the backward
    edge functions: gated (one- and two-output forms) and max gradient."""
    from helpers import new_context
    wl = si.workload(4, scale=10, f_in=F, f_out=32)
    g = wl.graph
    n = g.n
    cp, ri = g.col_ptr.numpy(), g.row_idx.numpy()
    dY = si.normal_features(n, 32, 3)
    okw = dict(W_gate=wl.W_gate.numpy(), b_gate=wl.b_gate.numpy(), W_msg=wl.W_msg.numpy())
    fwd = oracle.layer(cp, ri, wl.X.numpy(), "gated", W=wl.W.numpy(), act="relu", **okw)
    bwd = oracle.gated_backward(cp, ri, wl.X.numpy(), fwd["A"], dY.numpy(), wl.W.numpy(), act="relu", **okw)
    fwd_m = oracle.layer(cp, ri, wl.X.numpy(), "copy", agg="max", W=wl.W.numpy(), act="relu")
    bwd_m = oracle.max_backward(cp, ri, wl.X.numpy(), dY.numpy(), wl.W.numpy(), "copy", act="relu")
    with new_context(team=1, split=16, cut_degree=32, stripe_kb=16) as c:
        graph = make_graph(c, g)
        res = _gated_backward_gpu(c, graph, wl, fwd["A"], fwd["Y"], dY, "relu", None, True, True)
        for name in ["dW", "dX", "dW_gate", "db_gate", "dW_msg"]:
            assert_sum_close(res[name], bwd[name], bwd[name + "_abs"], TOL_F32, f"team mode, gated F={F}, {name}")
        f32 = lambda a: torch.as_tensor(np.ascontiguousarray(a), dtype=torch.float32).cuda()
        dX, dW = torch.full((n, F), float("nan"), device="cuda"), torch.full((F, 32), float("nan"), device="cuda")
        c.layer_backward(graph, f32(bwd_m["A"]), dY.cuda(), wl.W.cuda(), dW, X=wl.X.cuda(), Y=f32(fwd_m["Y"]), edge_op="copy", agg="max",
                         act="relu", dX=dX)
        torch.cuda.synchronize()
        assert_sum_close(dX.cpu().numpy(), bwd_m["dX"], bwd_m["dX_abs"], TOL_F32, f"team mode, max F={F}, dX")
        assert_sum_close(dW.cpu().numpy(), bwd_m["dW"], bwd_m["dW_abs"], TOL_F32, f"team mode, max F={F}, dW")
        assert graph.info()["n_split_vertices"] > 0
        graph.destroy()

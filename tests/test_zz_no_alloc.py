"""saga_layer_forward_noalloc (the entry point for callers that must not allocate) against saga_layer_forward, through
the C ABI on the GPU: same bits, on two calls in a row of which the second is smaller, so that what the first call left
in the shared static scratch array would show if the second read any of it."""
import numpy as np
import pytest
import torch

import saga_inputs as si

pytestmark = pytest.mark.gpu


def _graph(rng, n, m, hub):
    edges = set(zip(rng.integers(n, size=m).tolist(), rng.integers(n, size=m).tolist()))
    if hub:
        edges |= {(u, 5) for u in range(n)}        # a column long enough to be cut into pieces: partial rows in the scratch
    return si.csc_from_lists(n, sorted(edges))


@pytest.mark.parametrize("op,agg,dtype", [("mul_weight", "sum", torch.float32), ("copy", "max", torch.float32),
                                          ("mul_weight", "sum", torch.bfloat16), ("gated", "sum", torch.float32),
                                          ("pool", "max", torch.float32)])
def test_no_alloc_matches_the_ordinary_call(op, agg, dtype):
    import paper_1810_08403_amd as saga
    rng = np.random.default_rng(21)
    t = lambda *shape, s=1.0: torch.as_tensor((rng.standard_normal(shape) * s).astype(np.float32)).cuda()
    ctx = saga.Context(0)
    for n, m, hub, F, Fo in ((6000, 90000, True, 128, 64), (700, 5000, False, 64, 16)):   # the second call is the smaller one
        g = _graph(rng, n, m, hub)
        h = ctx.graph_create_csc(n, g.col_ptr.cuda(), g.row_idx.cuda())
        X, W, bias = t(n, F).to(dtype), t(F, Fo, s=0.3).to(dtype), t(Fo, s=0.2)
        kw = {}
        if op == "mul_weight":
            kw["edge_weight"] = t(g.nnz)
        if op == "gated":
            kw.update(W_gate=t(F, 2 * F, s=0.2), b_gate=t(F, s=0.2), W_msg=t(F, F, s=0.2))
        if op == "pool":
            kw.update(W_pool=t(F, F, s=0.2), b_pool=t(F, s=0.2))
        args = dict(edge_op=op, agg=agg, W=W, bias=bias, act="relu", **kw)
        Y0, A0 = torch.full((n, Fo), float("nan"), device="cuda", dtype=dtype), torch.full((n, F), float("nan"), device="cuda")
        Y1, A1 = torch.full_like(Y0, float("nan")), torch.full_like(A0, float("nan"))
        ctx.layer_forward(h, X, Y0, accum_out=A0, **args)             # the ordinary call also builds the work list for this width
        ctx.layer_forward(h, X, Y1, accum_out=A1, no_alloc=True, **args)
        torch.cuda.synchronize()
        what = f"{op} {agg} {dtype} n={n} F={F}->{Fo}"
        assert not torch.isnan(Y1.float()).any() and not torch.isnan(A1).any(), what
        assert torch.equal(Y0, Y1), what + ": Y differs from saga_layer_forward"
        assert torch.equal(A0, A1), what + ": the Gather output differs from saga_layer_forward"
        assert h.info()["n_split_vertices"] > 0 or not hub, what
        h.destroy()
    ctx.destroy()


def test_no_alloc_refusals():
    import paper_1810_08403_amd as saga
    rng = np.random.default_rng(22)
    ctx = saga.Context(0)
    n = 9000
    g = si.csc_from_lists(n, [(i, (i * 7) % n) for i in range(n)])
    h = ctx.graph_create_csc(n, g.col_ptr.cuda(), g.row_idx.cuda())
    X = torch.zeros(n, 2048, device="cuda")
    W = torch.zeros(2048, 4, device="cuda")
    Y = torch.empty(n, 4, device="cuda")
    with pytest.raises(saga.SagaError) as e:                          # no work list for this row width yet
        ctx.layer_forward(h, X, Y, edge_op="copy", W=W, no_alloc=True)
    assert e.value.status == 3
    ctx.layer_forward(h, X, Y, edge_op="copy", W=W)
    with pytest.raises(saga.SagaError) as e:                          # 9000 x 2048 x 4 bytes of Gather output: beyond 64 MiB
        ctx.layer_forward(h, X, Y, edge_op="copy", W=W, no_alloc=True)
    assert e.value.status == 4 and "scratch" in str(e.value)
    Xs, Ws, Ys = X[:, :256].contiguous(), W[:256].contiguous(), torch.full((n, 4), float("nan"), device="cuda")
    ctx.layer_forward(h, Xs, Y, edge_op="copy", W=Ws)
    ctx.layer_forward(h, Xs, Ys, edge_op="copy", W=Ws, no_alloc=True)   # and a layer that fits goes through afterwards
    torch.cuda.synchronize()
    assert torch.equal(Y, Ys)
    h.destroy()
    ctx.destroy()

"""A seeded random session of streamed layer calls on one context, written once for two back ends: the HIP library on
a GPU (tests/test_gpu_random_cases.py) and the library's host code built against the CPU stand-in of the HIP runtime
under AddressSanitizer (tests/test_hoststub_cpu.py). Both check every call against the oracle."""
import numpy as np
import torch

import oracle
from helpers import TOL_F32, assert_sum_close


class GpuBackend:
    def context(self, budget):
        import paper_1810_08403_amd as saga
        return saga.Context(0, hbm_budget_bytes=budget)

    def dev(self, t):
        return t.cuda()

    def host(self, a):
        return torch.as_tensor(np.ascontiguousarray(a), dtype=torch.float32).clone().pin_memory()

    def host_full(self, shape, value):
        return torch.full(shape, value).pin_memory()

    def dev_full(self, shape, value):
        return torch.full(shape, value, device="cuda")

    def numpy(self, t):
        return t.cpu().numpy()

    @property
    def error(self):
        import paper_1810_08403_amd as saga
        return saga.SagaError


def session_graphs(seed, case):
    """The two graphs of a session: the first of up to 20 seeded small cases with enough vertices for any grid."""
    out = []
    for k in range(2):
        gk = None
        for attempt in range(20):
            _, gk, *_ = case(8100 + 40 * seed + 20 * k + attempt)
            if gk.n >= 33:
                break
        out.append(gk)
    return out


def streamed_session(be, seed, new_edge_data, case, log=lambda s: None, tol=TOL_F32):
    """The chunk grid a graph handle keeps (rebuilt when the row width changes its tunables, reused when a later call
    fits it), the interval buffers the context keeps and the budget they all count against, over a random sequence of
    streamed forward and backward calls on two graphs; with new_edge_data, edge data are attached again between calls."""
    rng = np.random.default_rng(8000 + seed)
    t = lambda *shape, s=1.0: torch.as_tensor((rng.standard_normal(shape) * s).astype(np.float32))
    use_budget = rng.random() < 0.5
    budget = int(rng.uniform(1.5, 6.0) * (1 << 20)) if use_budget else 0
    ctx = be.context(budget)
    if not use_budget:
        ctx.set_option("dst_intervals", int(rng.integers(1, 4)))
        ctx.set_option("src_intervals", int(rng.integers(1, 6)))
    ctx.set_option("bwd_tile_rows", int(rng.choice([0, 100, 1000])))
    graphs = []
    for gk in session_graphs(seed, case):
        h = ctx.graph_create_csc(gk.n, gk.col_ptr, gk.row_idx)
        wk = t(gk.nnz)
        h.set_edge_data(wk)
        graphs.append([gk, h, wk])
    for step in range(8):
        slot = graphs[int(rng.integers(2))]
        if new_edge_data and rng.random() < 0.25:                # new edge data: the handle's chunks are rebuilt
            slot[2] = t(slot[0].nnz)
            slot[1].set_edge_data(slot[2])
        g, h, wk = slot
        n, cp, ri = g.n, g.col_ptr.numpy(), g.row_idx.numpy()
        F = int(rng.choice([3, 8, 16, 40, 64, 128]))
        Fo = int(rng.choice([1, 8, 24]))
        op = str(rng.choice(["copy", "mul_weight", "mul_weight", "gated", "pool"]))
        agg = str(rng.choice(["sum", "max"]))
        act = str(rng.choice(["none", "relu"]))
        X, bias = t(n, F), t(Fo, s=0.2)
        kw, okw, Fm = {}, {}, F
        if op == "gated":
            F = min(F, 40)
            X = t(n, F)
            Fm = F
            Wg, bg = t(F, 2 * F, s=0.3), t(F, s=0.2)
            kw, okw = dict(W_gate=be.dev(Wg), b_gate=be.dev(bg)), dict(W_gate=Wg.numpy(), b_gate=bg.numpy())
        if op == "pool":
            Fm = int(rng.choice([4, 20]))
            Wp, bp = t(Fm, F, s=0.3), t(Fm, s=0.2)
            kw, okw = dict(W_pool=be.dev(Wp), b_pool=be.dev(bp)), dict(W_pool=Wp.numpy(), b_pool=bp.numpy())
        W = t(Fm, Fo, s=0.3)
        wn = wk.numpy() if op == "mul_weight" else None
        what = f"seed {seed} step {step}: n={n} nnz={g.nnz} F={F}->{Fm}->{Fo} {op} {agg} {act} budget={budget}"
        log(what)
        ref = oracle.layer(cp, ri, X.numpy(), op, wn, agg=agg, W=W.numpy(), bias=bias.numpy(), act=act, **okw)
        X_h, Y_h = be.host(X), be.host_full((n, Fo), float("nan"))
        try:
            ctx.layer_forward(h, X_h, Y_h, edge_op=op, agg=agg, W=be.dev(W), bias=be.dev(bias), act=act, **kw)
        except be.error as e:
            assert budget and e.status == 4, what          # SAGA_ERR_BUDGET: this layer does not fit; the next one may
            continue
        assert_sum_close(Y_h.numpy(), ref["Y"], ref["Y_abs"], tol, what + " layer", tiny_outputs=True)
        if budget:
            assert ctx.peak_device_bytes() <= budget, what
        if op in ("copy", "mul_weight") and agg == "sum" and rng.random() < 0.6:
            dY = t(n, Fo)
            bwd = oracle.layer_backward(cp, ri, X.numpy(), ref["A"], dY.numpy(), W.numpy(), op, wn, bias=bias.numpy(), act=act)
            dX_h = be.host_full((n, F), float("nan"))
            dW, db = be.dev_full((F, Fo), float("nan")), be.dev_full((Fo,), float("nan"))
            try:
                ctx.layer_backward(h, be.host(ref["A"]), be.host(dY), be.dev(W), dW, X=X_h, Y=be.host(ref["Y"]), edge_op=op,
                                   bias=be.dev(bias), act=act, dX=dX_h, dbias=db)
            except be.error as e:
                assert budget and e.status == 4, what
                continue
            assert_sum_close(be.numpy(dW), bwd["dW"], bwd["dW_abs"], tol, what + " dW", tiny_outputs=True)
            assert_sum_close(dX_h.numpy(), bwd["dX"], bwd["dX_abs"], tol, what + " dX", tiny_outputs=True)
            if budget:
                assert ctx.peak_device_bytes() <= budget, what + " (backward)"
    for _, h, _ in graphs:
        h.destroy()
    ctx.destroy()

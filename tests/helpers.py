"""Shared pieces of the GPU parity tests: run a workload through the C ABI and
through the CPU oracle, and the comparison rules."""
import contextlib

import numpy as np
import torch

import oracle
import saga_inputs as si

# Tolerances of the sum paths (relative to the sum of absolute terms, and to
# the largest reference magnitude); max paths are compared bit for bit.
TOL_F32 = 1e-5
TOL_BF16 = 1e-2


def assert_sum_close(got, ref, ref_abs, tol, what="", tiny_outputs=False):
    """|got - ref| <= tol * (sum of |terms|) element-wise, and max error <= tol * max|ref|.

    tiny_outputs (the random small cases, whose outputs can be a handful of values that all cancel or are cut off by
    ReLU): the second bar is left out where the arithmetic the layer is defined in cannot meet it, that is where one
    rounding of one term is already more than tol * max|ref|: 2^-24 of the largest sum of absolute terms under the
    fp32 bar, 2^-9 of it under the bf16 bar (there the Gather output is rounded to bf16 before the product)."""
    got = np.asarray(got, np.float64)
    err = np.abs(got - ref)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    scale = np.maximum(ref_abs, 1e-30)
    worst = (err / scale).max() if err.size else 0.0
    assert worst <= tol, f"{what}: element error {worst:.3e} of the absolute-term sum exceeds {tol}"
    if err.size and np.abs(ref).max() > 0:
        if tiny_outputs and 2.0 ** (-9 if tol >= 1e-3 else -24) * np.max(ref_abs) > tol * np.abs(ref).max():
            return
        nw = err.max() / np.abs(ref).max()
        assert nw <= tol, f"{what}: normwise error {nw:.3e} exceeds {tol}"


def assert_bit_equal(got, ref, what=""):
    """Equality of fp32 values; +0 and -0 count as equal."""
    got = np.asarray(got, np.float32)
    ref = np.asarray(ref, np.float64).astype(np.float32)
    bad = got != ref
    assert not bad.any(), f"{what}: {int(bad.sum())} of {bad.size} values differ, first at {np.argwhere(bad)[0]}"


def to_device_dtype(x: torch.Tensor, dtype: str, device="cuda"):
    return x.to(device=device, dtype=torch.bfloat16 if dtype == "bf16" else torch.float32).contiguous()


def run_gpu(ctx, wl, graph, agg="sum", want_accum=True, with_vertex=True, bias=None, W=None, act=None, X=None):
    """One layer of workload `wl` on the GPU through the C ABI; returns (Y, A) as CPU float32/float64 arrays."""
    dev = "cuda"
    Xh = wl.X if X is None else X
    Xd = to_device_dtype(Xh, wl.dtype)
    n, F = Xd.shape
    Wt = wl.W if W is None else W
    kw = {}
    if wl.edge_op == "mul_weight":
        kw["edge_weight"] = wl.edge_weight.to(dev)
    if wl.edge_op == "gated":
        kw.update(W_gate=wl.W_gate.to(dev), b_gate=None if wl.b_gate is None else wl.b_gate.to(dev),
                  W_msg=None if wl.W_msg is None else wl.W_msg.to(dev))
    Fm = F
    if wl.edge_op == "pool":
        kw.update(W_pool=wl.W_pool.to(dev), b_pool=None if wl.b_pool is None else wl.b_pool.to(dev))
        Fm = wl.W_pool.shape[0]
    if with_vertex:
        Wd = to_device_dtype(Wt, wl.dtype)
        kw.update(W=Wd, act=wl.act if act is None else act, bias=None if bias is None else bias.to(dev))
        if wl.W_self is not None:
            kw["W_self"] = to_device_dtype(wl.W_self, wl.dtype)
        Y = torch.empty(n, Wd.shape[1], device=dev, dtype=Xd.dtype)
    else:
        Y = torch.empty(n, Fm, device=dev, dtype=Xd.dtype)
    A = torch.empty(n, Fm, device=dev, dtype=torch.float32) if want_accum else None
    ctx.layer_forward(graph, Xd, Y, edge_op=wl.edge_op, agg=agg, accum_out=A, **kw)
    torch.cuda.synchronize()
    return Y.float().cpu().numpy(), (None if A is None else A.cpu().numpy())


def run_oracle(wl, agg="sum", with_vertex=True, bias=None, vlist=None, W=None, act=None, X=None, hoisted=False):
    g = wl.graph
    Xh = (wl.X if X is None else X).cpu().numpy()
    kw = dict(edge_op=wl.edge_op, agg=agg, vlist=vlist)
    if wl.edge_op == "mul_weight":
        kw["edge_weight"] = wl.edge_weight.cpu().numpy()
    if wl.edge_op == "gated":
        kw.update(W_gate=wl.W_gate.cpu().numpy(), b_gate=None if wl.b_gate is None else wl.b_gate.cpu().numpy(),
                  W_msg=None if wl.W_msg is None else wl.W_msg.cpu().numpy())
        if hoisted:
            kw["hoisted"] = oracle.hoist(Xh, kw["W_gate"], kw["W_msg"])
    if wl.edge_op == "pool":
        if hoisted:
            kw["hoisted"] = oracle.hoist_pool(Xh, wl.W_pool.cpu().numpy(), None if wl.b_pool is None else wl.b_pool.cpu().numpy())
        else:
            kw.update(W_pool=wl.W_pool.cpu().numpy(), b_pool=None if wl.b_pool is None else wl.b_pool.cpu().numpy())
    if with_vertex:
        kw.update(W=(wl.W if W is None else W).cpu().numpy(), act=wl.act if act is None else act,
                  bias=None if bias is None else bias.cpu().numpy(),
                  W_self=None if wl.W_self is None else wl.W_self.cpu().numpy())
    return oracle.layer(g.col_ptr.cpu().numpy(), g.row_idx.cpu().numpy(), Xh, **kw)


def make_graph(ctx, g: si.CSC, device="cuda"):
    gd = g.to(device)
    return ctx.graph_create_csc(g.n, gd.col_ptr, gd.row_idx)


@contextlib.contextmanager
def new_context(budget=0, **options):
    """A library context that is destroyed when the block ends, also when an assertion fails
    (a context left to the interpreter's shutdown would call into a HIP runtime that is gone)."""
    import paper_1810_08403_amd as saga
    c = saga.Context(0, hbm_budget_bytes=budget)
    try:
        for k, v in options.items():
            c.set_option(k, v)
        yield c
    finally:
        c.destroy()


def coarse_gated_workload(scale, F, Fo):
    """Configuration 4's layer shape with X, W_gate, b_gate and W_msg on coarse grids (multiples of 1/4 and 1/8): the
    hoisted products are then exact in fp32 in any order of summation, so the GPU's fp32 messages sigmoid(z) * m and the
    oracle's fp64 ones are formed from the same z and m and rank alike, ties included (two different (z, m) pairs give
    messages that differ by far more than the 1e-7 the two sigmoids differ by)."""
    wl = si.workload(4, scale=scale, f_in=F, f_out=Fo)
    q = lambda t, lim, s: torch.round(t.clamp(-lim, lim) * s) / s
    wl.X = q(wl.X, 1.0, 4)
    wl.W_gate, wl.b_gate, wl.W_msg = q(wl.W_gate, 1.0, 8), q(wl.b_gate, 0.5, 8), q(wl.W_msg, 1.0, 8)
    Xd = wl.X.double()
    z = (Xd @ wl.W_gate[:, :F].double().T).abs().max() + (Xd @ wl.W_gate[:, F:].double().T).abs().max() + 0.5
    assert z.item() <= 12.0 and (wl.W_gate != 0).float().mean().item() > 0.2
    return wl

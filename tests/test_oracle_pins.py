"""Pins for the CPU oracle: things the paper and the mathematics fix.

None of these re-types the oracle's loop. They are: hand-worked values, the
dense matrix form of the layer (the sparse-dense product identity of
Section 6.1), a library sparse product, closed forms and invariants, and
special cases in which one edge function must collapse to another.
"""
import json
import os

import numpy as np
import pytest
import scipy.sparse as sp
import torch

import oracle
import saga_inputs as si

HERE = os.path.dirname(os.path.abspath(__file__))


def _np(g):
    return g.col_ptr.numpy(), g.row_idx.numpy()


def _coo(g):
    return g.row_idx.numpy().astype(np.int64), g.dst_of_edges().numpy()


def _random_graph(n, m, seed, self_loops=False, symmetrise=False):
    s, d = si.uniform_edges(n, m, seed)
    return si.build_csc(n, s, d, symmetrise=symmetrise, self_loops=self_loops)


def _dense_adj(g, w=None):
    """Adj[v, u] = weight of edge u -> v (1 if unweighted), built from the COO list."""
    src, dst = _coo(g)
    A = np.zeros((g.n, g.n))
    A[dst, src] = 1.0 if w is None else w.astype(np.float64)
    return A


# --------------------------------------------------------------------------
# hand-worked values (tests/golden/hand_worked_layer.json)
# --------------------------------------------------------------------------

@pytest.fixture(scope="module")
def hand():
    with open(os.path.join(HERE, "golden", "hand_worked_layer.json")) as f:
        return json.load(f)


def test_hand_worked_graph_builds_the_stated_csc(hand):
    g = si.csc_from_lists(hand["n"], [tuple(e) for e in hand["edges_src_dst"]])
    assert g.col_ptr.tolist() == hand["csc_col_ptr"] and g.row_idx.tolist() == hand["csc_row_idx"]


@pytest.mark.parametrize("op,agg,key", [("copy", "sum", "copy_sum_A"), ("mul_weight", "sum", "mul_weight_sum_A"),
                                        ("copy", "max", "copy_max_A"), ("mul_weight", "max", "mul_weight_max_A")])
def test_hand_worked_gather(hand, op, agg, key):
    o = oracle.layer(hand["csc_col_ptr"], hand["csc_row_idx"], hand["X"], op,
                     hand["edge_weight_in_csc_order"] if op == "mul_weight" else None, agg=agg)
    assert np.array_equal(o["A"], np.array(hand[key], float))


def test_hand_worked_apply_vertex(hand):
    args = (hand["csc_col_ptr"], hand["csc_row_idx"], hand["X"], "copy")
    y = oracle.layer(*args, W=hand["W"], act="relu")["Y"]
    assert np.array_equal(y, np.array(hand["copy_sum_relu_Y_no_bias"], float))
    y = oracle.layer(*args, W=hand["W"], bias=hand["bias"], act="relu")["Y"]
    assert np.array_equal(y, np.array(hand["copy_sum_relu_Y_with_bias"], float))
    y = oracle.layer(*args, W=hand["W"], bias=hand["bias"], act="none")["Y"]
    assert np.array_equal(y, np.array(hand["copy_sum_none_Y_with_bias"], float))


def test_hand_worked_gate_closed_form():
    """Example 2.1 with F = 1: x = (L, -L, 2L), L = fp32(ln 3), gate row (2, -1).

    The gate pre-activation is 2 x_src - x_dst, an integer multiple k of L, so
    sigmoid = 3^k / (1 + 3^k) up to the rounding of L. Swapping the roles of
    source and destination, or the sign inside the sigmoid, changes every value.
    """
    L = float(np.float32(np.log(3.0)))
    g = si.csc_from_lists(3, [(0, 1), (2, 1), (1, 0), (0, 0), (1, 2)])
    X = np.array([[L], [-L], [2 * L]], np.float32)
    o = oracle.layer(*_np(g), X, "gated", W_gate=np.array([[2.0, -1.0]], np.float32))
    want = np.array([[L * (3 / 4 - 1 / 28)], [L * (27 / 28 + 2 * 243 / 244)], [-L / 82]])
    assert np.allclose(o["A"], want, rtol=2e-6, atol=0)
    # error scale of each message g t: g (|t| + |t| (1 - g) Z), Z = 2 |x_src| + |x_dst|
    def s(g, xu, xv):
        return g * (abs(xu) + abs(xu) * (1 - g) * (2 * abs(xu) + abs(xv)))
    want_abs = np.array([[s(3 / 4, L, L) + s(1 / 28, -L, L)],
                         [s(27 / 28, L, -L) + s(243 / 244, 2 * L, -L)],
                         [s(1 / 82, -L, 2 * L)]])
    assert np.allclose(o["A_abs"], want_abs, rtol=2e-6, atol=0)


# --------------------------------------------------------------------------
# dense matrix form: Y = act((Adj o w) X W + bias)
# --------------------------------------------------------------------------

@pytest.mark.parametrize("op", ["copy", "mul_weight"])
@pytest.mark.parametrize("act", ["relu", "none"])
def test_sum_layer_equals_dense_matrix_product(op, act):
    g = _random_graph(150, 1200, seed=21)            # directed: Adj is not symmetric
    rng = np.random.default_rng(0)
    X = rng.standard_normal((g.n, 7)).astype(np.float32)
    W = rng.standard_normal((7, 5)).astype(np.float32)   # F_in != F_out: a transposed W cannot pass
    bias = rng.standard_normal(5).astype(np.float32)
    w = rng.standard_normal(g.nnz).astype(np.float32) if op == "mul_weight" else None
    o = oracle.layer(*_np(g), X, op, w, W=W, bias=bias, act=act)
    if op == "mul_weight":
        # the per-edge message is the fp32 product; reproduce that rounding term by term
        src, dst = _coo(g)
        A = np.zeros((g.n, 7))
        np.add.at(A, dst, (w[:, None] * X[src]).astype(np.float32).astype(np.float64))
    else:
        A = _dense_adj(g) @ X.astype(np.float64)
    Y = A @ W.astype(np.float64) + bias
    if act == "relu":
        Y = np.maximum(Y, 0.0)
    assert np.allclose(o["A"], A, rtol=1e-12, atol=1e-12)
    assert np.allclose(o["Y"], Y, rtol=1e-12, atol=1e-12)
    if op == "mul_weight":   # the exact-product matrix form agrees to fp32 rounding of each term
        A2 = _dense_adj(g, w) @ X.astype(np.float64)
        assert np.abs(o["A"] - A2).max() <= 2.0 ** -23 * o["A_abs"].max()


def test_gather_equals_scipy_sparse_product_on_config_shapes():
    for wl in (si.workload(1), si.workload(2, scale=11)):
        g = wl.graph
        src, dst = _coo(g)
        S = sp.csr_matrix((wl.edge_weight.numpy().astype(np.float64), (dst, src)), shape=(g.n, g.n))
        want = S @ wl.X.numpy().astype(np.float64)
        o = oracle.layer(*_np(g), wl.X.numpy(), "mul_weight", wl.edge_weight.numpy())
        assert np.abs(o["A"] - want).max() <= 2.0 ** -23 * np.abs(o["A_abs"]).max()
        Sabs = sp.csr_matrix((np.abs(wl.edge_weight.numpy()).astype(np.float64), (dst, src)), shape=(g.n, g.n))
        want_abs = Sabs @ np.abs(wl.X.numpy()).astype(np.float64)
        assert np.allclose(o["A_abs"], want_abs, rtol=1e-6, atol=1e-30)


def test_all_ones_features_give_the_in_degree():
    wl = si.workload(4, scale=11)                    # directed R-MAT, empty columns included
    g = wl.graph
    o = oracle.layer(*_np(g), np.ones((g.n, 3), np.float32), "copy")
    deg = g.in_degree().numpy().astype(np.float64)
    assert (deg == 0).any() and np.array_equal(o["A"], np.repeat(deg[:, None], 3, 1))
    # out-degree would be a different vector on a directed graph
    out_deg = np.bincount(g.row_idx.numpy(), minlength=g.n)
    assert not np.array_equal(out_deg, deg)


# --------------------------------------------------------------------------
# max accumulator
# --------------------------------------------------------------------------

@pytest.mark.parametrize("op", ["copy", "mul_weight"])
def test_max_gather_equals_brute_force_over_the_edge_list(op):
    g = _random_graph(60, 500, seed=33)
    g = si.CSC(g.n + 4, torch.cat([g.col_ptr, g.col_ptr[-1:].repeat(4)]), g.row_idx)  # 4 isolated vertices
    rng = np.random.default_rng(1)
    X = rng.standard_normal((g.n, 6)).astype(np.float32)
    w = rng.standard_normal(g.nnz).astype(np.float32)
    o = oracle.layer(*_np(g), X, op, w if op == "mul_weight" else None, agg="max")
    src, dst = _coo(g)
    msg = X[src] * w[:, None] if op == "mul_weight" else X[src]        # float32 arithmetic
    assert msg.dtype == np.float32
    for v in range(g.n):
        sel = msg[dst == v]
        want = sel.max(axis=0) if len(sel) else np.zeros(6, np.float32)
        assert np.array_equal(o["A"][v], want.astype(np.float64))


def test_max_is_not_sum_and_handles_negative_only_columns():
    g = si.csc_from_lists(3, [(0, 2), (1, 2)])
    X = np.array([[-5.0], [-2.0], [9.0]], np.float32)
    assert oracle.layer(*_np(g), X, "copy", agg="max")["A"].tolist() == [[0.0], [0.0], [-2.0]]
    assert oracle.layer(*_np(g), X, "copy", agg="sum")["A"].tolist() == [[0.0], [0.0], [-7.0]]


# --------------------------------------------------------------------------
# gated edge function
# --------------------------------------------------------------------------

def _gated_setup(n=40, m=300, F=5, seed=4):
    g = _random_graph(n, m, seed=seed)
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((n, F)).astype(np.float32)
    Wg = (0.5 * rng.standard_normal((F, 2 * F))).astype(np.float32)
    bg = rng.standard_normal(F).astype(np.float32)
    Wm = rng.standard_normal((F, F)).astype(np.float32)
    return g, X, Wg, bg, Wm


def test_gated_equals_dense_broadcast_form():
    g, X, Wg, bg, Wm = _gated_setup()
    F = X.shape[1]
    Xd = X.astype(np.float64)
    Ps = Xd @ Wg[:, :F].astype(np.float64).T
    Pd = Xd @ Wg[:, F:].astype(np.float64).T
    M = Xd @ Wm.astype(np.float64).T
    Z = Pd[:, None, :] + Ps[None, :, :] + bg            # Z[v, u, f]
    G = 1.0 / (1.0 + np.exp(-Z))
    Adj = _dense_adj(g)
    want = np.einsum("vu,vuf,uf->vf", Adj, G, M)
    o = oracle.layer(*_np(g), X, "gated", W_gate=Wg, b_gate=bg, W_msg=Wm)
    assert np.allclose(o["A"], want, rtol=1e-12, atol=1e-13)
    # error scale: every term of the inner sums by absolute value, the gate through its derivative
    Xa = np.abs(Xd)
    T_abs = Xa @ np.abs(Wm).astype(np.float64).T
    Z_abs = (Xa @ np.abs(Wg[:, F:]).astype(np.float64).T)[:, None, :] + \
        (Xa @ np.abs(Wg[:, :F]).astype(np.float64).T)[None, :, :] + np.abs(bg)
    S = G * (T_abs[None, :, :] + np.abs(M)[None, :, :] * (1.0 - G) * Z_abs)
    want_abs = np.einsum("vu,vuf->vf", Adj, S)
    assert np.allclose(o["A_abs"], want_abs, rtol=1e-12, atol=1e-13)
    h = oracle.layer(*_np(g), X, "gated", W_gate=Wg, b_gate=bg, W_msg=Wm, hoisted=oracle.hoist(X, Wg, Wm))
    assert np.allclose(h["A_abs"], want_abs, rtol=1e-12, atol=1e-13)
    # Example 2.1 proper: no bias, no message matrix
    Z0 = Pd[:, None, :] + Ps[None, :, :]
    want0 = np.einsum("vu,vuf,uf->vf", Adj, 1.0 / (1.0 + np.exp(-Z0)), Xd)
    o0 = oracle.layer(*_np(g), X, "gated", W_gate=Wg)
    assert np.allclose(o0["A"], want0, rtol=1e-12, atol=1e-13)


def test_gate_with_zero_weights_is_a_half():
    g, X, Wg, bg, Wm = _gated_setup()
    o = oracle.layer(*_np(g), X, "gated", W_gate=np.zeros_like(Wg), W_msg=Wm)
    want = 0.5 * (_dense_adj(g) @ (X.astype(np.float64) @ Wm.astype(np.float64).T))
    assert np.allclose(o["A"], want, rtol=1e-12, atol=1e-13)


def test_saturated_gate_is_commnet_passthrough():
    # bias +40 opens the gate to 1 within 1e-17: Figure 9's ApplyEdge (return edge.src)
    g, X, Wg, bg, Wm = _gated_setup()
    o = oracle.layer(*_np(g), X, "gated", W_gate=np.zeros_like(Wg), b_gate=np.full_like(bg, 40.0))
    c = oracle.layer(*_np(g), X, "copy")
    assert np.allclose(o["A"], c["A"], rtol=1e-15, atol=1e-15)
    # and bias -40 closes it
    z = oracle.layer(*_np(g), X, "gated", W_gate=np.zeros_like(Wg), b_gate=np.full_like(bg, -40.0))
    assert np.abs(z["A"]).max() < 1e-15


def test_gate_halves_address_source_and_destination():
    g, X, Wg, bg, Wm = _gated_setup()
    F = X.shape[1]
    Xd, Adj = X.astype(np.float64), _dense_adj(g)
    M = Xd @ Wm.astype(np.float64).T
    sig = lambda z: 1.0 / (1.0 + np.exp(-z))
    # only the destination half is non-zero: the gate factors out of the sum
    Wd = Wg.copy(); Wd[:, :F] = 0
    o = oracle.layer(*_np(g), X, "gated", W_gate=Wd, b_gate=bg, W_msg=Wm)
    want = sig(Xd @ Wd[:, F:].astype(np.float64).T + bg) * (Adj @ M)
    assert np.allclose(o["A"], want, rtol=1e-11, atol=1e-12)
    # only the source half is non-zero: the gate folds into the source rows
    Ws = Wg.copy(); Ws[:, F:] = 0
    o = oracle.layer(*_np(g), X, "gated", W_gate=Ws, b_gate=bg, W_msg=Wm)
    want = Adj @ (sig(Xd @ Ws[:, :F].astype(np.float64).T + bg) * M)
    assert np.allclose(o["A"], want, rtol=1e-11, atol=1e-12)


def test_hoisted_equals_naive():
    # Section 3.2: moving the vertex-only products out of ApplyEdge changes nothing
    g, X, Wg, bg, Wm = _gated_setup(n=80, m=900, F=9, seed=8)
    W = np.random.default_rng(3).standard_normal((9, 4)).astype(np.float32)
    for wm in (Wm, None):
        for b in (bg, None):
            a = oracle.layer(*_np(g), X, "gated", W_gate=Wg, b_gate=b, W_msg=wm, W=W, act="relu")
            h = oracle.layer(*_np(g), X, "gated", W_gate=Wg, b_gate=b, W_msg=wm, W=W, act="relu",
                             hoisted=oracle.hoist(X, Wg, wm))
            assert np.allclose(a["A"], h["A"], rtol=1e-12, atol=1e-13)
            assert np.allclose(a["Y"], h["Y"], rtol=1e-12, atol=1e-13)
    Ps, Pd, M, Ps_abs, Pd_abs, M_abs = oracle.hoist(X, Wg, Wm)
    Xd = X.astype(np.float64)
    assert np.allclose(Ps_abs, np.abs(Xd) @ np.abs(Wg[:, :9]).astype(np.float64).T, rtol=1e-13, atol=1e-13)
    assert np.allclose(Pd_abs, np.abs(Xd) @ np.abs(Wg[:, 9:]).astype(np.float64).T, rtol=1e-13, atol=1e-13)
    assert np.allclose(M_abs, np.abs(Xd) @ np.abs(Wm).astype(np.float64).T, rtol=1e-13, atol=1e-13)
    assert np.allclose(Ps, Xd @ Wg[:, :9].astype(np.float64).T, rtol=1e-13, atol=1e-13)
    assert np.allclose(Pd, Xd @ Wg[:, 9:].astype(np.float64).T, rtol=1e-13, atol=1e-13)
    assert np.allclose(M, Xd @ Wm.astype(np.float64).T, rtol=1e-13, atol=1e-13)


# --------------------------------------------------------------------------
# ApplyVertex alone, invariances, degenerate shapes
# --------------------------------------------------------------------------

def test_self_loops_only_reduce_the_layer_to_a_dense_product():
    n = 33
    g = si.csc_from_lists(n, [(v, v) for v in range(n)])
    rng = np.random.default_rng(5)
    X = rng.standard_normal((n, 6)).astype(np.float32)
    W = rng.standard_normal((6, 11)).astype(np.float32)
    b = rng.standard_normal(11).astype(np.float32)
    o = oracle.layer(*_np(g), X, "mul_weight", np.ones(n, np.float32), W=W, bias=b, act="relu")
    want = np.maximum(X.astype(np.float64) @ W.astype(np.float64) + b, 0)
    assert np.allclose(o["Y"], want, rtol=1e-13, atol=1e-13) and (o["Y"] >= 0).all()
    want_abs = np.abs(X).astype(np.float64) @ np.abs(W).astype(np.float64) + np.abs(b)
    assert np.allclose(o["Y_abs"], want_abs, rtol=1e-13, atol=1e-13)


@pytest.mark.parametrize("agg", ["sum", "max"])
def test_relabelling_vertices_permutes_the_output(agg):
    n = 90
    s, d = si.uniform_edges(n, 700, seed=13)
    g = si.build_csc(n, s, d)
    perm = torch.randperm(n, generator=torch.Generator().manual_seed(2))   # old id -> new id
    g2 = si.build_csc(n, perm[s], perm[d])
    rng = np.random.default_rng(6)
    X = rng.standard_normal((n, 4)).astype(np.float32)
    X2 = np.empty_like(X); X2[perm.numpy()] = X
    a = oracle.layer(*_np(g), X, "copy", agg=agg)["A"]
    b = oracle.layer(*_np(g2), X2, "copy", agg=agg)["A"]
    if agg == "max":
        assert np.array_equal(b[perm.numpy()], a)
    else:
        assert np.allclose(b[perm.numpy()], a, rtol=1e-13, atol=1e-13)


def test_sum_layer_without_activation_is_linear():
    wl = si.workload(1)
    g = wl.graph
    Z = si.normal_features(g.n, 64, seed=77).numpy()
    f = lambda x: oracle.layer(*_np(g), x, "mul_weight", wl.edge_weight.numpy(), W=wl.W.numpy())["Y"]
    a, b = 0.5, -2.0   # powers of two: a*X + b*Z has no extra rounding beyond one add
    X = wl.X.numpy()
    lhs = f((a * X + b * Z).astype(np.float32))
    rhs = a * f(X) + b * f(Z)
    assert np.abs(lhs - rhs).max() <= 1e-5 * np.abs(rhs).max()


def test_degenerate_graphs():
    # no edges at all
    g = si.csc_from_lists(5, [])
    W = np.array([[1.0, -1.0]], np.float32)
    o = oracle.layer(*_np(g), np.ones((5, 1), np.float32), "copy", W=W, bias=np.array([0.25, 0.5], np.float32), act="relu")
    assert np.array_equal(o["A"], np.zeros((5, 1))) and np.array_equal(o["Y"], np.tile([0.25, 0.5], (5, 1)))
    # a single vertex with a self-loop
    g = si.csc_from_lists(1, [(0, 0)])
    assert oracle.layer(*_np(g), np.array([[3.0, 4.0]], np.float32), "copy")["A"].tolist() == [[3.0, 4.0]]
    # star: every vertex points at vertex 0
    n = 3000
    g = si.csc_from_lists(n, [(u, 0) for u in range(n)])
    X = np.arange(n, dtype=np.float32)[:, None]
    o = oracle.layer(*_np(g), X, "copy")
    assert o["A"][0, 0] == n * (n - 1) / 2 and not o["A"][1:].any()
    # path 0 -> 1 -> 2 -> ... shifts the rows by one
    g = si.csc_from_lists(50, [(v, v + 1) for v in range(49)])
    X = np.random.default_rng(0).standard_normal((50, 3)).astype(np.float32)
    o = oracle.layer(*_np(g), X, "copy")
    assert np.array_equal(o["A"][1:], X[:-1].astype(np.float64)) and not o["A"][0].any()


def test_vertex_list_selects_rows_of_the_full_result():
    wl = si.workload(4, scale=9, f_in=8, f_out=5)
    g = wl.graph
    kw = dict(edge_op="gated", W_gate=wl.W_gate.numpy(), b_gate=wl.b_gate.numpy(), W_msg=wl.W_msg.numpy(),
              W=wl.W.numpy(), act="relu")
    full = oracle.layer(*_np(g), wl.X.numpy(), **kw)
    vl = np.array([7, 0, 300, 7, g.n - 1])
    part = oracle.layer(*_np(g), wl.X.numpy(), vlist=vl, **kw)
    for k in ("A", "A_abs", "Y", "Y_abs"):
        assert np.array_equal(part[k], full[k][vl])
    with pytest.raises(ValueError):
        oracle.layer(*_np(g), wl.X.numpy(), vlist=[g.n], **kw)


# --------------------------------------------------------------------------
# CommNet's two-term ApplyVertex (Figure 9) and the max-pooling layer (Figure 11)
# --------------------------------------------------------------------------

def test_hand_worked_commnet_apply_vertex(hand):
    y = oracle.layer(hand["csc_col_ptr"], hand["csc_row_idx"], hand["X"], "copy", W=hand["W"], W_self=hand["W_self"],
                     act="relu")["Y"]
    assert np.array_equal(y, np.array(hand["commnet_relu_Y_no_bias"], float))


def test_commnet_layer_equals_dense_form():
    g = _random_graph(120, 900, seed=41)
    rng = np.random.default_rng(2)
    X = rng.standard_normal((g.n, 6)).astype(np.float32)
    Wc = rng.standard_normal((6, 4)).astype(np.float32)
    Wh = rng.standard_normal((6, 4)).astype(np.float32)
    b = rng.standard_normal(4).astype(np.float32)
    o = oracle.layer(*_np(g), X, "copy", W=Wc, W_self=Wh, bias=b, act="relu")
    Xd = X.astype(np.float64)
    want = np.maximum(Xd @ Wh.astype(np.float64) + (_dense_adj(g) @ Xd) @ Wc.astype(np.float64) + b, 0)
    assert np.allclose(o["Y"], want, rtol=1e-12, atol=1e-12)
    want_abs = np.abs(Xd) @ np.abs(Wh).astype(np.float64) + (_dense_adj(g) @ np.abs(Xd)) @ np.abs(Wc).astype(np.float64) + np.abs(b)
    assert np.allclose(o["Y_abs"], want_abs, rtol=1e-12, atol=1e-12)
    # the self term uses the vertex's own row, not a neighbour's: zero W_C isolates it
    o2 = oracle.layer(*_np(g), X, "copy", W=np.zeros_like(Wc), W_self=Wh, act="none")
    assert np.allclose(o2["Y"], Xd @ Wh.astype(np.float64), rtol=1e-13, atol=1e-13)


def _pool_setup(n=50, m=90, F=6, Fp=4, seed=9):
    g = _random_graph(n, m, seed=seed)
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((n, F)).astype(np.float32)
    Wp = rng.standard_normal((Fp, F)).astype(np.float32)
    bp = rng.standard_normal(Fp).astype(np.float32)
    return g, X, Wp, bp


def test_max_pooling_layer_equals_dense_form():
    g, X, Wp, bp = _pool_setup()
    H = 1.0 / (1.0 + np.exp(-(X.astype(np.float64) @ Wp.astype(np.float64).T + bp)))
    Adj = _dense_adj(g)
    masked = np.where(Adj[:, :, None] > 0, H[None, :, :], -np.inf).max(axis=1)
    want = np.where(np.isfinite(masked), masked, 0.0)           # empty columns give 0
    assert (Adj.sum(1) == 0).any()
    W = np.random.default_rng(4).standard_normal((4, 3)).astype(np.float32)
    o = oracle.layer(*_np(g), X, "pool", W_pool=Wp, b_pool=bp, agg="max", W=W, act="relu")
    assert np.allclose(o["A"], want, rtol=1e-13, atol=1e-14)
    assert np.allclose(o["Y"], np.maximum(want @ W.astype(np.float64), 0), rtol=1e-12, atol=1e-13)
    # the sum accumulator over the same messages is a plain product with the adjacency matrix
    s = oracle.layer(*_np(g), X, "pool", W_pool=Wp, b_pool=bp, agg="sum")
    assert np.allclose(s["A"], Adj @ H, rtol=1e-12, atol=1e-13)
    # message uses the source row: pooling the destination's own row would give H[v] for every v with edges
    assert not np.allclose(o["A"][Adj.sum(1) > 0], H[Adj.sum(1) > 0])


def test_max_pooling_closed_forms_and_hoisting():
    g, X, Wp, bp = _pool_setup()
    deg = np.diff(g.col_ptr.numpy())
    # zero weights: every message is sigmoid(b); with b = ln 3 that is 3/4
    b = np.full(4, np.log(3.0), np.float32)
    o = oracle.layer(*_np(g), X, "pool", W_pool=np.zeros_like(Wp), b_pool=b, agg="max")
    assert np.allclose(o["A"][deg > 0], 0.75, rtol=1e-7) and not o["A"][deg == 0].any()
    # hoisting (Section 3.2) changes nothing
    a = oracle.layer(*_np(g), X, "pool", W_pool=Wp, b_pool=bp, agg="max")
    h = oracle.layer(*_np(g), X, "pool", agg="max", hoisted=oracle.hoist_pool(X, Wp, bp))
    assert np.array_equal(a["A"], h["A"]) and np.allclose(a["A_abs"], h["A_abs"], rtol=1e-13)
    H, Ha = oracle.hoist_pool(X, Wp, bp)
    Z = X.astype(np.float64) @ Wp.astype(np.float64).T + bp
    Za = np.abs(X).astype(np.float64) @ np.abs(Wp).astype(np.float64).T + np.abs(bp)
    G = 1.0 / (1.0 + np.exp(-Z))
    assert np.allclose(H, G, rtol=1e-13) and np.allclose(Ha, G * (1 + (1 - G) * Za), rtol=1e-12)


def test_sigmoid_activation_in_apply_vertex():
    g = si.csc_from_lists(4, [(v, v) for v in range(4)])
    X = np.array([[0.0], [np.log(3.0)], [-np.log(3.0)], [40.0]], np.float32)
    o = oracle.layer(*_np(g), X, "copy", W=np.array([[1.0]], np.float32), act="sigmoid")
    assert np.allclose(o["Y"][:, 0], [0.5, 0.75, 0.25, 1.0], rtol=1e-7)


# --------------------------------------------------------------------------
# backward stages (Section 2.2): pinned by the dense form and by finite differences of the
# (already pinned) forward oracle
# --------------------------------------------------------------------------

def _bwd_setup(seed=12, n=40, m=260, F=5, Fo=4):
    g = _random_graph(n, m, seed=seed)
    rng = np.random.default_rng(seed)
    # coarse values: X +- h stays exactly representable in fp32 for h = 2^-10
    X = (np.round(rng.standard_normal((n, F)) * 32) / 32).astype(np.float32)
    W = (np.round(rng.standard_normal((F, Fo)) * 32) / 32).astype(np.float32)
    Ws = (np.round(rng.standard_normal((F, Fo)) * 32) / 32).astype(np.float32)
    b = (np.round(rng.standard_normal(Fo) * 32) / 32).astype(np.float32)
    w = (np.round(rng.standard_normal(g.nnz) * 16) / 16).astype(np.float32)
    dY = rng.standard_normal((n, Fo)).astype(np.float32)
    return g, X, W, Ws, b, w, dY


@pytest.mark.parametrize("act", ["none", "relu", "sigmoid"])
@pytest.mark.parametrize("with_self", [False, True])
def test_backward_equals_dense_matrix_form(act, with_self):
    g, X, W, Ws, b, w, dY = _bwd_setup()
    Ws_ = Ws if with_self else None
    fwd = oracle.layer(*_np(g), X, "mul_weight", w, W=W, W_self=Ws_, bias=b, act="none")
    bwd = oracle.layer_backward(*_np(g), X, fwd["A"], dY, W, "mul_weight", w, bias=b, W_self=Ws_, act=act)
    Adj = _dense_adj(g, w)                                   # Adj[v, u] = w(u -> v)
    Xd, Wd, dYd = X.astype(np.float64), W.astype(np.float64), dY.astype(np.float64)
    A = Adj @ Xd
    Z = A @ Wd + b + (Xd @ Ws.astype(np.float64) if with_self else 0.0)
    Sg = 1.0 / (1.0 + np.exp(-Z))
    dZ = dYd * (Z > 0) if act == "relu" else (dYd * Sg * (1.0 - Sg) if act == "sigmoid" else dYd)
    assert np.allclose(bwd["dW"], A.T @ dZ, rtol=1e-12, atol=1e-12)
    assert np.allclose(bwd["dbias"], dZ.sum(0), rtol=1e-12, atol=1e-12)
    assert np.allclose(bwd["dA"], dZ @ Wd.T, rtol=1e-12, atol=1e-12)
    dX = Adj.T @ (dZ @ Wd.T) + (dZ @ Ws.astype(np.float64).T if with_self else 0.0)
    assert np.allclose(bwd["dX"], dX, rtol=1e-12, atol=1e-12)
    if with_self:
        assert np.allclose(bwd["dW_self"], Xd.T @ dZ, rtol=1e-12, atol=1e-12)
    # the scales: |dZ| for none and ReLU; for the sigmoid the scale of a derivative formed from the stored output
    dZa = np.abs(dZ)
    if act == "sigmoid":
        Za = np.abs(A) @ np.abs(Wd) + np.abs(b) + (np.abs(Xd) @ np.abs(Ws).astype(np.float64) if with_self else 0.0)
        D, C = Sg * (1.0 - Sg), np.abs(1.0 - 2.0 * Sg)
        dZa = np.abs(dYd) * (D + C * (D * Za + Sg))
    assert np.allclose(bwd["dW_abs"], np.abs(A).T @ dZa, rtol=1e-12, atol=1e-12)
    assert np.allclose(bwd["dbias_abs"], dZa.sum(0), rtol=1e-12, atol=1e-12)
    if with_self:
        assert np.allclose(bwd["dW_self_abs"], np.abs(Xd).T @ dZa, rtol=1e-12, atol=1e-12)
    dXa = np.abs(Adj).T @ (dZa @ np.abs(Wd).T) + (dZa @ np.abs(Ws).astype(np.float64).T if with_self else 0.0)
    assert np.allclose(bwd["dX_abs"], dXa, rtol=1e-12, atol=1e-12)


def test_sigmoid_derivative_from_the_stored_output_stays_within_its_scale():
    """The backward stage forms sigmoid'(z) from the stored fp32 output y as y (1 - y). Whatever z is, the distance of
    dY y (1 - y), evaluated in fp32, from the exact dZ is at most a few units of 2^-24 of the scale the oracle reports
    (here through dbias_abs of a one-vertex graph without edges, where za = |b|), also for saturated outputs."""
    g = si.csc_from_lists(1, [])
    X = np.zeros((1, 1), np.float32)
    W = np.zeros((1, 1), np.float32)
    for z in [-30.0, -17.0, -9.0, -2.5, -0.3, 0.0, 0.4, 3.0, 8.0, 12.5, 16.6, 25.0]:
        b = np.array([z], np.float32)
        dY = np.array([[1.7]], np.float32)
        bwd = oracle.layer_backward(*_np(g), X, np.zeros((1, 1)), dY, W, "copy", bias=b, act="sigmoid")
        sg = 1.0 / (1.0 + np.exp(-np.float64(b[0])))
        assert abs(bwd["dbias"][0] - np.float64(dY[0, 0]) * sg * (1.0 - sg)) <= 1e-15
        y = np.float32(sg)
        got = np.float32(dY[0, 0]) * (y * (np.float32(1.0) - y))
        assert abs(np.float64(got) - bwd["dbias"][0]) <= 4 * 2.0 ** -24 * bwd["dbias_abs"][0], z
        assert bwd["dbias_abs"][0] >= abs(bwd["dbias"][0])


def test_backward_matches_finite_differences_of_the_forward_oracle():
    g, X, W, Ws, b, w, dY = _bwd_setup(seed=5, n=25, m=120, F=3, Fo=3)
    R = dY.astype(np.float64)                                # loss L = sum(R * Y)
    def loss(Xp, Wp, Wsp, bp):
        y = oracle.layer(*_np(g), Xp, "mul_weight", w, W=Wp, W_self=Wsp, bias=bp, act="none")["Y"]
        return float((R * y).sum())
    fwd = oracle.layer(*_np(g), X, "mul_weight", w, W=W, W_self=Ws, bias=b, act="none")
    bwd = oracle.layer_backward(*_np(g), X, fwd["A"], dY, W, "mul_weight", w, bias=b, W_self=Ws, act="none")
    h = 2.0 ** -10
    rng = np.random.default_rng(0)
    for _ in range(12):                                       # the layer is linear in each argument: differences are exact
        u, f = rng.integers(g.n), rng.integers(3)
        Xp, Xm = X.copy(), X.copy(); Xp[u, f] += h; Xm[u, f] -= h
        num = (loss(Xp, W, Ws, b) - loss(Xm, W, Ws, b)) / (2 * h)
        assert abs(num - bwd["dX"][u, f]) <= 1e-9 * max(1.0, abs(num))
        f, o = rng.integers(3), rng.integers(3)
        Wp, Wm = W.copy(), W.copy(); Wp[f, o] += h; Wm[f, o] -= h
        num = (loss(X, Wp, Ws, b) - loss(X, Wm, Ws, b)) / (2 * h)
        assert abs(num - bwd["dW"][f, o]) <= 1e-9 * max(1.0, abs(num))
        Sp, Sm = Ws.copy(), Ws.copy(); Sp[f, o] += h; Sm[f, o] -= h
        num = (loss(X, W, Sp, b) - loss(X, W, Sm, b)) / (2 * h)
        assert abs(num - bwd["dW_self"][f, o]) <= 1e-9 * max(1.0, abs(num))
        bp, bm = b.copy(), b.copy(); bp[o] += h; bm[o] -= h
        num = (loss(X, W, Ws, bp) - loss(X, W, Ws, bm)) / (2 * h)
        assert abs(num - bwd["dbias"][o]) <= 1e-9 * max(1.0, abs(num))


def test_backward_relu_mask_and_copy_edges():
    g, X, W, Ws, b, w, dY = _bwd_setup(seed=21)
    fwd = oracle.layer(*_np(g), X, "copy", W=W, act="relu")
    bwd = oracle.layer_backward(*_np(g), X, fwd["A"], dY, W, "copy", act="relu")
    dead = fwd["Y"] <= 0
    assert dead.any() and (~dead).any()
    # a vertex whose outputs are all clipped contributes nothing to dW
    Adj = _dense_adj(g)
    dZ = np.where(dead, 0.0, dY.astype(np.float64))
    assert np.allclose(bwd["dW"], (Adj @ X.astype(np.float64)).T @ dZ, rtol=1e-12, atol=1e-12)
    assert np.allclose(bwd["dX"], Adj.T @ (dZ @ W.astype(np.float64).T), rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("act", ["none", "relu", "sigmoid"])
def test_sampled_backward_equals_the_whole_graph_form(act):
    g, X, W, Ws, b, w, dY = _bwd_setup(seed=8, n=60, m=500)
    fwd = oracle.layer(*_np(g), X, "mul_weight", w, W=W, W_self=Ws, bias=b, act="none")
    whole = oracle.layer_backward(*_np(g), X, fwd["A"], dY, W, "mul_weight", w, bias=b, W_self=Ws, act=act)
    ul = [0, 7, 33, 59, 12]
    we = [(0, 0), (4, 3), (2, 1), (4, 0)]
    part = oracle.backward_sample(*_np(g), X, fwd["A"], dY, W, ul, we, "mul_weight", w, bias=b, W_self=Ws, act=act, want_dbias=True)
    assert np.allclose(part["dX"], whole["dX"][ul], rtol=1e-12, atol=1e-13)
    assert np.allclose(part["dX_abs"], whole["dX_abs"][ul], rtol=1e-12, atol=1e-13)
    assert np.allclose(part["dW"], [whole["dW"][f, o] for f, o in we], rtol=1e-12, atol=1e-13)
    assert np.allclose(part["dW_abs"], [whole["dW_abs"][f, o] for f, o in we], rtol=1e-12, atol=1e-13)
    assert np.allclose(part["dbias"], whole["dbias"], rtol=1e-12, atol=1e-13)
    assert np.allclose(part["dbias_abs"], whole["dbias_abs"], rtol=1e-12, atol=1e-13)
    if act == "relu":
        assert not np.allclose(part["dbias"], dY.astype(np.float64).sum(0))     # the mask really removes terms


# --------------------------------------------------------------------------
# gated backward (Example 2.1 / Figure 2 through Section 2.2's backward stages)
# --------------------------------------------------------------------------

def _gated_bwd_setup(seed=3, n=30, m=170, F=4, Fo=3, with_msg=True, with_b=True):
    g = _random_graph(n, m, seed=seed)
    rng = np.random.default_rng(seed)
    q = lambda a, s: (np.round(a * s) / s).astype(np.float32)          # coarse values: +- 2^-10 stays exact in fp32
    X = q(rng.standard_normal((n, F)), 32)
    Wg = q(rng.standard_normal((F, 2 * F)) * 0.7, 32)
    bg = q(rng.standard_normal(F) * 0.5, 32) if with_b else None
    Wm = q(rng.standard_normal((F, F)) * 0.7, 32) if with_msg else None
    W = q(rng.standard_normal((F, Fo)), 32)
    b = q(rng.standard_normal(Fo) * 0.5, 32)
    dY = rng.standard_normal((n, Fo)).astype(np.float32)
    return g, X, Wg, bg, Wm, W, b, dY


@pytest.mark.parametrize("act,with_self", [("none", False), ("relu", False), ("sigmoid", False), ("relu", True), ("sigmoid", True)])
@pytest.mark.parametrize("with_msg,with_b", [(True, True), (False, False)])
def test_gated_backward_equals_autograd_of_the_dense_form(act, with_self, with_msg, with_b):
    import torch
    g, X, Wg, bg, Wm, W, b, dY = _gated_bwd_setup(with_msg=with_msg, with_b=with_b)
    n, F = X.shape
    Ws = (np.round(np.random.default_rng(77).standard_normal(W.shape) * 32) / 32).astype(np.float32) if with_self else None
    fwd = oracle.layer(*_np(g), X, "gated", W_gate=Wg, b_gate=bg, W_msg=Wm, W=W, bias=b, act=act, W_self=Ws)
    bwd = oracle.gated_backward(*_np(g), X, fwd["A"], dY, W, Wg, b_gate=bg, W_msg=Wm, bias=b, act=act, W_self=Ws)
    t = lambda a: torch.tensor(np.asarray(a, np.float64), requires_grad=True)
    Xt, Wgt, Wt, bt = t(X), t(Wg), t(W), t(b)
    Wst = t(Ws if with_self else np.zeros(W.shape))
    bgt = t(bg if with_b else np.zeros(F))
    Wmt = t(Wm if with_msg else np.eye(F))
    Adj = torch.tensor(_dense_adj(g))                                    # Adj[v, u] = 1 for an edge u -> v
    Ps, Pd, M = Xt @ Wgt[:, :F].T, Xt @ Wgt[:, F:].T, Xt @ Wmt.T
    gate = torch.sigmoid(Ps[None, :, :] + Pd[:, None, :] + bgt)           # [v, u, f]
    A = (Adj[:, :, None] * gate * M[None, :, :]).sum(1)
    Z = A @ Wt + Xt @ Wst + bt
    Y = torch.relu(Z) if act == "relu" else (torch.sigmoid(Z) if act == "sigmoid" else Z)
    assert np.allclose(Y.detach().numpy(), fwd["Y"], rtol=1e-12, atol=1e-12)
    (Y * torch.tensor(dY.astype(np.float64))).sum().backward()
    for name, ref in [("dX", Xt.grad), ("dW", Wt.grad), ("dbias", bt.grad), ("dW_gate", Wgt.grad), ("db_gate", bgt.grad),
                      ("dW_msg", Wmt.grad)] + ([("dW_self", Wst.grad)] if with_self else []):
        assert np.allclose(bwd[name], ref.numpy(), rtol=1e-10, atol=1e-11), name
    for name in ["dX", "dW", "dW_gate", "db_gate", "dW_msg", "dbias"] + (["dW_self"] if with_self else []):
        assert (bwd[name + "_abs"] >= np.abs(bwd[name]) * (1 - 1e-12)).all(), name    # a scale bounds its value


@pytest.mark.parametrize("act,with_self", [("none", False), ("relu", False), ("sigmoid", True), ("relu", True)])
@pytest.mark.parametrize("with_msg,with_b", [(True, True), (False, False)])
def test_gated_max_backward_equals_autograd_of_the_dense_form(act, with_self, with_msg, with_b):
    """Max over gated messages: the recomputed Gather output is the forward oracle's, and every gradient is what autograd
    gives for the dense formulation (amax over a masked [v, u, f] tensor; no two messages of a column tie here)."""
    import torch
    g, X, Wg, bg, Wm, W, b, dY = _gated_bwd_setup(seed=4, n=40, m=90, with_msg=with_msg, with_b=with_b)
    n, F = X.shape
    deg = np.diff(g.col_ptr.numpy())
    assert (deg == 0).any() and (deg > 3).any()
    Ws = (np.round(np.random.default_rng(78).standard_normal(W.shape) * 32) / 32).astype(np.float32) if with_self else None
    fwd = oracle.layer(*_np(g), X, "gated", agg="max", W_gate=Wg, b_gate=bg, W_msg=Wm, W=W, bias=b, act=act, W_self=Ws)
    bwd = oracle.gated_backward(*_np(g), X, None, dY, W, Wg, b_gate=bg, W_msg=Wm, bias=b, act=act, W_self=Ws, agg="max")
    assert np.allclose(bwd["A"], fwd["A"], rtol=1e-12, atol=1e-13)
    t = lambda a: torch.tensor(np.asarray(a, np.float64), requires_grad=True)
    Xt, Wgt, Wt, bt = t(X), t(Wg), t(W), t(b)
    Wst = t(Ws if with_self else np.zeros(W.shape))
    bgt = t(bg if with_b else np.zeros(F))
    Wmt = t(Wm if with_msg else np.eye(F))
    Adj = torch.tensor(_dense_adj(g)) > 0                                 # [v, u]
    Ps, Pd, M = Xt @ Wgt[:, :F].T, Xt @ Wgt[:, F:].T, Xt @ Wmt.T
    msg = torch.sigmoid(Ps[None, :, :] + Pd[:, None, :] + bgt) * M[None, :, :]      # [v, u, f]
    masked = torch.where(Adj[:, :, None], msg, torch.tensor(-np.inf, dtype=torch.float64))
    A = torch.where(Adj.any(1)[:, None], masked.amax(1), torch.zeros(n, F, dtype=torch.float64))
    Z = A @ Wt + Xt @ Wst + bt
    Y = torch.relu(Z) if act == "relu" else (torch.sigmoid(Z) if act == "sigmoid" else Z)
    assert np.allclose(Y.detach().numpy(), fwd["Y"], rtol=1e-12, atol=1e-12)
    (Y * torch.tensor(dY.astype(np.float64))).sum().backward()
    for name, ref in [("dX", Xt.grad), ("dW", Wt.grad), ("dbias", bt.grad), ("dW_gate", Wgt.grad), ("db_gate", bgt.grad),
                      ("dW_msg", Wmt.grad)] + ([("dW_self", Wst.grad)] if with_self else []):
        assert np.allclose(bwd[name], ref.numpy(), rtol=1e-10, atol=1e-11), name
        assert np.abs(ref.numpy()).max() > 1e-3, name
    for name in ["dX", "dW", "dW_gate", "db_gate", "dW_msg", "dbias"] + (["dW_self"] if with_self else []):
        assert (bwd[name + "_abs"] >= np.abs(bwd[name]) * (1 - 1e-12)).all(), name
    # it is not the sum layer's gradient: with more than one in-edge somewhere, most edges carry nothing
    sum_fwd = oracle.layer(*_np(g), X, "gated", W_gate=Wg, b_gate=bg, W_msg=Wm, W=W, bias=b, act=act, W_self=Ws)
    sum_bwd = oracle.gated_backward(*_np(g), X, sum_fwd["A"], dY, W, Wg, b_gate=bg, W_msg=Wm, bias=b, act=act, W_self=Ws)
    assert not np.allclose(sum_bwd["dW_gate"], bwd["dW_gate"], rtol=1e-3, atol=1e-6)


def test_gated_max_backward_on_a_tie_and_on_a_single_edge():
    # vertices 0 and 1 carry the same features: their messages to vertex 2 tie in every feature, both get the whole gradient;
    # vertex 3 has the single in-edge 2 -> 3, where max and sum are the same layer
    g = si.csc_from_lists(4, [(0, 2), (1, 2), (2, 3)])
    X = np.array([[0.5, -1.0], [0.5, -1.0], [0.25, 2.0], [1.0, 1.0]], np.float32)
    Wg = np.array([[0.5, 0.25, -0.5, 1.0], [1.0, -0.75, 0.25, 0.5]], np.float32)
    W = np.array([[1.0, 0.5], [-0.5, 2.0]], np.float32)
    dY = np.array([[0, 0], [0, 0], [3.0, 7.0], [-2.0, 0.5]], np.float32)
    mx = oracle.gated_backward(*_np(g), X, None, dY, W, Wg, agg="max")
    fwd = oracle.layer(*_np(g), X, "gated", W_gate=Wg, W=W)
    sm = oracle.gated_backward(*_np(g), X, fwd["A"], dY, W, Wg)
    assert np.allclose(mx["A"][3], fwd["A"][3], rtol=1e-14) and np.allclose(mx["A"][2], fwd["A"][2] / 2, rtol=1e-14)
    assert np.array_equal(mx["dX"][0], mx["dX"][1]) and np.abs(mx["dX"][0]).max() > 0
    # per edge the two layers send back the same thing when both edges of vertex 2 are maximal: the sum layer's dA[2] is
    # dZ[2] W^T as well, so the rows of the two tied sources agree between the layers, and so does everything at vertex 3
    assert np.allclose(mx["dX"][0], sm["dX"][0], rtol=1e-13, atol=1e-15)
    assert np.allclose(mx["dW_gate"], sm["dW_gate"], rtol=1e-13, atol=1e-15)
    assert np.allclose(mx["dW_msg"], sm["dW_msg"], rtol=1e-13, atol=1e-15)
    # dW = A^T dZ differs: the max layer's A[2] is one message, the sum layer's two
    assert not np.allclose(mx["dW"], sm["dW"])


@pytest.mark.parametrize("with_msg,with_b", [(True, True), (False, False)])
def test_sampled_gated_backward_equals_the_whole_graph_form(with_msg, with_b):
    g, X, Wg, bg, Wm, W, b, dY = _gated_bwd_setup(seed=6, n=70, m=600, F=5, Fo=4, with_msg=with_msg, with_b=with_b)
    fwd = oracle.layer(*_np(g), X, "gated", W_gate=Wg, b_gate=bg, W_msg=Wm, W=W, bias=b, act="none")
    whole = oracle.gated_backward(*_np(g), X, fwd["A"], dY, W, Wg, b_gate=bg, W_msg=Wm, bias=b, act="none")
    od = np.bincount(g.row_idx.numpy(), minlength=g.n)
    ul = sorted({0, 69, 13, 41, int(od.argmax()), int(od.argmin()), int(np.diff(g.col_ptr.numpy()).argmax())})
    part = oracle.gated_backward_sample(*_np(g), X, dY, W, Wg, ul, b_gate=bg, W_msg=Wm)
    assert np.allclose(part["dX"], whole["dX"][ul], rtol=1e-12, atol=1e-13)
    assert np.allclose(part["dX_abs"], whole["dX_abs"][ul], rtol=1e-12, atol=1e-13)
    assert np.abs(whole["dX"][ul]).max() > 0.1


def test_gated_backward_matches_finite_differences_of_the_naive_forward_oracle():
    g, X, Wg, bg, Wm, W, b, dY = _gated_bwd_setup(seed=9, n=20, m=90, F=3, Fo=2)
    R = dY.astype(np.float64)
    def loss(X_=X, Wg_=Wg, bg_=bg, Wm_=Wm, W_=W, b_=b):
        return float((R * oracle.layer(*_np(g), X_, "gated", W_gate=Wg_, b_gate=bg_, W_msg=Wm_, W=W_, bias=b_, act="none")["Y"]).sum())
    fwd = oracle.layer(*_np(g), X, "gated", W_gate=Wg, b_gate=bg, W_msg=Wm, W=W, bias=b, act="none")
    bwd = oracle.gated_backward(*_np(g), X, fwd["A"], dY, W, Wg, b_gate=bg, W_msg=Wm, bias=b, act="none")
    h = 2.0 ** -10
    rng = np.random.default_rng(1)
    def fd(name, arr, idx):
        p, m = arr.copy(), arr.copy()
        p[idx] += h
        m[idx] -= h
        return (loss(**{name: p}) - loss(**{name: m})) / (2 * h)
    for _ in range(10):
        u, k, f, k2 = rng.integers(g.n), rng.integers(3), rng.integers(3), rng.integers(6)
        checks = [(fd("X_", X, (u, k)), bwd["dX"][u, k]), (fd("Wg_", Wg, (f, k2)), bwd["dW_gate"][f, k2]),
                  (fd("bg_", bg, (f,)), bwd["db_gate"][f]), (fd("Wm_", Wm, (f, k)), bwd["dW_msg"][f, k])]
        for num, ana in checks:                                   # central differences: error O(h^2)
            assert abs(num - ana) <= 2e-5 * max(1.0, abs(ana)), (num, ana)


# --------------------------------------------------------------------------
# max-accumulator backward (Figure 11's layer, and max over COPY / MUL_WEIGHT messages)
# --------------------------------------------------------------------------

def _max_bwd_setup(seed=4, n=40, m=70, F=5, Fp=4, Fo=3):
    g = _random_graph(n, m, seed=seed)
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((n, F)).astype(np.float32)
    w = (rng.standard_normal(g.nnz) * 0.8).astype(np.float32)        # both signs: a negative weight flips the order
    Wp = (rng.standard_normal((Fp, F)) * 0.6).astype(np.float32)
    bp = (rng.standard_normal(Fp) * 0.3).astype(np.float32)
    b = (rng.standard_normal(Fo) * 0.3).astype(np.float32)
    return g, X, w, Wp, bp, b, rng


@pytest.mark.parametrize("edge_op", ["copy", "mul_weight", "pool"])
@pytest.mark.parametrize("act,with_self", [("none", False), ("relu", False), ("sigmoid", False), ("relu", True), ("sigmoid", True)])
def test_max_backward_equals_autograd_of_the_dense_form(edge_op, act, with_self):
    import torch
    g, X, w, Wp, bp, b, rng = _max_bwd_setup()
    n, F = X.shape
    Fm = Wp.shape[0] if edge_op == "pool" else F
    W = rng.standard_normal((Fm, 3)).astype(np.float32)
    dY = rng.standard_normal((n, 3)).astype(np.float32)
    Ws = rng.standard_normal((F, 3)).astype(np.float32) if with_self else None
    deg = np.diff(g.col_ptr.numpy())
    assert (deg == 0).any() and (deg > 1).any()
    kw = dict(edge_weight=w) if edge_op == "mul_weight" else (dict(W_pool=Wp, b_pool=bp) if edge_op == "pool" else {})
    fwd = oracle.layer(*_np(g), X, edge_op, agg="max", W=W, bias=b, act=act, W_self=Ws, **kw)
    bwd = oracle.max_backward(*_np(g), X, dY, W, edge_op, bias=b, act=act, W_self=Ws, **kw)
    assert np.array_equal(bwd["A"], fwd["A"])                             # the Gather it differentiates is the pinned one
    t = lambda a: torch.tensor(np.asarray(a, np.float64), requires_grad=True)
    Xt, Wt, bt, Wpt, bpt = t(X), t(W), t(b), t(Wp), t(bp)
    Wst = t(Ws if with_self else np.zeros((F, 3)))
    Adj = torch.tensor(_dense_adj(g)) > 0                                  # [v, u]
    if edge_op == "pool":
        S = torch.sigmoid(Xt @ Wpt.T + bpt)[None, :, :].expand(n, n, Fm)
    elif edge_op == "mul_weight":
        # the message is one fp32 multiply: form it in fp32, differentiate through the fp64 product, which agrees to rounding
        Wd = torch.tensor(_dense_adj(g, w))
        S = Wd[:, :, None] * Xt[None, :, :]
    else:
        S = Xt[None, :, :].expand(n, n, F)
    masked = torch.where(Adj[:, :, None], S, torch.tensor(-np.inf, dtype=torch.float64))
    A = torch.where(Adj.any(1)[:, None], masked.amax(1), torch.zeros(n, Fm, dtype=torch.float64))
    Z = A @ Wt + Xt @ Wst + bt
    Y = torch.relu(Z) if act == "relu" else (torch.sigmoid(Z) if act == "sigmoid" else Z)
    assert np.allclose(Y.detach().numpy(), fwd["Y"], rtol=1e-6, atol=1e-7)
    (Y * torch.tensor(dY.astype(np.float64))).sum().backward()
    tol = dict(rtol=1e-6, atol=1e-7) if edge_op == "mul_weight" else dict(rtol=1e-10, atol=1e-11)
    assert np.allclose(bwd["dX"], Xt.grad.numpy(), **tol)
    assert np.allclose(bwd["dW"], Wt.grad.numpy(), **tol)
    assert np.allclose(bwd["dbias"], bt.grad.numpy(), **tol)
    if with_self:
        assert np.allclose(bwd["dW_self"], Wst.grad.numpy(), **tol)
        assert (bwd["dW_self_abs"] >= np.abs(bwd["dW_self"]) * (1 - 1e-12)).all()
    assert (bwd["dbias_abs"] >= np.abs(bwd["dbias"]) * (1 - 1e-12)).all()
    if edge_op == "pool":
        assert np.allclose(bwd["dW_pool"], Wpt.grad.numpy(), **tol)
        assert np.allclose(bwd["db_pool"], bpt.grad.numpy(), **tol)
    for name in ["dX", "dW"] + (["dW_pool", "db_pool"] if edge_op == "pool" else []):
        assert (bwd[name + "_abs"] >= np.abs(bwd[name]) * (1 - 1e-12)).all(), name


@pytest.mark.parametrize("edge_op", ["copy", "mul_weight", "pool"])
@pytest.mark.parametrize("act,with_self", [("none", False), ("relu", False), ("sigmoid", True), ("relu", True)])
def test_sampled_max_backward_equals_the_whole_graph_form_and_autograd(edge_op, act, with_self):
    """Rows of dX from the sampled form: the same numbers as the whole-graph form (itself pinned to autograd above), and
    directly the gradient autograd gives for those rows of the dense formulation."""
    import torch
    g, X, w, Wp, bp, b, rng = _max_bwd_setup(seed=8, n=60, m=400)
    n, F = X.shape
    Fm = Wp.shape[0] if edge_op == "pool" else F
    W = rng.standard_normal((Fm, 3)).astype(np.float32)
    dY = rng.standard_normal((n, 3)).astype(np.float32)
    Ws = rng.standard_normal((F, 3)).astype(np.float32) if with_self else None
    kw = dict(edge_weight=w) if edge_op == "mul_weight" else (dict(W_pool=Wp, b_pool=bp) if edge_op == "pool" else {})
    whole = oracle.max_backward(*_np(g), X, dY, W, edge_op, bias=b, act=act, W_self=Ws, **kw)
    od = np.bincount(g.row_idx.numpy(), minlength=n)
    deg = np.diff(g.col_ptr.numpy())
    ul = sorted({0, n - 1, 13, 41, int(od.argmax()), int(od.argmin()), int(deg.argmax()), int(deg.argmin())})
    part = oracle.max_backward_sample(*_np(g), X, dY, W, ul, edge_op, bias=b, act=act, W_self=Ws, **kw)
    assert np.allclose(part["dX"], whole["dX"][ul], rtol=1e-12, atol=1e-13)
    assert np.allclose(part["dX_abs"], whole["dX_abs"][ul], rtol=1e-12, atol=1e-13)
    assert np.abs(whole["dX"][ul]).max() > 0.05
    t = lambda a: torch.tensor(np.asarray(a, np.float64), requires_grad=True)
    Xt = t(X)
    Adj = torch.tensor(_dense_adj(g)) > 0
    if edge_op == "pool":
        S = torch.sigmoid(Xt @ torch.tensor(Wp, dtype=torch.float64).T + torch.tensor(bp, dtype=torch.float64))[None, :, :].expand(n, n, Fm)
    elif edge_op == "mul_weight":
        S = torch.tensor(_dense_adj(g, w))[:, :, None] * Xt[None, :, :]
    else:
        S = Xt[None, :, :].expand(n, n, F)
    masked = torch.where(Adj[:, :, None], S, torch.tensor(-np.inf, dtype=torch.float64))
    A = torch.where(Adj.any(1)[:, None], masked.amax(1), torch.zeros(n, Fm, dtype=torch.float64))
    Z = A @ torch.tensor(W, dtype=torch.float64) + torch.tensor(b, dtype=torch.float64)
    if with_self:
        Z = Z + Xt @ torch.tensor(Ws, dtype=torch.float64)
    Y = torch.relu(Z) if act == "relu" else (torch.sigmoid(Z) if act == "sigmoid" else Z)
    (Y * torch.tensor(dY.astype(np.float64))).sum().backward()
    tol = dict(rtol=1e-6, atol=1e-7) if edge_op == "mul_weight" else dict(rtol=1e-10, atol=1e-11)
    assert np.allclose(part["dX"], Xt.grad.numpy()[ul], **tol)


def test_sampled_max_backward_on_ties_and_rejected_arguments():
    g = si.csc_from_lists(3, [(0, 2), (1, 2)])
    X = np.array([[2.0, 1.0], [2.0, 5.0], [0.0, 0.0]], np.float32)
    W = np.eye(2, dtype=np.float32)
    dY = np.array([[0, 0], [0, 0], [3.0, 7.0]], np.float32)
    part = oracle.max_backward_sample(*_np(g), X, dY, W, [1, 0, 2], "copy")
    assert np.array_equal(part["dX"], [[3, 7], [3, 0], [0, 0]])            # rows in the order asked for; the tie gives both 3
    assert oracle.max_backward_sample(*_np(g), X, dY, W, [], "copy")["dX"].shape == (0, 2)
    with pytest.raises(ValueError):
        oracle.max_backward_sample(*_np(g), X, dY, W, [3], "copy")


def test_max_backward_sends_the_whole_gradient_to_every_tied_source():
    # vertex 2 has in-edges from 0 and 1 with equal features in column 0 and distinct ones in column 1
    g = si.csc_from_lists(3, [(0, 2), (1, 2)])
    X = np.array([[2.0, 1.0], [2.0, 5.0], [0.0, 0.0]], np.float32)
    W = np.eye(2, dtype=np.float32)
    dY = np.array([[0, 0], [0, 0], [3.0, 7.0]], np.float32)
    bwd = oracle.max_backward(*_np(g), X, dY, W, "copy")
    assert np.array_equal(bwd["A"], [[0, 0], [0, 0], [2, 5]])
    assert np.array_equal(bwd["dX"], [[3, 0], [3, 7], [0, 0]])            # the tie in column 0: both get 3
    assert np.array_equal(bwd["dW"], [[6, 14], [15, 35]])                  # A^T dZ

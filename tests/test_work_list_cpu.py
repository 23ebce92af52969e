"""The host-side work list (no GPU): every edge exactly once, cuts on stripe boundaries,
slots contiguous per vertex, pieces ordered by source stripe."""
import numpy as np
import pytest
import torch

import paper_1810_08403_amd as saga
import saga_inputs as si


def _plan(g, **kw):
    items, info = saga.plan_work_list(g.col_ptr, g.row_idx, **kw)
    return items.numpy(), info


@pytest.mark.parametrize("kw", [dict(min_edges=64, cut_degree=128, stripe_rows=256),
                                dict(min_edges=16, cut_degree=16, stripe_rows=64),
                                dict(min_edges=100, cut_degree=300, stripe_rows=0),
                                dict(min_edges=256, cut_degree=512, stripe_rows=1024),
                                dict(min_edges=64, cut_degree=1 << 30, stripe_rows=256)])
def test_work_list_partitions_the_edges(kw):
    g = si.workload(3, scale=12, edge_factor=60).graph
    cp, ri = g.col_ptr.numpy(), g.row_idx.numpy()
    items, info = _plan(g, **kw)
    assert info["n_items"] == len(items)
    cover = np.zeros(g.nnz + 1, np.int64)
    np.add.at(cover, items[:, 1], 1)
    np.add.at(cover, items[:, 2], -1)
    assert (np.cumsum(cover)[:-1] == 1).all()                  # each edge in exactly one item
    v, e0, e1, slot = items.T
    assert (e0 >= cp[v]).all() and (e1 <= cp[v + 1]).all() and (e0 <= e1).all()
    whole = slot < 0
    assert (e0[whole] == cp[v[whole]]).all() and (e1[whole] == cp[v[whole] + 1]).all()
    # a column above cut_degree stays whole only if cutting it would give a single piece
    one_piece = kw["min_edges"] + kw["stripe_rows"] + kw["min_edges"] // 2
    assert ((e1 - e0)[whole] <= max(kw["cut_degree"], one_piece)).all()
    assert set(v[whole]).isdisjoint(set(v[~whole])) and len(set(v)) == g.n   # every vertex has an item
    # slots: 0..n_slots-1, each once; per vertex contiguous and in edge order
    s = slot[~whole]
    assert sorted(s.tolist()) == list(range(info["n_slots"]))
    order = np.argsort(s)
    vs, es = v[~whole][order], e0[~whole][order]
    assert (np.diff(vs) >= 0).all()
    same = np.diff(vs) == 0
    assert (np.diff(es)[same] > 0).all()
    assert info["n_split_vertices"] == len(set(vs.tolist()))
    # piece sizes and stripe alignment
    ln = (e1 - e0)[~whole]
    R, m = kw["stripe_rows"], kw["min_edges"]
    last = e1[~whole] == cp[v[~whole] + 1]
    assert (ln[~last] >= m).all()
    if R > 0:
        assert (ln <= m + R + m // 2).all()
        inner_end = e1[~whole][~last]
        assert (ri[inner_end] // R > ri[inner_end - 1] // R).all()     # a cut sits on a stripe boundary
        first_stripe = ri[e0[~whole]] // R
        assert (np.diff(first_stripe) >= 0).all()                       # pieces come stripe by stripe
    assert whole[np.argmax(whole):].all()                               # whole columns follow the pieces


def test_work_list_of_degenerate_graphs():
    g = si.csc_from_lists(5, [])
    items, info = _plan(g)
    assert info == {"n_items": 5, "n_split_vertices": 0, "n_slots": 0} and (items[:, 3] == -1).all()
    g = si.csc_from_lists(3000, [(u, 7) for u in range(3000)])
    items, info = _plan(g, min_edges=100, cut_degree=200, stripe_rows=128)
    assert info["n_split_vertices"] == 1 and info["n_slots"] == info["n_items"] - 2999
    assert (items[items[:, 3] >= 0][:, 0] == 7).all()

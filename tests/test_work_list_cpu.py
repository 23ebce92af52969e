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


@pytest.mark.parametrize("kw", [dict(min_edges=64, cut_degree=128, stripe_rows=256, team=1),
                                dict(min_edges=16, cut_degree=16, stripe_rows=64, team=1),
                                dict(min_edges=100, cut_degree=300, stripe_rows=0, team=1),
                                dict(min_edges=64, cut_degree=128, stripe_rows=1024, team=4),
                                dict(min_edges=16, cut_degree=32, stripe_rows=128, team=4),
                                dict(min_edges=50, cut_degree=100, stripe_rows=0, team=4),
                                dict(min_edges=64, cut_degree=1 << 30, stripe_rows=256, team=4)])
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
    nt = info["n_team_items"]
    assert nt == (0 if kw["team"] == 1 else nt) and (kw["team"] == 4 or nt == 0)
    is_team = np.arange(len(items)) < nt
    whole = slot < 0
    assert (e0[whole] == cp[v[whole]]).all() and (e1[whole] == cp[v[whole] + 1]).all()
    assert len(set(v)) == g.n                                   # every vertex has an item
    assert set(v[whole]).isdisjoint(set(v[~whole]))
    # solo items are whole columns at or below cut_degree (or, without teams, columns that gave one piece)
    min_piece = kw["min_edges"] * kw["team"]
    one_piece = min_piece + kw["stripe_rows"] + min_piece // 2
    solo = ~is_team
    if kw["team"] == 4:
        assert whole[solo].all() and ((e1 - e0)[solo] <= kw["cut_degree"]).all()
        assert ((e1 - e0)[is_team] > 0).all()
        assert ((cp[v[is_team] + 1] - cp[v[is_team]]) > kw["cut_degree"]).all()    # teams only work cut columns
    else:
        assert ((e1 - e0)[whole] <= max(kw["cut_degree"], one_piece)).all()
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
    R = kw["stripe_rows"]
    last = e1[~whole] == cp[v[~whole] + 1]
    assert (ln[~last] >= min_piece).all()
    if R > 0:
        assert (ln <= min_piece + R + min_piece // 2).all()
        inner_end = e1[~whole][~last]
        assert (ri[inner_end] // R > ri[inner_end - 1] // R).all()     # a cut sits on a stripe boundary
        pieces = is_team if kw["team"] == 4 else ~whole
        first_stripe = ri[e0[pieces]] // R
        assert (np.diff(first_stripe) >= 0).all()                       # pieces come stripe by stripe
        last_stripe = ri[e1[pieces] - 1] // R                             # ... and within a stripe by the stripe they reach
        same_first = np.diff(first_stripe) == 0
        assert (np.diff(last_stripe)[same_first] >= 0).all()
    if kw["team"] == 1:
        assert whole[np.argmax(whole):].all()                           # whole columns follow the pieces


def test_work_list_of_degenerate_graphs():
    g = si.csc_from_lists(5, [])
    items, info = _plan(g)
    assert info == {"n_items": 5, "n_team_items": 0, "n_split_vertices": 0, "n_slots": 0} and (items[:, 3] == -1).all()
    g = si.csc_from_lists(3000, [(u, 7) for u in range(3000)])
    for team in (1, 4):
        items, info = _plan(g, min_edges=100, cut_degree=200, stripe_rows=128, team=team)
        assert info["n_split_vertices"] == 1 and info["n_slots"] == info["n_items"] - 2999
        assert (items[items[:, 3] >= 0][:, 0] == 7).all()
        assert info["n_team_items"] == (info["n_slots"] if team == 4 else 0)
    # a column just above cut_degree is one team item that writes its row directly
    g = si.csc_from_lists(400, [(u, 3) for u in range(300)])
    items, info = _plan(g, min_edges=64, cut_degree=128, stripe_rows=1024, team=4)
    assert info["n_team_items"] == 1 and info["n_slots"] == 0 and items[0].tolist() == [3, 0, 300, -1]


# --------------------------------------------------------------------------
# vertex id re-encoding for chunk balance (Section 3.1)
# --------------------------------------------------------------------------

def _chunk_counts(g, Q, P):
    n = g.n
    Dq, Sp = -(-n // Q), -(-n // P)
    deg = (g.col_ptr[1:] - g.col_ptr[:-1])
    dst = torch.repeat_interleave(torch.arange(n), deg)
    cell = (dst // Dq) * P + g.row_idx.long() // Sp
    return torch.bincount(cell, minlength=Q * P)


@pytest.mark.parametrize("Q,P", [(4, 4), (1, 16), (2, 8), (3, 7)])
def test_reencoding_is_a_permutation_that_evens_out_the_chunks(Q, P):
    import paper_1810_08403_amd as saga
    src, dst = si.rmat_edges(13, 16 << 13, seed=5)
    g = si.build_csc(1 << 13, src, dst, self_loops=True)
    new_id, stats = saga.plan_reencoding(g.col_ptr, g.row_idx, Q, P, seed=3)
    assert torch.equal(torch.sort(new_id.long()).values, torch.arange(g.n))
    before = _chunk_counts(g, Q, P)
    g2 = si.relabel_csc(g, new_id)
    after = _chunk_counts(g2, Q, P)
    assert g2.nnz == g.nnz
    assert stats["before"] == {"max_chunk_edges": int(before.max()), "min_chunk_edges": int(before.min()), "chunks": Q * P}
    assert stats["after"] == {"max_chunk_edges": int(after.max()), "min_chunk_edges": int(after.min()), "chunks": Q * P}
    mean = g.nnz / (Q * P)
    assert before.max() > 2.0 * mean                    # R-MAT without permutation: a few chunks hold most edges
    assert after.max() < 1.5 * mean and after.max() < 0.7 * before.max()   # what is left is the heaviest vertices themselves
    # degrees travel with the vertices
    assert torch.equal(g2.in_degree()[new_id.long()], g.in_degree())


def test_reencoding_is_deterministic_in_the_seed_and_rejects_bad_tilings():
    import paper_1810_08403_amd as saga
    g = si.build_csc(1000, *si.uniform_edges(1000, 8000, seed=2))
    a, _ = saga.plan_reencoding(g.col_ptr, g.row_idx, 2, 5, seed=1)
    b, _ = saga.plan_reencoding(g.col_ptr, g.row_idx, 2, 5, seed=1)
    c, _ = saga.plan_reencoding(g.col_ptr, g.row_idx, 2, 5, seed=2)
    assert torch.equal(a, b) and not torch.equal(a, c)
    for Q, P in [(0, 4), (5, 4), (1, 1001)]:
        with pytest.raises(saga.SagaError):
            saga.plan_reencoding(g.col_ptr, g.row_idx, Q, P)

"""Seeded generators: determinism, CSC well-formedness, stated distributions."""
import numpy as np
import torch

import saga_inputs as si


def test_hash_is_deterministic_and_sliceable():
    a = si.rand_u64(7, 3, 0, 1000)
    b = si.rand_u64(7, 3, 500, 500)
    assert torch.equal(a[500:], b)
    assert not torch.equal(a, si.rand_u64(8, 3, 0, 1000))
    assert not torch.equal(a, si.rand_u64(7, 4, 0, 1000))


def test_mix64_matches_python_big_int_arithmetic():
    # the torch int64 wrap-around version against exact unsigned arithmetic
    M = (1 << 64) - 1
    def ref(v):
        v &= M
        v = ((v ^ (v >> 30)) * 0xBF58476D1CE4E5B9) & M
        v = ((v ^ (v >> 27)) * 0x94D049BB133111EB) & M
        return v ^ (v >> 31)
    xs = [0, 1, 2, 12345678901234567, (1 << 63) + 5, M]
    t = torch.tensor([x - (1 << 64) if x >= (1 << 63) else x for x in xs], dtype=torch.int64)
    got = [int(v) & M for v in si.mix64(t).tolist()]
    assert got == [ref(x) for x in xs]


def test_uniform_and_normal_moments():
    u = si.uniform01(1, 9, 200000, dtype=torch.float64)
    assert 0.0 < u.min() and u.max() < 1.0
    assert abs(u.mean().item() - 0.5) < 5e-3 and abs(u.var().item() - 1 / 12) < 2e-3
    z = si.normal(1, 9, 200000, dtype=torch.float64)
    assert abs(z.mean().item()) < 1e-2 and abs(z.std().item() - 1.0) < 1e-2
    assert abs((z ** 3).mean().item()) < 5e-2


def test_csc_is_sorted_unique_and_complete():
    n = 64
    src, dst = si.uniform_edges(n, 2000, seed=5)
    g = si.build_csc(n, src, dst, symmetrise=True, self_loops=True)
    cp, ri = g.col_ptr.numpy(), g.row_idx.numpy()
    assert cp[0] == 0 and cp[-1] == g.nnz and (np.diff(cp) >= 1).all()
    want = set()
    for s, d in zip(src.tolist(), dst.tolist()):
        want.add((s, d)); want.add((d, s))
    for v in range(n):
        want.add((v, v))
    got = set()
    for v in range(n):
        col = ri[cp[v]:cp[v + 1]]
        assert (np.diff(col) > 0).all()
        got.update((int(u), v) for u in col)
    assert got == want


def test_edge_order_does_not_change_the_csc():
    n = 100
    src, dst = si.uniform_edges(n, 3000, seed=11)
    perm = torch.randperm(3000, generator=torch.Generator().manual_seed(0))
    g1 = si.build_csc(n, src, dst)
    g2 = si.build_csc(n, src[perm], dst[perm])
    assert torch.equal(g1.col_ptr, g2.col_ptr) and torch.equal(g1.row_idx, g2.row_idx)


def test_rmat_quadrant_probabilities_and_skew():
    scale, m = 10, 400000
    src, dst = si.rmat_edges(scale, m, seed=3)
    top_s = (src >> (scale - 1)).double().mean().item()   # P(src top bit = 1) = c + d
    top_d = (dst >> (scale - 1)).double().mean().item()   # P(dst top bit = 1) = b + d
    both0 = ((src >> (scale - 1) == 0) & (dst >> (scale - 1) == 0)).double().mean().item()
    assert abs(top_s - 0.24) < 5e-3 and abs(top_d - 0.24) < 5e-3 and abs(both0 - 0.57) < 5e-3
    # vertex 0 is the heaviest destination: P = (a + c)^scale
    p0 = (dst == 0).double().mean().item()
    assert abs(p0 - 0.76 ** scale) / 0.76 ** scale < 0.05
    assert src.min() >= 0 and src.max() < (1 << scale)


def test_gcn_weights_follow_in_degree():
    g = si.csc_from_lists(4, [(0, 1), (2, 1), (3, 1), (1, 0), (0, 0), (1, 1)])
    w = si.gcn_edge_weights(g).numpy()
    deg = g.in_degree().numpy().clip(min=1)
    dst = g.dst_of_edges().numpy()
    for e in range(g.nnz):
        want = np.float32(1.0 / np.sqrt(float(deg[g.row_idx[e]]) * float(deg[dst[e]])))
        assert w[e] == want


def test_workloads_have_the_stated_shapes():
    w1 = si.workload(1)
    assert w1.graph.n == 4096 and w1.X.shape == (4096, 64) and w1.W.shape == (64, 64)
    assert 32768 < w1.graph.nnz <= 32768 + 4096
    lim = (6 / 128) ** 0.5
    assert w1.W.abs().max().item() <= lim
    w2 = si.workload(2, scale=10)
    assert w2.X.shape[1] == 500 and w2.W.shape == (500, 16) and w2.extra["W2"].shape == (16, 3)
    assert abs((w2.X != 0).float().mean().item() - 0.1) < 0.01 and w2.X.min() >= 0
    w3 = si.workload(3, scale=8, edge_factor=20)
    assert w3.dtype == "bf16" and torch.equal(w3.X, si.round_to_bf16(w3.X))
    w4 = si.workload(4, scale=10)
    assert w4.W_gate.shape == (128, 256) and w4.W_msg.shape == (128, 128) and w4.b_gate.abs().max() <= 0.1
    assert (w4.graph.in_degree() == 0).any()          # no self-loops => empty columns exist
    w5 = si.workload(5, scale=8, edge_factor=8, f_in=32, f_out=32)
    assert (w5.graph.in_degree() >= 1).all()


def test_bf16_bits_roundtrip():
    x = si.round_to_bf16(si.normal(3, 1, 1000))
    bits = si.bf16_bits(x)
    back = (bits.to(torch.int32) << 16).view(torch.float32)
    assert torch.equal(back, x)

"""Seeded synthetic inputs for SAGA-NN layers (graphs, features, parameters).

This module serves both the CPU oracle's tests and the HIP path's tests/bench.
It holds none of the layer's arithmetic: it only draws random graphs and
tensors, sorts edges into destination-major CSC (the forward layout of the
paper's Section 3.1), and derives the static GCN edge data ("edge weight
determined by the vertex degree", Section 5 / Figure 10) which both sides then
receive as an input array.

Everything is counter based: element k of stream s under seed z is
mix64(z, s, k), so any slice can be produced independently and in parallel.
All integer work is done with torch int64 ops that wrap on overflow, which are
bit-identical on CPU and GPU; float transforms (Box-Muller) may differ in the
last ulp between devices, so one run always hands the *same arrays* to the
oracle and to the HIP path.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Optional

import torch

_MASK64 = (1 << 64) - 1


def _s64(c: int) -> int:
    """Reinterpret an unsigned 64-bit constant as the signed int64 torch holds."""
    c &= _MASK64
    return c - (1 << 64) if c >= (1 << 63) else c


_GOLDEN = _s64(0x9E3779B97F4A7C15)
_M1 = _s64(0xBF58476D1CE4E5B9)
_M2 = _s64(0x94D049BB133111EB)


def _lsr(x: torch.Tensor, k: int) -> torch.Tensor:
    """Logical shift right on int64 (torch's >> is arithmetic)."""
    return (x >> k) & ((1 << (64 - k)) - 1)


def mix64(x: torch.Tensor) -> torch.Tensor:
    """splitmix64 finaliser on an int64 tensor (wrapping arithmetic)."""
    x = (x ^ _lsr(x, 30)) * _M1
    x = (x ^ _lsr(x, 27)) * _M2
    return x ^ _lsr(x, 31)


def _stream_key(seed: int, stream: int) -> int:
    """Scalar key for (seed, stream), computed with Python ints."""
    def mix_py(v: int) -> int:
        v &= _MASK64
        v = ((v ^ (v >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
        v = ((v ^ (v >> 27)) * 0x94D049BB133111EB) & _MASK64
        return v ^ (v >> 31)
    return _s64(mix_py(mix_py(seed * 0x9E3779B97F4A7C15 + 1) ^ (stream * 0xD1B54A32D192ED03 + 7)))


def rand_u64(seed: int, stream: int, start: int, count: int, device="cpu") -> torch.Tensor:
    """int64 tensor of `count` 64-bit hashes for counters start..start+count-1."""
    idx = torch.arange(start, start + count, dtype=torch.int64, device=device)
    return mix64(idx * _GOLDEN + _stream_key(seed, stream))


_CHUNK = 1 << 24  # elements per generation slice (bounds temporaries)


def uniform01(seed: int, stream: int, count: int, device="cpu", dtype=torch.float32) -> torch.Tensor:
    """U(0,1) on the open interval: (k + 0.5) / 2^24 for a 24-bit k."""
    out = torch.empty(count, dtype=dtype, device=device)
    for s in range(0, count, _CHUNK):
        c = min(_CHUNK, count - s)
        k = _lsr(rand_u64(seed, stream, s, c, device), 40)
        out[s:s + c] = ((k.to(torch.float64) + 0.5) * (1.0 / (1 << 24))).to(dtype)
    return out


def normal(seed: int, stream: int, count: int, device="cpu", dtype=torch.float32) -> torch.Tensor:
    """N(0,1) by Box-Muller from two 24-bit uniforms of one 64-bit hash."""
    out = torch.empty(count, dtype=dtype, device=device)
    for s in range(0, count, _CHUNK):
        c = min(_CHUNK, count - s)
        h = rand_u64(seed, stream, s, c, device)
        u1 = (_lsr(h, 40).to(torch.float64) + 0.5) * (1.0 / (1 << 24))
        u2 = ((_lsr(h, 16) & 0xFFFFFF).to(torch.float64) + 0.5) * (1.0 / (1 << 24))
        z = torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2)
        out[s:s + c] = z.to(dtype)
    return out


# ----------------------------------------------------------------------------
# edge generators
# ----------------------------------------------------------------------------

def uniform_edges(n: int, m: int, seed: int, device="cpu"):
    """m directed edges with iid uniform endpoints in [0, n)."""
    src = torch.empty(m, dtype=torch.int64, device=device)
    dst = torch.empty(m, dtype=torch.int64, device=device)
    for s in range(0, m, _CHUNK):
        c = min(_CHUNK, m - s)
        h = rand_u64(seed, 1, s, c, device)
        src[s:s + c] = _lsr(h, 33) % n
        dst[s:s + c] = (h & 0x7FFFFFFF) % n
    return src, dst


def rmat_edges(scale: int, m: int, seed: int, a=0.57, b=0.19, c=0.19, d=0.05, device="cpu"):
    """m R-MAT tuples on 2^scale vertices, no noise, no vertex permutation.

    At each of `scale` levels one quadrant is drawn with probabilities
    (a, b, c, d): a = (src bit 0, dst bit 0), b = (0, 1), c = (1, 0),
    d = (1, 1). Each level consumes 16 bits of a 64-bit hash (4 levels per
    hash), so the probabilities are quantised to 1/65536.
    """
    assert abs(a + b + c + d - 1.0) < 1e-9
    ta = int(round(a * 65536))
    tab = int(round((a + b) * 65536))
    tabc = int(round((a + b + c) * 65536))
    src = torch.empty(m, dtype=torch.int64, device=device)
    dst = torch.empty(m, dtype=torch.int64, device=device)
    chunk = _CHUNK
    for s in range(0, m, chunk):
        cnt = min(chunk, m - s)
        sv = torch.zeros(cnt, dtype=torch.int64, device=device)
        dv = torch.zeros(cnt, dtype=torch.int64, device=device)
        h = None
        for lvl in range(scale):
            if lvl % 4 == 0:
                h = rand_u64(seed, 16 + lvl // 4, s, cnt, device)
            r = _lsr(h, 16 * (lvl % 4)) & 0xFFFF
            sbit = (r >= tab).to(torch.int64)
            dbit = (((r >= ta) & (r < tab)) | (r >= tabc)).to(torch.int64)
            sv = (sv << 1) | sbit
            dv = (dv << 1) | dbit
        src[s:s + cnt] = sv
        dst[s:s + cnt] = dv
    return src, dst


# ----------------------------------------------------------------------------
# COO -> CSC
# ----------------------------------------------------------------------------

@dataclass
class CSC:
    """Destination-major compressed sparse column graph.

    col_ptr[v] .. col_ptr[v+1] delimits the in-edges of destination v;
    row_idx holds their source ids in strictly ascending order.
    """
    n: int
    col_ptr: torch.Tensor  # int64 [n+1]
    row_idx: torch.Tensor  # int32 [nnz]

    @property
    def nnz(self) -> int:
        return int(self.row_idx.numel())

    def in_degree(self) -> torch.Tensor:
        return self.col_ptr[1:] - self.col_ptr[:-1]

    def dst_of_edges(self) -> torch.Tensor:
        """int64 [nnz]: destination id of every stored edge."""
        deg = self.in_degree()
        return torch.repeat_interleave(
            torch.arange(self.n, dtype=torch.int64, device=deg.device), deg)

    def to(self, device) -> "CSC":
        return CSC(self.n, self.col_ptr.to(device), self.row_idx.to(device))


def build_csc(n: int, src: torch.Tensor, dst: torch.Tensor, symmetrise=False, self_loops=False) -> CSC:
    """Sort-unique the edge list by (dst, src) and compress by destination.

    Duplicate tuples collapse to one edge; with self_loops every vertex gets
    exactly one (v, v) edge (generated ones merge with it).
    """
    dev = src.device
    key = dst * n + src
    if symmetrise:
        key = torch.cat([key, src * n + dst])
    if self_loops:
        v = torch.arange(n, dtype=torch.int64, device=dev)
        key = torch.cat([key, v * n + v])
    del src, dst
    key = torch.unique(key, sorted=True)
    d = torch.div(key, n, rounding_mode="floor")
    row_idx = (key - d * n).to(torch.int32)
    del key
    counts = torch.bincount(d, minlength=n)
    del d
    col_ptr = torch.zeros(n + 1, dtype=torch.int64, device=dev)
    torch.cumsum(counts, 0, out=col_ptr[1:])
    return CSC(n, col_ptr, row_idx)


def csc_from_lists(n: int, edges) -> CSC:
    """Tiny helper for hand-written graphs: edges = [(src, dst), ...]."""
    if len(edges) == 0:
        return CSC(n, torch.zeros(n + 1, dtype=torch.int64), torch.zeros(0, dtype=torch.int32))
    e = torch.tensor(edges, dtype=torch.int64)
    return build_csc(n, e[:, 0].contiguous(), e[:, 1].contiguous())


def relabel_csc(g: CSC, new_id: torch.Tensor) -> CSC:
    """The same graph with vertex v renamed new_id[v] (a permutation), columns sorted again."""
    new_id = new_id.to(device=g.col_ptr.device, dtype=torch.int64)
    deg = g.col_ptr[1:] - g.col_ptr[:-1]
    dst = torch.repeat_interleave(torch.arange(g.n, device=g.col_ptr.device), deg)
    return build_csc(g.n, new_id[g.row_idx.long()], new_id[dst])


def gcn_edge_weights(g: CSC) -> torch.Tensor:
    """Static GCN edge data w_e = 1/sqrt(d_src * d_dst), d = in-degree in g.

    Computed in fp64 and rounded once to fp32. Vertices that appear as a source
    with in-degree 0 (possible only without self-loops) use d = 1.
    """
    deg = g.in_degree().clamp(min=1).to(torch.float64)
    dv = g.dst_of_edges()
    w = 1.0 / torch.sqrt(deg[g.row_idx.long()] * deg[dv])
    return w.to(torch.float32)


# ----------------------------------------------------------------------------
# tensors
# ----------------------------------------------------------------------------

def normal_features(n: int, f: int, seed: int, device="cpu") -> torch.Tensor:
    return normal(seed, 2, n * f, device).view(n, f)


def sparse_uniform_features(n: int, f: int, seed: int, density=0.1, device="cpu") -> torch.Tensor:
    """Dense-stored matrix whose entries are nonzero w.p. `density`, value U(0,1)."""
    val = uniform01(seed, 3, n * f, device)
    keep = uniform01(seed, 4, n * f, device) < density
    return (val * keep).view(n, f)


def glorot_uniform(rows: int, cols: int, seed: int, device="cpu") -> torch.Tensor:
    """U(-L, L), L = sqrt(6 / (rows + cols)), shape rows x cols."""
    lim = math.sqrt(6.0 / (rows + cols))
    u = uniform01(seed, 5, rows * cols, device, torch.float64)
    return ((2.0 * u - 1.0) * lim).to(torch.float32).view(rows, cols)


def uniform_pm(count: int, lim: float, seed: int, device="cpu") -> torch.Tensor:
    u = uniform01(seed, 6, count, device, torch.float64)
    return ((2.0 * u - 1.0) * lim).to(torch.float32)


def round_to_bf16(x: torch.Tensor) -> torch.Tensor:
    """fp32 tensor -> fp32 tensor holding the nearest-even bf16 values."""
    return x.to(torch.bfloat16).to(torch.float32)


def bf16_bits(x: torch.Tensor) -> torch.Tensor:
    """fp32 tensor of bf16-representable values -> int16 tensor of their bits."""
    return x.to(torch.bfloat16).view(torch.int16)


def bernoulli_graph(n: int, density: float, seed: int, device="cpu") -> CSC:
    """n x n adjacency in which every cell (dst, src) is an edge independently with
    probability `density` (the uniformly sparse matrices of the paper's Section 6.1)."""
    thr = int(density * (1 << 53))
    keys = []
    cells = n * n
    for s in range(0, cells, _CHUNK):
        c = min(_CHUNK, cells - s)
        h = _lsr(rand_u64(seed, 7, s, c, device), 11)           # 53 uniform bits
        idx = torch.nonzero(h < thr).flatten() + s                # cell index = dst * n + src
        keys.append(idx)
    key = torch.cat(keys) if keys else torch.zeros(0, dtype=torch.int64, device=device)
    d = torch.div(key, n, rounding_mode="floor")
    row_idx = (key - d * n).to(torch.int32)
    col_ptr = torch.zeros(n + 1, dtype=torch.int64, device=device)
    torch.cumsum(torch.bincount(d, minlength=n), 0, out=col_ptr[1:])
    return CSC(n, col_ptr, row_idx)


# ----------------------------------------------------------------------------
# the five workloads
# ----------------------------------------------------------------------------

@dataclass
class Workload:
    name: str
    graph: CSC
    X: torch.Tensor                       # fp32 [n, f_in] (bf16-valued when dtype == "bf16")
    edge_op: str                          # "copy" | "mul_weight" | "gated"
    edge_weight: Optional[torch.Tensor]   # fp32 [nnz]
    W: torch.Tensor                       # fp32 [f_in, f_out]
    act: str                              # "relu" | "none"
    dtype: str                            # "f32" | "bf16"
    W_gate: Optional[torch.Tensor] = None  # fp32 [f, 2f]
    b_gate: Optional[torch.Tensor] = None  # fp32 [f]
    W_msg: Optional[torch.Tensor] = None   # fp32 [f, f]
    W_pool: Optional[torch.Tensor] = None  # fp32 [f_pool, f]   (edge_op "pool")
    b_pool: Optional[torch.Tensor] = None  # fp32 [f_pool]
    W_self: Optional[torch.Tensor] = None  # fp32 [f, f_out]    (CommNet's W_H)
    extra: dict = field(default_factory=dict)


def workload(k: int, device="cpu", scale: Optional[int] = None, edge_factor: Optional[int] = None,
             f_in: Optional[int] = None, f_out: Optional[int] = None) -> Workload:
    """Build configuration k in 1..5; the optional arguments shrink it for tests.

    1: uniform graph, 4,096 vertices, 32,768 tuples, self-loops; 64 -> 64 fp32 GCN.
    2: R-MAT scale 17, edge factor 16, symmetrised, self-loops; 500 -> 16 (-> 3) fp32 GCN,
       X ~ U(0,1) at 10 % density (pubmed-shaped bag-of-words, Table 1).
    3: R-MAT scale 18, edge factor 400, symmetrised, self-loops; 512 -> 256 bf16 GCN.
    4: R-MAT scale 20, edge factor 32, directed, no self-loops; 128-wide gated layer.
    5: R-MAT scale 23, edge factor 64, directed, self-loops; 256 -> 256 fp32 GCN
       (sum and max), meant to be streamed from host memory.
    """
    gseed, fseed, wseed = 1000 + k, 2000 + k, 3000 + k
    if k == 1:
        n = 1 << (scale if scale is not None else 12)
        m = n * (edge_factor if edge_factor is not None else 8)
        fi, fo = f_in or 64, f_out or 64
        s, d = uniform_edges(n, m, gseed, device)
        g = build_csc(n, s, d, symmetrise=False, self_loops=True)
        X = normal_features(n, fi, fseed, device)
        return Workload("config1_uniform_gcn_f32", g, X, "mul_weight", gcn_edge_weights(g),
                        glorot_uniform(fi, fo, wseed, device), "relu", "f32")
    defaults = {2: (17, 16, 500, 16), 3: (18, 400, 512, 256), 4: (20, 32, 128, 128), 5: (23, 64, 256, 256)}
    sc, ef, fi, fo = defaults[k]
    sc = scale if scale is not None else sc
    ef = edge_factor if edge_factor is not None else ef
    fi = f_in or fi
    fo = f_out or fo
    n = 1 << sc
    s, d = rmat_edges(sc, n * ef, gseed, device=device)
    if k == 2:
        g = build_csc(n, s, d, symmetrise=True, self_loops=True)
        X = sparse_uniform_features(n, fi, fseed, 0.1, device)
        wl = Workload("config2_rmat17_gcn_f32", g, X, "mul_weight", gcn_edge_weights(g),
                      glorot_uniform(fi, fo, wseed, device), "relu", "f32")
        wl.extra["W2"] = glorot_uniform(fo, 3, wseed + 100, device)
        return wl
    if k == 3:
        g = build_csc(n, s, d, symmetrise=True, self_loops=True)
        X = round_to_bf16(normal_features(n, fi, fseed, device))
        W = round_to_bf16(glorot_uniform(fi, fo, wseed, device))
        return Workload("config3_rmat18_gcn_bf16", g, X, "mul_weight", gcn_edge_weights(g), W, "relu", "bf16")
    if k == 4:
        g = build_csc(n, s, d, symmetrise=False, self_loops=False)
        X = normal_features(n, fi, fseed, device)
        wl = Workload("config4_rmat20_gated_f32", g, X, "gated", None,
                      glorot_uniform(fi, fo, wseed, device), "relu", "f32")
        wl.W_gate = glorot_uniform(fi, 2 * fi, wseed + 1, device)
        wl.b_gate = uniform_pm(fi, 0.1, wseed + 2, device)
        wl.W_msg = glorot_uniform(fi, fi, wseed + 3, device)
        return wl
    if k == 5:
        g = build_csc(n, s, d, symmetrise=False, self_loops=True)
        X = normal_features(n, fi, fseed, device)
        return Workload("config5_rmat23_gcn_f32_streamed", g, X, "mul_weight", gcn_edge_weights(g),
                        glorot_uniform(fi, fo, wseed, device), "relu", "f32")
    raise ValueError(f"no configuration {k}")


def commnet_workload(scale=12, edge_factor=16, f_in=64, f_out=64, device="cpu") -> Workload:
    """CommNet layer (Figure 9) on a symmetrised R-MAT graph: pass-through ApplyEdge, sum Gather,
    ApplyVertex ReLU(W_H (x) vertex + W_C (x) accum)."""
    n = 1 << scale
    s, d = rmat_edges(scale, n * edge_factor, 4100 + scale, device=device)
    g = build_csc(n, s, d, symmetrise=True, self_loops=False)
    wl = Workload(f"commnet_rmat{scale}", g, normal_features(n, f_in, 4200, device), "copy", None,
                  glorot_uniform(f_in, f_out, 4300, device), "relu", "f32")
    wl.W_self = glorot_uniform(f_in, f_out, 4301, device)
    return wl


def mpgcn_workload(scale=12, edge_factor=16, f_in=64, f_pool=32, f_out=16, device="cpu") -> Workload:
    """Max-pooling GCN layer (Figure 11) on a directed R-MAT graph: ApplyEdge sigmoid(W_pool (x) src + b),
    max Gather, ApplyVertex ReLU(W (x) accum)."""
    n = 1 << scale
    s, d = rmat_edges(scale, n * edge_factor, 4500 + scale, device=device)
    g = build_csc(n, s, d, symmetrise=False, self_loops=False)
    wl = Workload(f"mpgcn_rmat{scale}", g, normal_features(n, f_in, 4600, device), "pool", None,
                  glorot_uniform(f_pool, f_out, 4700, device), "relu", "f32")
    wl.W_pool = glorot_uniform(f_pool, f_in, 4701, device)
    wl.b_pool = uniform_pm(f_pool, 0.5, 4702, device)
    return wl


def spmm_workload(density: float, n: int = 10000, f: int = 128, device="cpu") -> Workload:
    """Sparse-dense product of Section 6.1's micro-benchmark: an n x n sparse matrix of the
    given density (values N(0,1)) times an n x f dense matrix, expressed as a layer whose
    ApplyEdge multiplies by the edge value, Gather sums, and there is no ApplyVertex."""
    seed = 7000 + int(round(density * 1e6))
    g = bernoulli_graph(n, density, seed, device)
    X = normal_features(n, f, seed + 1, device)
    w = normal(seed + 2, 8, g.nnz, device)
    return Workload(f"spmm_{n}x{n}_d{density:g}_x{f}", g, X, "mul_weight", w, torch.zeros(f, 0), "none", "f32")

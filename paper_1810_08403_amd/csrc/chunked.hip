// Streamed layer: graphs whose vertex data live in host memory are processed
// as vertex intervals x edge chunks through a fixed device budget (Section 3.1).
//
// The adjacency matrix is tiled into chunks C_ij (sources in interval V_i,
// destinations in interval V_j), each a destination-major CSC with local ids.
// Schedule (Section 3.1, the paper's own): for every destination interval j
// the accumulator A_j stays on the device while the source intervals V_i and
// their chunks C_ij stream through; fused Scatter-ApplyEdge-Gather adds each
// chunk into A_j; ApplyVertex consumes A_j while it is still resident; then
// the next j. Copies run on their own streams, double buffered, so that the
// transfer of chunk i+1 overlaps the kernels of chunk i, and the transfer of
// the output overlaps the next ApplyVertex tile.
//
// Differences from the paper: the grid may be rectangular (Q destination
// intervals x P source intervals, Q <= P): every destination interval re-reads
// all of X over the host link, so the planner takes the fewest destination
// intervals whose accumulator fits the budget and keeps the streamed source
// intervals small. Columns without edges in a chunk are left out of its work
// list. The static edge data travel with the chunk.
//
// The same schedule serves the other layer programs and the backward pass through
// two hooks: a vertex feed that produces a source interval's rows instead of copying
// them (the streamed backward pass forms dZ there), and extras for layers that need
// more than one kind of row (gated: rows [Ps | M] travel, the destination parts Pd
// of the resident interval sit beside its accumulator; W_self: the interval's own
// rows are copied in, or produced by a callback, for ApplyVertex; the backward pass
// of a max Gather: another edge function over rows [x | m], and a callback that works
// on an interval's sums before ApplyVertex). The device buffers belong to the context, so
// that the grid of a graph and the grid of its transposed twin share one budget.
#include <algorithm>
#include <atomic>
#include <chrono>
#include <cstring>
#include <thread>

#include "saga_internal.h"

struct ChunkMeta {
    int64_t nnz = 0, n_items = 0, n_team = 0, n_heavy = 0, n_slots = 0;
    size_t off_items = 0, off_heavy = 0, off_ridx = 0, off_w = 0, bytes = 0;
    char* host = nullptr;  // inside the tiling's pinned arena: [items | heavy | row_idx | weights]
};

struct ChunkGrid {
    int Q = 0, P = 0;
    int64_t Dq = 0, Sp = 0;  // rows per destination / source interval
    WorkListParams wlp{-1, -1, -1, true, 1};
    bool weighted = false;
    std::vector<ChunkMeta> chunks;  // [j * P + i]
    size_t max_chunk_bytes = 0;
    int64_t max_slots = 0;
    char* arena = nullptr;    // one pinned allocation that holds every chunk's payload
    size_t arena_bytes = 0;
    // device side: the buffers, streams and events belong to the context (one streamed call runs at a time, and the
    // forward grid of a graph and the grid of its transposed twin must share one budget)
    float* a_host = nullptr;  // pinned home of the accumulators for the swapping baselines
    size_t a_host_bytes = 0;
};

void chunk_grid_destroy(saga_ctx* ctx, ChunkGrid* g)
{
    if (!g) return;
    (void)ctx;
    if (g->arena) (void)hipHostFree(g->arena);
    if (g->a_host) (void)hipHostFree(g->a_host);
    delete g;
}

saga_status saga_ctx::ensure_stream_set()
{
    if (st.ready) return SAGA_OK;
    if (!st.s_in) HIP_TRY(this, hipStreamCreateWithFlags(&st.s_in, hipStreamNonBlocking));
    if (!st.s_out) HIP_TRY(this, hipStreamCreateWithFlags(&st.s_out, hipStreamNonBlocking));
    for (hipEvent_t* e : {&st.ev_ready[0], &st.ev_ready[1], &st.ev_free[0], &st.ev_free[1], &st.ev_y_ready[0], &st.ev_y_ready[1],
                          &st.ev_y_free[0], &st.ev_y_free[1], &st.ev_a_done, &st.ev_a_ready, &st.ev_a_in, &st.ev_d_free, &st.ev_s_ready[0],
                          &st.ev_s_ready[1]})
        if (!*e) HIP_TRY(this, hipEventCreateWithFlags(e, hipEventDisableTiming));
    st.ready = true;
    return SAGA_OK;
}

void saga_ctx::destroy_stream_set()
{
    for (hipEvent_t* e : {&st.ev_ready[0], &st.ev_ready[1], &st.ev_free[0], &st.ev_free[1], &st.ev_y_ready[0], &st.ev_y_ready[1],
                          &st.ev_y_free[0], &st.ev_y_free[1], &st.ev_a_done, &st.ev_a_ready, &st.ev_a_in, &st.ev_d_free, &st.ev_s_ready[0],
                          &st.ev_s_ready[1]}) {
        if (*e) (void)hipEventDestroy(*e);
        *e = nullptr;
    }
    if (st.s_in) (void)hipStreamDestroy(st.s_in);
    if (st.s_out) (void)hipStreamDestroy(st.s_out);
    st.s_in = st.s_out = nullptr;
    st.ready = false;
}

// After a streamed call that failed half-way: nothing it enqueued may still be reading or writing the caller's host
// tensors when the error is returned. Errors of the waits themselves are ignored (the call has failed already).
void chunk_grid_drain(saga_ctx* ctx)
{
    if (ctx->st.s_in) (void)hipStreamSynchronize(ctx->st.s_in);
    if (ctx->stream) (void)hipStreamSynchronize(ctx->stream);
    if (ctx->st.s_out) (void)hipStreamSynchronize(ctx->st.s_out);
}

namespace {

size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct BuiltChunk {
    std::vector<WorkItem> items;
    std::vector<HeavyVertex> heavy;
    std::vector<int32_t> ridx;
    std::vector<float> w;
    int64_t n_slots = 0, n_team = 0;
};

// Where chunk C_ij's edges sit in the host CSC: columns [j*Dq, ...), sources in [i*Sp, (i+1)*Sp). For local column c,
// lo[c] is the first such edge of the column and lcp[c + 1] - lcp[c] their number (they are consecutive: a column is
// ascending in source id).
void locate_chunk(const saga_graph* g, int64_t Dq, int64_t Sp, int i, int j, std::vector<int64_t>* lcp, std::vector<int64_t>* lo)
{
    const int64_t v0 = (int64_t)j * Dq, v1 = std::min(g->n, v0 + Dq);
    const int64_t s0 = (int64_t)i * Sp, s1 = std::min(g->n, s0 + Sp);
    const int64_t* cp = g->h_col_ptr.data();
    const int32_t* ri = g->h_row_idx.data();
    lcp->assign((size_t)(v1 - v0) + 1, 0);
    lo->assign((size_t)(v1 - v0), 0);
    for (int64_t v = v0; v < v1; ++v) {
        const int32_t* b = ri + cp[v];
        const int32_t* e = ri + cp[v + 1];
        const int32_t* l = std::lower_bound(b, e, (int32_t)s0);
        const int32_t* h = std::lower_bound(l, e, (int32_t)std::min<int64_t>(s1, 0x7fffffff));
        (*lo)[v - v0] = l - ri;
        (*lcp)[v - v0 + 1] = (*lcp)[v - v0] + (h - l);
    }
}

// The chunk's edge data in chunk order, from the graph's edge data.
void fill_chunk_weights(const saga_graph* g, const std::vector<int64_t>& lcp, const std::vector<int64_t>& lo, float* out)
{
    for (size_t c = 0; c + 1 < lcp.size(); ++c) {
        const int64_t cnt = lcp[c + 1] - lcp[c];
        if (cnt > 0) memcpy(out + lcp[c], g->h_edge_data.data() + lo[c], sizeof(float) * (size_t)cnt);
    }
}

// Chunk C_ij of the host CSC, local ids, with its work list.
void build_chunk(const saga_graph* g, int64_t Dq, int64_t Sp, int i, int j, const WorkListParams& wlp, bool weighted,
                 BuiltChunk* out)
{
    const int64_t v0 = (int64_t)j * Dq, v1 = std::min(g->n, v0 + Dq);
    const int64_t s0 = (int64_t)i * Sp;
    const int32_t* ri = g->h_row_idx.data();
    std::vector<int64_t> lcp, lo;
    locate_chunk(g, Dq, Sp, i, j, &lcp, &lo);
    const int64_t nnz = lcp.back();
    out->ridx.resize((size_t)nnz);
    if (weighted) out->w.resize((size_t)nnz);
    for (int64_t v = v0; v < v1; ++v) {
        const int64_t cnt = lcp[v - v0 + 1] - lcp[v - v0];
        const int64_t src = lo[v - v0], dst = lcp[v - v0];
        for (int64_t k = 0; k < cnt; ++k) out->ridx[dst + k] = (int32_t)(ri[src + k] - s0);
    }
    if (weighted && nnz > 0) fill_chunk_weights(g, lcp, lo, out->w.data());
    WorkList wl;
    build_work_list(lcp.data(), out->ridx.data(), v1 - v0, wlp, &wl);
    out->items.swap(wl.items);
    out->heavy.swap(wl.heavy);
    out->n_slots = wl.n_slots;
    out->n_team = wl.n_team;
}

// The Q x P tiling of a host graph, built aside and handed to the graph only when it is complete: a failure on the
// way (host memory, pinned memory) leaves the graph without a tiling, never with half of one.
saga_status build_grid(saga_ctx* ctx, saga_graph* g, int Q, int P, const WorkListParams& wlp, bool weighted)
{
    if (g->grid) {
        chunk_grid_destroy(ctx, g->grid);
        g->grid = nullptr;
    }
    ChunkGrid* grid = new (std::nothrow) ChunkGrid();
    if (!grid) return ctx->fail(SAGA_ERR_INTERNAL, "out of host memory");
    auto bail = [&](saga_status st) {
        chunk_grid_destroy(ctx, grid);
        return st;
    };
    grid->Q = Q;
    grid->P = P;
    grid->Dq = (g->n + Q - 1) / Q;
    grid->Sp = (g->n + P - 1) / P;
    grid->wlp = wlp;
    grid->weighted = weighted;
    std::vector<BuiltChunk> built;
    try {
        grid->chunks.resize((size_t)Q * P);
        built.resize((size_t)Q * P);
    } catch (...) {
        return bail(ctx->fail(SAGA_ERR_INTERNAL, "out of host memory while tiling the graph"));
    }
    std::atomic<bool> oom{false};
    parallel_for((int64_t)Q * P, 16, [&](int64_t c) {
        try {
            build_chunk(g, grid->Dq, grid->Sp, (int)(c % P), (int)(c / P), wlp, weighted, &built[(size_t)c]);
        } catch (...) {
            oom = true;
        }
    });
    if (oom) return bail(ctx->fail(SAGA_ERR_INTERNAL, "out of host memory while tiling the graph"));
    size_t total = 0;
    for (size_t c = 0; c < built.size(); ++c) {
        ChunkMeta& m = grid->chunks[c];
        const BuiltChunk& b = built[c];
        m.nnz = (int64_t)b.ridx.size();
        m.n_items = (int64_t)b.items.size();
        m.n_heavy = (int64_t)b.heavy.size();
        m.n_slots = b.n_slots;
        m.n_team = b.n_team;
        size_t off = 0;
        m.off_items = off;
        off = round_up(off + sizeof(WorkItem) * b.items.size(), 256);
        m.off_heavy = off;
        off = round_up(off + sizeof(HeavyVertex) * b.heavy.size(), 256);
        m.off_ridx = off;
        off = round_up(off + sizeof(int32_t) * b.ridx.size(), 256);
        m.off_w = off;
        off = round_up(off + sizeof(float) * b.w.size(), 256);
        m.bytes = off;
        grid->max_chunk_bytes = std::max(grid->max_chunk_bytes, m.bytes);
        grid->max_slots = std::max(grid->max_slots, m.n_slots);
        if (m.nnz > 0) total += m.bytes;
    }
    if (total > 0) {
        hipError_t e = hipHostMalloc(reinterpret_cast<void**>(&grid->arena), total, hipHostMallocDefault);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            grid->arena = nullptr;
            return bail(ctx->fail(SAGA_ERR_HIP, "hipHostMalloc(%zu) for the tiling's payloads failed: %s", total, hipGetErrorString(e)));
        }
        grid->arena_bytes = total;
        size_t at = 0;
        for (ChunkMeta& m : grid->chunks)
            if (m.nnz > 0) {
                m.host = grid->arena + at;
                at += m.bytes;
            }
    }
    parallel_for((int64_t)built.size(), 8, [&](int64_t c) {
        ChunkMeta& m = grid->chunks[(size_t)c];
        BuiltChunk& b = built[(size_t)c];
        if (!m.host) return;
        // (an empty vector's data() may be null, which memcpy must not be given even for zero bytes)
        if (!b.items.empty()) memcpy(m.host + m.off_items, b.items.data(), sizeof(WorkItem) * b.items.size());
        if (!b.heavy.empty()) memcpy(m.host + m.off_heavy, b.heavy.data(), sizeof(HeavyVertex) * b.heavy.size());
        if (!b.ridx.empty()) memcpy(m.host + m.off_ridx, b.ridx.data(), sizeof(int32_t) * b.ridx.size());
        if (!b.w.empty()) memcpy(m.host + m.off_w, b.w.data(), sizeof(float) * b.w.size());
        BuiltChunk().items.swap(b.items);
        std::vector<int32_t>().swap(b.ridx);
        std::vector<float>().swap(b.w);
    });
    g->grid = grid;
    return SAGA_OK;
}

// Edge counts of a Q x P tiling with equal intervals, from one pass over the columns.
void count_grid(const saga_graph* g, int Q, int P, std::vector<int64_t>* nnz, std::vector<int64_t>* pairs)
{
    const int64_t Dq = (g->n + Q - 1) / Q, Sp = (g->n + P - 1) / P;
    nnz->assign((size_t)Q * P, 0);
    pairs->assign((size_t)Q * P, 0);
    const int64_t* cp = g->h_col_ptr.data();
    const int32_t* ri = g->h_row_idx.data();
    const int nt = 16;
    std::vector<std::vector<int64_t>> part((size_t)nt, std::vector<int64_t>((size_t)Q * P * 2, 0));
    parallel_for(nt, nt, [&](int64_t t) {
        std::vector<int64_t>& acc = part[(size_t)t];
        const int64_t a = g->n * t / nt, b = g->n * (t + 1) / nt;
        for (int64_t v = a; v < b; ++v) {
            const int64_t j = v / Dq;
            int64_t prev = -1;
            for (int64_t e = cp[v]; e < cp[v + 1]; ++e) {
                const int64_t i = ri[e] / Sp;
                acc[(size_t)(j * P + i) * 2] += 1;
                if (i != prev) acc[(size_t)(j * P + i) * 2 + 1] += 1;
                prev = i;
            }
        }
    });
    for (int t = 0; t < nt; ++t)
        for (size_t c = 0; c < (size_t)Q * P; ++c) {
            (*nnz)[c] += part[(size_t)t][c * 2];
            (*pairs)[c] += part[(size_t)t][c * 2 + 1];
        }
}

struct Plan {
    int Q, P;
    int64_t y_tile_rows;
    size_t bytes;
};

// Upper bounds on the largest chunk payload and the most partial rows of a tiling, from its edge counts.
void chunk_bounds(const std::vector<int64_t>& nnz, const std::vector<int64_t>& pairs, bool weighted, int64_t min_edges, size_t* max_chunk,
                  size_t* max_slots)
{
    *max_chunk = *max_slots = 0;
    for (size_t c = 0; c < nnz.size(); ++c) {
        const size_t pieces = (size_t)(pairs[c] + nnz[c] / std::max<int64_t>(min_edges, 1));
        const size_t b = 16 * pieces + 16 * (pieces / 2 + 1) + (weighted ? 8 : 4) * (size_t)nnz[c] + 4 * 256;
        *max_chunk = std::max(*max_chunk, b);
        *max_slots = std::max(*max_slots, (size_t)(nnz[c] / std::max<int64_t>(min_edges, 1)) + 1);
    }
}

// Device bytes a Q x P plan needs, given its largest chunk payload and its most partial rows.
size_t plan_bytes(const saga_graph* g, int Q, int P, int64_t F, int64_t Fa, int64_t F_out, bool has_w, int64_t y_tile_rows, size_t max_chunk,
                  size_t max_slots, int64_t Fd, int64_t F_self)
{
    const int64_t Dq = (g->n + Q - 1) / Q, Sp = (g->n + P - 1) / P;
    size_t total = (size_t)Dq * Fa * 4;                // A_j
    total += (size_t)Dq * Fd * 4;                      // constant rows of the interval's destinations (gated)
    total += 2 * (size_t)Sp * F * 4;                   // V_i, double buffered
    total += 2 * max_chunk;                            // C_ij, double buffered
    total += max_slots * (size_t)Fa * 4;               // partial rows of cut columns
    if (has_w) total += 2 * (size_t)y_tile_rows * (F_out + F_self) * 4 + (size_t)(F_out + 128) * (Fa + F_self + 128) * 4;  // Y tiles (+ own rows) + packed W
    return total + (1 << 20);
}

}  // namespace

saga_status streamed_forward(saga_ctx* ctx, saga_graph* g, const saga_tensor* X, const saga_edge_params* ep, int32_t agg,
                             const saga_vertex_params* vp, saga_tensor* Y, const VertexFeed* feed, const StreamExtras* extras)
{
    const auto t_begin = std::chrono::steady_clock::now();
    const int64_t n = g->n;
    const int64_t F = X->cols;                                            // width of the rows that travel over the edges
    const int64_t Fa = extras && extras->acc_width ? extras->acc_width : F;  // width of the accumulator rows
    const int32_t op = extras && extras->op ? extras->op : (int32_t)ep->op;
    const bool gated = ep->op == SAGA_EDGE_GATED || (extras && extras->op);  // rows [x | m] travel, constant rows are resident
    const bool has_w = vp && vp->W;
    const bool has_self = has_w && extras && (extras->self_rows || extras->self_fill);
    const int64_t F_self = has_self ? extras->F_self : 0;
    const bool weighted = ep->op == SAGA_EDGE_MUL_WEIGHT;
    const int64_t n_out = extras && extras->n_out == 2 ? 2 : 1;            // accumulator rows are n_out * Fa wide
    const int64_t Fd = extras && extras->dst_width ? extras->dst_width : Fa;  // width of the resident constant rows
    const int64_t Fw = Fa * n_out;
    const int64_t F_out = has_w ? vp->W->cols : Fw;
    if (n == 0) return SAGA_OK;
    if (n_out == 2 && (!extras->op || Fd != 2 * Fa)) return ctx->fail(SAGA_ERR_INTERNAL, "two outputs need a two-row edge function");
    // rows [x | m] travel, or [x | m | t] for the out-edge gradient under the max accumulator (t: the maximum gathered at the
    // edge's far end)
    const bool third_row = op == kGatherOpGateBothMax;
    if (gated && (!extras || (!extras->dst_rows && !extras->dst_fill) || F != (third_row ? 3 : 2) * Fa))
        return ctx->fail(SAGA_ERR_INTERNAL, "streamed gated call without its hoisted rows");
    if (op == kGatherOpGateGradMax && Fd != 3 * Fa) return ctx->fail(SAGA_ERR_INTERNAL, "the in-edge gradient under max needs three constant rows");

    WorkListParams wlp = work_list_params(ctx, F * 4);
    wlp.skip_empty = true;

    // ---- plan: fewest destination intervals, then the fewest source intervals, that fit the budget ----
    int Q = ctx->opt_dst_intervals, P = ctx->opt_src_intervals;
    int64_t y_tile_rows = 0;
    auto tile_rows_for = [&](int q) {
        const int64_t Dq = (n + q - 1) / q;
        return std::min<int64_t>(Dq, std::max<int64_t>(4096, (64 << 20) / (F_out * 4)));  // about 64 MiB per tile
    };
    const bool same_grid = g->grid && g->grid->wlp.min_edges == wlp.min_edges && g->grid->wlp.cut_degree == wlp.cut_degree &&
                           g->grid->wlp.stripe_rows == wlp.stripe_rows && g->grid->wlp.team == wlp.team &&
                           g->grid->weighted == weighted;
    // what the context holds apart from the schedule's own buffers (packed weights, other graphs) counts too
    size_t held = ctx->cur_bytes;
    for (const DevBuf* b : {&ctx->st_A, &ctx->st_V[0], &ctx->st_V[1], &ctx->st_C[0], &ctx->st_C[1], &ctx->st_Y[0], &ctx->st_Y[1],
                            &ctx->st_partials, &ctx->st_D, &ctx->st_S[0], &ctx->st_S[1]})
        held -= std::min(held, b->bytes);
    std::vector<int64_t> nnz, pairs;
    auto need_of = [&](int q, int p, size_t max_chunk, size_t max_slots) {
        return plan_bytes(g, q, p, F, Fw, F_out, has_w, tile_rows_for(q), max_chunk, max_slots, gated ? Fd : 0, F_self) +
               (feed ? feed->bytes_per_row * (size_t)((n + p - 1) / p) : 0) +
               (extras ? extras->bytes_per_dst_row * (size_t)((n + q - 1) / q) : 0);
    };
    auto need_for = [&](int q, int p) {  // a tiling that does not exist yet: one pass over the edges for its counts
        size_t max_chunk, max_slots;
        count_grid(g, q, p, &nnz, &pairs);
        chunk_bounds(nnz, pairs, weighted, wlp.min_edges, &max_chunk, &max_slots);
        return need_of(q, p, max_chunk, max_slots);
    };
    // the grid of an earlier call is kept if it was made for the same tunables and, under a budget, this call fits
    // it too (a backward pass holds more per vertex than the forward pass whose grid it finds)
    // k intervals of ceil(n / k) rows leave the last ones empty when n is small against k * k (7 vertices in 5 intervals
    // of 2): a grid only ever has the intervals that hold vertices
    auto whole = [&](int k) {
        const int64_t rows = (n + k - 1) / k;
        return (int)((n + rows - 1) / rows);
    };
    if (Q > 0 && Q <= n) Q = whole(Q);
    if (P > 0 && P <= n) P = whole(P);
    bool reuse = same_grid && (Q == 0 || Q == g->grid->Q) && (P == 0 || P == g->grid->P);
    if (reuse && ctx->budget > 0 && (Q == 0 || P == 0) &&
        need_of(g->grid->Q, g->grid->P, g->grid->max_chunk_bytes, (size_t)g->grid->max_slots) + held > ctx->budget)
        reuse = false;  // (the existing tiling's payload sizes are known exactly: no pass over the edges on this path)
    if (reuse) {
        Q = g->grid->Q;
        P = g->grid->P;
    } else if (Q > 0 && P > 0) {
        if (Q > n || P > n) return ctx->fail(SAGA_ERR_INVALID_ARG, "more intervals than vertices");
    } else {
        int best_q = 0, best_p = 0;
        // For every number of destination intervals, the fewest source intervals that fit. Every destination interval
        // re-reads all vertex data over the link, so fewer of them is better, unless what is left of the budget then
        // only fits slivers of source intervals: each (destination, source) step costs a fixed time on top of its
        // bytes (taken as the time of 2 MiB on the link), so a plan with a few more destination intervals and far
        // fewer steps can be cheaper. The search goes on past the first fit while that fit is this fine-grained.
        bool found = false;
        double best_cost = 0.0;
        int further = 0;
        const int qs[] = {1, 2, 3, 4, 6, 8, 12, 16, 24, 32, 48, 64, 96, 128, 256, 512, 1024};
        const int ps[] = {1, 2, 4, 8, 16, 32, 64, 128, 256, 512, 1024, 2048, 4096};
        for (int q : qs) {
            if ((Q > 0 && whole(q) != Q) || q > n) continue;
            int fit_p = 0;
            for (int p : ps) {
                if ((P > 0 && whole(p) != P) || p > n || p < q) continue;
                // without a cap, stop growing P once a source interval is below 1 GiB
                const size_t need = need_for(q, p);
                const bool small_enough = (size_t)((n + p - 1) / p) * F * 4 <= ((size_t)1 << 30);
                if ((ctx->budget == 0 && small_enough) || (ctx->budget > 0 && need + held <= ctx->budget)) {
                    fit_p = p;
                    break;
                }
            }
            if (!fit_p) continue;
            const double cost = (double)q * (double)n * F * 4 + (double)q * fit_p * (double)(2 << 20);
            if (!found || cost < best_cost) {
                found = true;
                best_cost = cost;
                best_q = q;
                best_p = fit_p;
            }
            if (fit_p <= 32 || ++further > 3) break;
        }
        if (!found)
            return ctx->fail(SAGA_ERR_BUDGET, "no vertex-interval x edge-chunk plan fits %zu bytes of device memory", ctx->budget);
        Q = whole(best_q);
        P = whole(best_p);
    }
    y_tile_rows = tile_rows_for(Q);
    if (!(same_grid && g->grid->Q == Q && g->grid->P == P))
        if (saga_status st = build_grid(ctx, g, Q, P, wlp, weighted)) return st;
    ChunkGrid* grid = g->grid;
    const int64_t Dq = grid->Dq, Sp = grid->Sp;
    if (saga_status sst = ctx->ensure_stream_set()) return sst;
    saga_ctx::StreamSet& ss = ctx->st;

    // ---- device buffers, all counted against the budget ----
    saga_status st;
    {
        constexpr int NB = 11;
        DevBuf* bufs[NB] = {&ctx->st_A, &ctx->st_V[0], &ctx->st_V[1], &ctx->st_C[0], &ctx->st_C[1], &ctx->st_Y[0], &ctx->st_Y[1],
                            &ctx->st_partials, &ctx->st_D, &ctx->st_S[0], &ctx->st_S[1]};
        const size_t c_bytes = std::max<size_t>(grid->max_chunk_bytes, 256);
        const size_t y_bytes = has_w ? (size_t)y_tile_rows * F_out * 4 : 0;
        const size_t s_bytes = has_self ? (size_t)y_tile_rows * F_self * 4 : 0;
        const size_t want[NB] = {(size_t)Dq * Fw * 4, (size_t)Sp * F * 4, (size_t)Sp * F * 4, c_bytes, c_bytes, y_bytes, y_bytes,
                                 grid->max_slots > 0 ? (size_t)grid->max_slots * Fw * 4 : 0, gated ? (size_t)Dq * Fd * 4 : 0, s_bytes, s_bytes};
        // under a budget a buffer left by another plan must not be larger than this plan counted either
        bool fits = true;
        for (int b = 0; b < NB; ++b)
            fits = fits && bufs[b]->bytes >= want[b] && (ctx->budget == 0 || bufs[b]->bytes <= round_up(want[b], 256));
        if (!fits) {
            // another plan left its buffers: start from nothing, so that this plan's own sizes are what counts against the budget
            for (DevBuf* b : bufs) ctx->dev_free(b);
            for (int b = 0; b < NB; ++b)
                if (want[b] > 0 && (st = ctx->dev_alloc(bufs[b], want[b]))) return st;
        }
    }
    if (ctx->budget > 0 && ctx->cur_bytes > ctx->budget)
        return ctx->fail(SAGA_ERR_BUDGET, "plan %d x %d needs %zu bytes of device memory, budget is %zu", Q, P, ctx->cur_bytes,
                         ctx->budget);

    // "overlap" 0 puts every copy on the compute stream: nothing overlaps (the streaming-off baseline)
    hipStream_t sc = ctx->stream;
    hipStream_t sin = ctx->opt_overlap ? ss.s_in : sc, sout = ctx->opt_overlap ? ss.s_out : sc;
    const int schedule = (feed || extras) ? 0 : (has_w || ctx->opt_schedule == 2 ? ctx->opt_schedule : 0);
    std::vector<char> seen(feed ? (size_t)P : 0, 0);  // source intervals the feed has been called for
    const float* Xh = static_cast<const float*>(X->data);
    float* Yh = static_cast<float*>(Y->data);
    float* A = static_cast<float*>(ctx->st_A.p);
    int64_t bytes_h2d = 0, bytes_d2h = 0;
    int64_t step = 0, ystep = 0;
    bool used[2] = {false, false}, yused[2] = {false, false};
    bool a_busy = false;  // ev_a_done guards the accumulator buffer

    bool d_busy = false;  // ev_d_free guards the destination parts
    if (schedule != 0 && grid->a_host_bytes < (size_t)n * F * 4) {  // host home of the swapped accumulators
        if (grid->a_host) (void)hipHostFree(grid->a_host);
        grid->a_host = nullptr;
        grid->a_host_bytes = 0;
        HIP_TRY(ctx, hipHostMalloc(reinterpret_cast<void**>(&grid->a_host), (size_t)n * F * 4, hipHostMallocDefault));
        grid->a_host_bytes = (size_t)n * F * 4;
    }

    // pack W^T once (on the compute stream)
    int64_t n_pad = 0, k_pad = 0, ldbt = 0;
    if (has_w) {
        int64_t n_pad2 = 0, k_pad2 = 0;
        bt_padded_shape((int32_t)F_out, (int32_t)Fw, SAGA_F32, &n_pad, &k_pad);
        if (has_self) bt_padded_shape((int32_t)F_out, (int32_t)F_self, SAGA_F32, &n_pad2, &k_pad2);
        ldbt = k_pad + k_pad2;
        if ((st = ctx->dev_alloc(&ctx->ws_bt, (size_t)(n_pad * ldbt) * 4))) return st;
        HIP_TRY(ctx, launch_zero_bytes(ctx->ws_bt.p, (size_t)(n_pad * ldbt) * 4, sc));
        HIP_TRY(ctx, launch_pack_bt_transpose(vp->W->data, vp->W->ld, (int32_t)Fw, (int32_t)F_out, SAGA_F32, ctx->ws_bt.p, ldbt, 0, sc));
        if (has_self)
            HIP_TRY(ctx, launch_pack_bt_transpose(vp->W_self->data, vp->W_self->ld, (int32_t)F_self, (int32_t)F_out, SAGA_F32,
                                                  ctx->ws_bt.p, ldbt, k_pad, sc));
    }

    auto rows_of = [&](int j) { return std::min(n, ((int64_t)j + 1) * Dq) - (int64_t)j * Dq; };

    // A_j <- identity of the accumulator, once nobody reads the buffer any more
    auto fill_a = [&](int j) -> saga_status {
        if (a_busy) HIP_TRY(ctx, hipStreamWaitEvent(sc, ss.ev_a_done, 0));
        HIP_TRY(ctx, launch_fill_f32(A, rows_of(j) * Fw, agg == SAGA_AGG_SUM ? 0.f : -__builtin_huge_valf(), sc));
        if (gated) {  // the destination parts of this interval, once the previous interval's kernels have let go of the buffer
            if (d_busy) HIP_TRY(ctx, hipStreamWaitEvent(sin, ss.ev_d_free, 0));
            if (extras->dst_fill) {
                if (saga_status fs = extras->dst_fill((int64_t)j * Dq, rows_of(j), static_cast<float*>(ctx->st_D.p), sin, &bytes_h2d)) return fs;
            } else {
                const int64_t w1 = extras->dst2_rows ? Fa : Fd;  // columns that come from dst_rows
                HIP_TRY(ctx, hipMemcpy2DAsync(ctx->st_D.p, (size_t)Fd * 4, extras->dst_rows + (int64_t)j * Dq * extras->ld_dst,
                                              (size_t)extras->ld_dst * 4, (size_t)w1 * 4, (size_t)rows_of(j), hipMemcpyHostToDevice, sin));
                if (extras->dst2_rows)
                    HIP_TRY(ctx, hipMemcpy2DAsync(static_cast<float*>(ctx->st_D.p) + Fa, (size_t)Fd * 4,
                                                  extras->dst2_rows + (int64_t)j * Dq * extras->ld_dst2, (size_t)extras->ld_dst2 * 4,
                                                  (size_t)Fa * 4, (size_t)rows_of(j), hipMemcpyHostToDevice, sin));
                bytes_h2d += rows_of(j) * Fd * 4;
            }
            HIP_TRY(ctx, hipEventRecord(ss.ev_a_in, sin));
            HIP_TRY(ctx, hipStreamWaitEvent(sc, ss.ev_a_in, 0));
        }
        return SAGA_OK;
    };
    // stream V_i (unless it already sits in V[vbuf]) and C_ij in, then add the chunk into A_j
    auto load_and_gather = [&](int i, int j, int vbuf, bool load_v) -> saga_status {
        const ChunkMeta& m = grid->chunks[(size_t)j * P + i];
        const int b = (int)(step & 1);
        const int vb = vbuf >= 0 ? vbuf : b;
        const int64_t s0 = (int64_t)i * Sp, srows = std::min(n, s0 + Sp) - s0;
        // copy stream: wait until the kernels that last read this buffer pair are done
        if (used[b]) HIP_TRY(ctx, hipStreamWaitEvent(sin, ss.ev_free[b], 0));
        if (load_v) {
            // a source buffer chosen by the caller (destination order innermost) was last read by the kernels of the
            // interval before the previous one, which may be the step just before this one when an interval had no
            // edges at all: wait for both buffer pairs then
            if (used[1 - b] && (vb != b || vbuf >= 0)) HIP_TRY(ctx, hipStreamWaitEvent(sin, ss.ev_free[1 - b], 0));
            if (feed) {
                if (saga_status fs = feed->fill(s0, srows, static_cast<float*>(ctx->st_V[vb].p), sin, !seen[(size_t)i], &bytes_h2d))
                    return fs;
                seen[(size_t)i] = 1;
            } else {
                HIP_TRY(ctx, hipMemcpy2DAsync(ctx->st_V[vb].p, (size_t)F * 4, Xh + s0 * X->ld, (size_t)X->ld * 4, (size_t)F * 4,
                                              (size_t)srows, hipMemcpyHostToDevice, sin));
                bytes_h2d += srows * F * 4;
            }
        }
        if (m.nnz == 0) {  // only a feed brings us here: the interval had to be visited, there is nothing to add
            HIP_TRY(ctx, hipEventRecord(ss.ev_free[b], sin));
            used[b] = true;
            ++step;
            return SAGA_OK;
        }
        HIP_TRY(ctx, hipMemcpyAsync(ctx->st_C[b].p, m.host, m.bytes, hipMemcpyHostToDevice, sin));
        HIP_TRY(ctx, hipEventRecord(ss.ev_ready[b], sin));
        bytes_h2d += (int64_t)m.bytes;
        HIP_TRY(ctx, hipStreamWaitEvent(sc, ss.ev_ready[b], 0));
        const char* cb = static_cast<const char*>(ctx->st_C[b].p);
        GatherArgs ga{};
        ga.items = reinterpret_cast<const WorkItem*>(cb + m.off_items);
        ga.n_items = m.n_items;
        ga.n_team = m.n_team;
        ga.row_idx = reinterpret_cast<const int32_t*>(cb + m.off_ridx);
        ga.edge_w = weighted ? reinterpret_cast<const float*>(cb + m.off_w) : nullptr;
        ga.src = ctx->st_V[vb].p;
        ga.ld_src = F;
        ga.F = (int32_t)Fa;
        ga.dtype = SAGA_F32;
        ga.op = op;
        ga.agg = agg;
        ga.out = A;
        ga.ld_out = Fw;
        if (gated) {  // rows [Ps | M] travel, the destination parts are resident
            ga.src2 = static_cast<const float*>(ctx->st_V[vb].p) + Fa;
            ga.ld_src2 = F;
            ga.dst = static_cast<const float*>(ctx->st_D.p);
            ga.dst_sigmoid = extras->dst_sigmoid ? 1 : 0;
            ga.ld_dst = Fd;
            if (Fd >= 2 * Fa) {
                ga.dst2 = ga.dst + Fa;
                ga.ld_dst2 = Fd;
            }
            if (Fd == 3 * Fa) {  // third constant row: the maximum gathered at this destination
                ga.dst3 = ga.dst + 2 * Fa;
                ga.ld_dst3 = Fd;
            }
            if (third_row) {
                ga.src3 = static_cast<const float*>(ctx->st_V[vb].p) + 2 * Fa;
                ga.ld_src3 = F;
            }
        }
        ga.partials = static_cast<float*>(ctx->st_partials.p);
        if (n_out == 2) {
            ga.out2 = A + Fa;
            ga.ld_out2 = Fw;
            ga.partials2 = ga.partials + (size_t)m.n_slots * Fa;
        }
        ga.accumulate = 1;
        ga.xcd_remap = ctx->opt_xcd_remap;
        ga.mma = ctx->opt_mma;
        HIP_TRY(ctx, launch_gather(ga, sc));
        if (m.n_heavy > 0) {
            CombineArgs ca{};
            ca.heavy = reinterpret_cast<const HeavyVertex*>(cb + m.off_heavy);
            ca.n_heavy = m.n_heavy;
            ca.partials = ga.partials;
            ca.F = (int32_t)Fa;
            ca.agg = agg;
            ca.out = A;
            ca.ld_out = Fw;
            ca.accumulate = 1;
            HIP_TRY(ctx, launch_combine(ca, sc));
            if (n_out == 2) {
                ca.partials = ga.partials2;
                ca.out = ga.out2;
                HIP_TRY(ctx, launch_combine(ca, sc));
            }
        }
        HIP_TRY(ctx, hipEventRecord(ss.ev_free[b], sc));
        used[b] = true;
        ++step;
        return SAGA_OK;
    };
    // ApplyVertex on the resident A_j (or A_j itself when there is none) and its way back to the host
    auto apply_and_drain = [&](int j) -> saga_status {
        const int64_t v0 = (int64_t)j * Dq, rows = rows_of(j);
        if (agg == SAGA_AGG_MAX) HIP_TRY(ctx, launch_neg_inf_to_zero(A, rows * Fw, sc));
        if (extras && extras->after_gather)
            if (saga_status hs = extras->after_gather(v0, rows, A, sc, &bytes_h2d)) return hs;
        if (gated) {  // every kernel that reads the destination parts of this interval (or what dst_fill left beside them,
                      // which after_gather may use) has been enqueued
            HIP_TRY(ctx, hipEventRecord(ss.ev_d_free, sc));
            d_busy = true;
        }
        if (!Yh) {  // nobody wants the rows (a backward pass that only needs what after_gather adds up)
            HIP_TRY(ctx, hipEventRecord(ss.ev_a_done, sc));
            a_busy = true;
            return SAGA_OK;
        }
        // the Gather output itself, for a caller that keeps it for back-propagation (on the outbound stream)
        auto accum_to_host = [&]() -> saga_status {
            HIP_TRY(ctx, hipMemcpy2DAsync(extras->accum_rows + v0 * extras->ld_accum, (size_t)extras->ld_accum * 4, A, (size_t)Fw * 4,
                                          (size_t)Fa * 4, (size_t)rows, hipMemcpyDeviceToHost, sout));
            bytes_d2h += rows * Fa * 4;
            return SAGA_OK;
        };
        const bool want_accum = extras && extras->accum_rows;
        if (!has_w) {
            HIP_TRY(ctx, hipEventRecord(ss.ev_a_ready, sc));
            HIP_TRY(ctx, hipStreamWaitEvent(sout, ss.ev_a_ready, 0));
            HIP_TRY(ctx, hipMemcpy2DAsync(Yh + v0 * Y->ld, (size_t)Y->ld * 4, A, (size_t)Fw * 4, (size_t)Fw * 4, (size_t)rows,
                                          hipMemcpyDeviceToHost, sout));
            bytes_d2h += rows * Fw * 4;
            if (want_accum)
                if (saga_status as = accum_to_host()) return as;
            HIP_TRY(ctx, hipEventRecord(ss.ev_a_done, sout));
            a_busy = true;
            return SAGA_OK;
        }
        for (int64_t r0 = 0; r0 < rows; r0 += y_tile_rows) {
            const int64_t tr = std::min(y_tile_rows, rows - r0);
            const int b = (int)(ystep & 1);
            if (yused[b]) HIP_TRY(ctx, hipStreamWaitEvent(sc, ss.ev_y_free[b], 0));
            GemmArgs ge{};
            if (has_self) {
                // the tile's own rows of the layer input, for the second operand; the staging buffer is free once the
                // product that last read it has been followed by its copy-out (ev_y_free)
                if (yused[b]) HIP_TRY(ctx, hipStreamWaitEvent(sin, ss.ev_y_free[b], 0));
                if (extras->self_fill) {
                    if (saga_status fs = extras->self_fill(v0 + r0, tr, static_cast<float*>(ctx->st_S[b].p), sin, &bytes_h2d)) return fs;
                } else {
                    HIP_TRY(ctx, hipMemcpy2DAsync(ctx->st_S[b].p, (size_t)F_self * 4, extras->self_rows + (v0 + r0) * extras->ld_self,
                                                  (size_t)extras->ld_self * 4, (size_t)F_self * 4, (size_t)tr, hipMemcpyHostToDevice, sin));
                    bytes_h2d += tr * F_self * 4;
                }
                HIP_TRY(ctx, hipEventRecord(ss.ev_s_ready[b], sin));
                HIP_TRY(ctx, hipStreamWaitEvent(sc, ss.ev_s_ready[b], 0));
                ge.A2 = ctx->st_S[b].p;
                ge.lda2 = F_self;
                ge.K2 = (int32_t)F_self;
            }
            ge.A = A + r0 * Fw;
            ge.lda = Fw;
            ge.Bt = ctx->ws_bt.p;
            ge.ldbt = ldbt;
            ge.bias = vp->bias ? static_cast<const float*>(vp->bias->data) : nullptr;
            ge.C = ctx->st_Y[b].p;
            ge.ldc = F_out;
            ge.M = tr;
            ge.N = (int32_t)F_out;
            ge.K = (int32_t)Fw;
            ge.dtype = ge.out_dtype = SAGA_F32;
            ge.act = vp->act;
            HIP_TRY(ctx, launch_gemm(ge, sc));
            HIP_TRY(ctx, hipEventRecord(ss.ev_y_ready[b], sc));
            HIP_TRY(ctx, hipStreamWaitEvent(sout, ss.ev_y_ready[b], 0));
            HIP_TRY(ctx, hipMemcpy2DAsync(Yh + (v0 + r0) * Y->ld, (size_t)Y->ld * 4, ctx->st_Y[b].p, (size_t)F_out * 4,
                                          (size_t)F_out * 4, (size_t)tr, hipMemcpyDeviceToHost, sout));
            HIP_TRY(ctx, hipEventRecord(ss.ev_y_free[b], sout));
            bytes_d2h += tr * F_out * 4;
            yused[b] = true;
            ++ystep;
        }
        if (want_accum) {  // A_j is free again when the products that read it are done and its copy has left
            HIP_TRY(ctx, hipEventRecord(ss.ev_a_ready, sc));
            HIP_TRY(ctx, hipStreamWaitEvent(sout, ss.ev_a_ready, 0));
            if (saga_status as = accum_to_host()) return as;
            HIP_TRY(ctx, hipEventRecord(ss.ev_a_done, sout));
        } else {
            HIP_TRY(ctx, hipEventRecord(ss.ev_a_done, sc));
        }
        a_busy = true;
        return SAGA_OK;
    };
    // the baselines swap the accumulator of interval j between the device and its host home
    auto swap_out = [&](int j) -> saga_status {
        HIP_TRY(ctx, hipEventRecord(ss.ev_a_ready, sc));
        HIP_TRY(ctx, hipStreamWaitEvent(sout, ss.ev_a_ready, 0));
        HIP_TRY(ctx, hipMemcpyAsync(grid->a_host + (int64_t)j * Dq * F, A, (size_t)rows_of(j) * F * 4, hipMemcpyDeviceToHost, sout));
        HIP_TRY(ctx, hipEventRecord(ss.ev_a_done, sout));
        a_busy = true;
        bytes_d2h += rows_of(j) * F * 4;
        return SAGA_OK;
    };
    auto swap_in = [&](int j) -> saga_status {
        if (a_busy) HIP_TRY(ctx, hipStreamWaitEvent(sin, ss.ev_a_done, 0));
        HIP_TRY(ctx, hipMemcpyAsync(A, grid->a_host + (int64_t)j * Dq * F, (size_t)rows_of(j) * F * 4, hipMemcpyHostToDevice, sin));
        HIP_TRY(ctx, hipEventRecord(ss.ev_a_in, sin));
        HIP_TRY(ctx, hipStreamWaitEvent(sc, ss.ev_a_in, 0));
        bytes_h2d += rows_of(j) * F * 4;
        return SAGA_OK;
    };
    auto has_edges = [&](int i, int j) { return grid->chunks[(size_t)j * P + i].nnz > 0 || (feed && !seen[(size_t)i]); };
#define SAGA_STEP(call)                       \
    do {                                      \
        if (saga_status st__ = (call)) return st__; \
    } while (0)

    if (schedule == 0) {
        // the paper's schedule: A_j stays resident until its ApplyVertex has consumed it
        for (int j = 0; j < Q && rows_of(j) > 0; ++j) {
            SAGA_STEP(fill_a(j));
            for (int i = 0; i < P; ++i)
                if (has_edges(i, j)) SAGA_STEP(load_and_gather(i, j, -1, true));
            SAGA_STEP(apply_and_drain(j));
        }
    } else if (schedule == 1) {
        // stage by stage: the whole Gather stage first (accumulators swapped out), then ApplyVertex
        for (int j = 0; j < Q && rows_of(j) > 0; ++j) {
            SAGA_STEP(fill_a(j));
            for (int i = 0; i < P; ++i)
                if (has_edges(i, j)) SAGA_STEP(load_and_gather(i, j, -1, true));
            SAGA_STEP(swap_out(j));
        }
        for (int j = 0; j < Q && rows_of(j) > 0; ++j) {
            SAGA_STEP(swap_in(j));
            SAGA_STEP(apply_and_drain(j));
        }
    } else {
        // destination order innermost: a source interval stays, the accumulators are swapped per chunk
        for (int j = 0; j < Q && rows_of(j) > 0; ++j) {
            SAGA_STEP(fill_a(j));
            SAGA_STEP(swap_out(j));
        }
        for (int i = 0; i < P; ++i) {
            bool first = true;
            for (int j = 0; j < Q && rows_of(j) > 0; ++j) {
                if (!has_edges(i, j)) continue;
                SAGA_STEP(swap_in(j));
                SAGA_STEP(load_and_gather(i, j, i & 1, first));
                first = false;
                SAGA_STEP(swap_out(j));
            }
        }
        for (int j = 0; j < Q && rows_of(j) > 0; ++j) {
            SAGA_STEP(swap_in(j));
            SAGA_STEP(apply_and_drain(j));
        }
    }
#undef SAGA_STEP
    HIP_TRY(ctx, hipStreamSynchronize(sin));
    HIP_TRY(ctx, hipStreamSynchronize(sc));
    HIP_TRY(ctx, hipStreamSynchronize(sout));

    const double ms = std::chrono::duration<double, std::milli>(std::chrono::steady_clock::now() - t_begin).count();
    ctx->acc.ms_wall_streamed += ms;
    ctx->acc.bytes_h2d += bytes_h2d;
    ctx->acc.bytes_d2h += bytes_d2h;
    ctx->acc.plan_dst_intervals = Q;
    ctx->acc.plan_src_intervals = P;
    int64_t items = 0, heavy = 0;
    for (const auto& m : grid->chunks) {
        items += m.n_items;
        heavy += m.n_heavy;
    }
    ctx->acc.n_work_items = items;
    ctx->acc.n_split_vertices = heavy;
    ctx->acc.n_calls += 1;
    return SAGA_OK;
}

// New edge data on a host graph that already has a tiling: the weights inside the pinned payloads are written again
// from g->h_edge_data, chunk by chunk. Nothing is allocated or freed; the caller has made sure no streamed call is in
// flight (every streamed call synchronises its streams before it returns).
void chunk_grid_refresh_weights(saga_graph* g)
{
    ChunkGrid* grid = g->grid;
    if (!grid || !grid->weighted || g->h_edge_data.empty()) return;
    parallel_for((int64_t)grid->chunks.size(), 8, [&](int64_t c) {
        const ChunkMeta& m = grid->chunks[(size_t)c];
        if (!m.host || m.nnz == 0) return;
        try {
            std::vector<int64_t> lcp, lo;
            locate_chunk(g, grid->Dq, grid->Sp, (int)(c % grid->P), (int)(c / grid->P), &lcp, &lo);
            fill_chunk_weights(g, lcp, lo, reinterpret_cast<float*>(m.host + m.off_w));
        } catch (...) {
            // out of host memory for two small index vectors: fall back to one column at a time
            const int64_t v0 = (c / grid->P) * grid->Dq, v1 = std::min(g->n, v0 + grid->Dq);
            const int64_t s0 = (c % grid->P) * grid->Sp, s1 = std::min(g->n, s0 + grid->Sp);
            float* out = reinterpret_cast<float*>(m.host + m.off_w);
            const int32_t* ri = g->h_row_idx.data();
            for (int64_t v = v0; v < v1; ++v) {
                const int32_t* b = ri + g->h_col_ptr[(size_t)v];
                const int32_t* e = ri + g->h_col_ptr[(size_t)v + 1];
                const int32_t* l = std::lower_bound(b, e, (int32_t)s0);
                const int32_t* h = std::lower_bound(l, e, (int32_t)std::min<int64_t>(s1, 0x7fffffff));
                for (const int32_t* q = l; q < h; ++q) *out++ = g->h_edge_data[(size_t)(q - ri)];
            }
        }
    });
}

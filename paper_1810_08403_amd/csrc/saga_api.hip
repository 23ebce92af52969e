// C ABI of libsaga: contexts, graph ingest, the host-side work list and id re-encoding,
// the device-resident layer (Scatter-ApplyEdge-Gather fused, then ApplyVertex; Sections
// 2.2 and 3.2), the per-vertex products hoisted out of gated and pooled ApplyEdge
// functions, and argument checking for every entry point.
#include <algorithm>
#include <cstring>
#include <exception>
#include <new>

#include "saga_internal.h"

// ---------------------------------------------------------------------------
// context plumbing
// ---------------------------------------------------------------------------
saga_status saga_ctx::fail(saga_status s, const char* fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    err = buf;
    return s;
}

// Scratch memory of saga_layer_forward_noalloc: the Gather output, the partial rows of cut columns, the packed weights
// and the per-vertex products of one resident layer, for callers that must not allocate. One array per GPU for the
// life of the process; every call on that GPU shares it.
constexpr size_t kScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

saga_status saga_ctx::dev_alloc(DevBuf* b, size_t bytes)
{
    if (arena_active) {
        if (b->p && b->bytes >= bytes) return SAGA_OK;
        const size_t rounded = (bytes + 255) / 256 * 256;
        if (arena_used + rounded > kScratchBytes)
            return fail(SAGA_ERR_BUDGET, "this layer needs more than the %zu bytes of scratch memory saga_layer_forward_noalloc has",
                        kScratchBytes);
        b->p = bytes ? scratch_ptr + arena_used : nullptr;
        b->bytes = bytes ? rounded : 0;
        arena_used += bytes ? rounded : 0;
        return SAGA_OK;
    }
    if (b->p && b->bytes >= bytes) return SAGA_OK;
    dev_free(b);
    if (bytes == 0) return SAGA_OK;
    const size_t rounded = (bytes + 255) / 256 * 256;
    void* p = nullptr;
    hipError_t e = hipMalloc(&p, rounded);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return fail(SAGA_ERR_HIP, "hipMalloc(%zu) failed: %s", rounded, hipGetErrorString(e));
    }
    b->p = p;
    b->bytes = rounded;
    cur_bytes += rounded;
    peak_bytes = std::max(peak_bytes, cur_bytes);
    return SAGA_OK;
}

void saga_ctx::dev_free(DevBuf* b)
{
    if (arena_active) {  // carved from the static array: nothing to give back
        b->p = nullptr;
        b->bytes = 0;
        return;
    }
    if (b->p) {
        (void)hipFree(b->p);
        cur_bytes -= b->bytes;
    }
    b->p = nullptr;
    b->bytes = 0;
}

void saga_ctx::make_room(size_t bytes)
{
    if (budget == 0 || cur_bytes + bytes <= budget) return;
    for (DevBuf* b : {&st_A, &st_V[0], &st_V[1], &st_C[0], &st_C[1], &st_Y[0], &st_Y[1], &st_partials, &st_D, &st_S[0], &st_S[1]}) dev_free(b);
}

saga_status saga_ctx::drain_events()
{
    if (ev_used == 0) return SAGA_OK;
    HIP_TRY(this, hipStreamSynchronize(stream));
    for (size_t i = 0; i < ev_used; ++i) {
        EventSet& es = ev_pool[i];
        float ms = 0.f;
        // ev[0] start, ev[1] after hoist, ev[2] after gather, ev[3] after combine, ev[4] after ApplyVertex
        if (es.has_hoist) {
            HIP_TRY(this, hipEventElapsedTime(&ms, es.ev[0], es.ev[1]));
            acc.ms_hoist += ms;
        }
        HIP_TRY(this, hipEventElapsedTime(&ms, es.ev[1], es.ev[2]));
        acc.ms_gather += ms;
        if (es.has_dense) {
            HIP_TRY(this, hipEventElapsedTime(&ms, es.ev[1], es.ev_dense));
            acc.ms_dense_blocks += ms;
        }
        if (es.has_combine) {
            HIP_TRY(this, hipEventElapsedTime(&ms, es.ev[2], es.ev[3]));
            acc.ms_combine += ms;
        }
        if (es.has_apply) {
            HIP_TRY(this, hipEventElapsedTime(&ms, es.ev[3], es.ev[4]));
            acc.ms_apply_vertex += ms;
        }
        HIP_TRY(this, hipEventElapsedTime(&ms, es.ev[0], es.ev[4]));
        acc.ms_total += ms;
        acc.n_gather_launches += es.n_gather_launches;
        acc.n_calls += 1;
    }
    ev_used = 0;
    return SAGA_OK;
}

// Work list of a CSC block (Section 3.3: one in-edge group per execution unit,
// heavy groups cut into consecutive sub-groups). Columns with more than
// cut_degree in-edges are cut into pieces that end on multiples of stripe_rows
// source rows and hold at least team * min_edges edges; the pieces of all
// columns are then ordered by source stripe, so that the wavefronts in flight
// at any time read one narrow band of the source rows: the 2-D tiling of
// Section 3.1 applied at the level of the L2. With team = 4 a piece is
// processed by the four wavefronts of one workgroup (team items come first in
// the list); with team = 1 by one wavefront like a whole light column.
void build_work_list(const int64_t* col_ptr, const int32_t* row_idx, int64_t n_cols, const WorkListParams& p,
                     WorkList* out, const int32_t* extra_slots)
{
    out->items.clear();
    out->heavy.clear();
    out->n_slots = 0;
    out->n_team = 0;
    out->max_degree = 0;
    std::vector<WorkItem> whole;
    whole.reserve((size_t)n_cols);
    // A piece's place in the list: the band of its first source, then the band of its last one, then its column. The
    // wavefronts that run at the same time take neighbouring pieces; a piece of a column with few edges per band reaches
    // over many bands, and with the pieces of one first band in column order a band's rows were shared with pieces that
    // reach anywhere between one band and fifty further. Next to pieces with the same reach the window of rows the
    // neighbours read is the same one (an LRU model of the L2s that reproduces the measured miss rate of the remainder of
    // the R-MAT 18 workload, 27 %, gives 17 % for this order; order 0 is the old one).
    struct Piece {
        int64_t first, last;  // stripes
        WorkItem it;
    };
    std::vector<Piece> pieces;
    const int64_t R = p.stripe_rows > 0 ? p.stripe_rows : 0;
    const int64_t team = p.team > 1 ? p.team : 1;
    const int64_t min_piece = std::max<int64_t>(1, p.min_edges * team);
    for (int64_t v = 0; v < n_cols; ++v) {
        const int64_t b = col_ptr[v], e = col_ptr[v + 1];
        const int64_t deg = e - b;
        out->max_degree = std::max(out->max_degree, deg);
        const int32_t extra = extra_slots ? extra_slots[v] : 0;
        if (deg == 0 && p.skip_empty && extra == 0) continue;
        if (extra > 0 && deg <= p.cut_degree) {
            // partial rows written elsewhere come first; what is left of the column is one more partial row (or none)
            HeavyVertex h{(int32_t)v, (int32_t)out->n_slots, extra + (deg > 0 ? 1 : 0), 0};
            out->n_slots += extra;
            if (deg > 0) whole.push_back(WorkItem{(int32_t)v, (int32_t)b, (int32_t)e, (int32_t)(out->n_slots++)});
            out->heavy.push_back(h);
            continue;
        }
        if (deg <= p.cut_degree) {
            whole.push_back(WorkItem{(int32_t)v, (int32_t)b, (int32_t)e, -1});
            continue;
        }
        const size_t first_piece = pieces.size();
        int64_t pos = b;
        while (pos < e) {
            int64_t q = std::min(e, pos + min_piece);
            if (R > 0 && q < e) {
                // extend to the end of the stripe that holds the last edge taken
                const int64_t bound = ((int64_t)row_idx[q - 1] / R + 1) * R;
                q = std::lower_bound(row_idx + q, row_idx + e, bound,
                                     [](int32_t a, int64_t bnd) { return (int64_t)a < bnd; }) - row_idx;
            }
            if (e - q < min_piece / 2) q = e;  // do not leave a sliver behind
            const int64_t stripe = R > 0 ? (int64_t)row_idx[pos] / R : (pos - b) / min_piece;
            const int64_t last = (R > 0 && p.order == 1) ? (int64_t)row_idx[q - 1] / R : 0;
            pieces.push_back(Piece{stripe, last, WorkItem{(int32_t)v, (int32_t)pos, (int32_t)q, -1}});
            pos = q;
        }
        const size_t n_p = pieces.size() - first_piece;
        if (extra > 0) {
            HeavyVertex h{(int32_t)v, (int32_t)out->n_slots, (int32_t)(extra + n_p), 0};
            out->n_slots += extra;
            for (size_t i = 0; i < n_p; ++i) pieces[first_piece + i].it.slot = (int32_t)(out->n_slots++);
            out->heavy.push_back(h);
            continue;
        }
        if (n_p == 1) {
            // one piece after all: its result is the vertex's row. A team still takes it
            // (four wavefronts share the edges); without teams it is an ordinary whole column.
            if (team == 1) {
                whole.push_back(pieces.back().it);
                pieces.pop_back();
            }
            continue;
        }
        HeavyVertex h{(int32_t)v, (int32_t)out->n_slots, (int32_t)n_p, 0};
        for (size_t i = 0; i < n_p; ++i) pieces[first_piece + i].it.slot = (int32_t)(out->n_slots++);
        out->heavy.push_back(h);
    }
    std::sort(pieces.begin(), pieces.end(), [](const Piece& a, const Piece& b) {
        if (a.first != b.first) return a.first < b.first;
        if (a.last != b.last) return a.last < b.last;
        if (a.it.v != b.it.v) return a.it.v < b.it.v;
        return a.it.e0 < b.it.e0;
    });
    out->items.reserve(pieces.size() + whole.size());
    for (const Piece& pc : pieces) out->items.push_back(pc.it);
    out->n_team = team > 1 ? (int64_t)pieces.size() : 0;
    out->items.insert(out->items.end(), whole.begin(), whole.end());
}

// The dense-block plan of a CSC (see HybridPlan). Two passes over the edges, destination tile by destination tile, on
// several threads: the first counts the edges of every (destination tile, source tile) block and decides which blocks
// and tiles go to the matrix cores, the second writes the dense edges block by block and the remainder as a CSC.
void build_hybrid_plan(const int64_t* col_ptr, const int32_t* row_idx, int64_t n, const HybridParams& hp, HybridPlan* out)
{
    *out = HybridPlan{};
    const int64_t nnz = col_ptr[n];
    const int64_t n_dt = (n + kDenseM - 1) / kDenseM, n_st = (n + kDenseK - 1) / kDenseK;
    out->n_dst_tiles = n_dt;
    out->n_src_tiles = n_st;
    // ranks: heavy first, ties by id
    std::vector<int64_t> outdeg((size_t)n, 0);
    for (int64_t e = 0; e < nnz; ++e) ++outdeg[(size_t)row_idx[e]];
    std::vector<int32_t> dorder((size_t)n), sorder((size_t)n);
    for (int64_t v = 0; v < n; ++v) dorder[(size_t)v] = sorder[(size_t)v] = (int32_t)v;
    std::stable_sort(dorder.begin(), dorder.end(),
                     [&](int32_t a, int32_t b) { return col_ptr[a + 1] - col_ptr[a] > col_ptr[b + 1] - col_ptr[b]; });
    std::stable_sort(sorder.begin(), sorder.end(), [&](int32_t a, int32_t b) { return outdeg[(size_t)a] > outdeg[(size_t)b]; });
    std::vector<int32_t> spos((size_t)n);
    for (int64_t r = 0; r < n; ++r) spos[(size_t)sorder[(size_t)r]] = (int32_t)r;
    out->dst_order.assign((size_t)n_dt * kDenseM, -1);
    out->src_tile_ids.assign((size_t)n_st * kDenseK, 0);
    for (int64_t r = 0; r < n; ++r) {
        out->dst_order[(size_t)r] = dorder[(size_t)r];
        out->src_tile_ids[(size_t)r] = sorder[(size_t)r];
    }
    out->extra_slots.assign((size_t)n, 0);

    // pass 1: per destination tile, the dense source tiles (ascending) and their edge counts
    struct TilePlan {
        std::vector<int32_t> st;   // dense source tiles
        std::vector<int32_t> cnt;  // edges of each
    };
    std::vector<TilePlan> tp((size_t)n_dt);
    std::vector<int64_t> rem_deg((size_t)n, 0);
    const int n_threads = 16;
    std::atomic<bool> failed{false};
    parallel_for(n_threads, n_threads, [&](int64_t th) {
        try {
            std::vector<int32_t> cnt((size_t)n_st, 0), touched;
            for (int64_t t = th; t < n_dt; t += n_threads) {
                touched.clear();
                for (int m = 0; m < kDenseM; ++m) {
                    const int32_t v = out->dst_order[(size_t)t * kDenseM + m];
                    if (v < 0) continue;
                    for (int64_t e = col_ptr[v]; e < col_ptr[v + 1]; ++e) {
                        const int32_t st = spos[(size_t)row_idx[e]] / kDenseK;
                        if (cnt[(size_t)st]++ == 0) touched.push_back(st);
                    }
                }
                int64_t gain = 0;
                for (int32_t st : touched)
                    if (cnt[(size_t)st] >= hp.min_block_edges) gain += cnt[(size_t)st] - hp.min_block_edges;
                if (gain >= hp.min_tile_gain && gain > 0) {
                    std::sort(touched.begin(), touched.end());
                    for (int32_t st : touched)
                        if (cnt[(size_t)st] >= hp.min_block_edges) {
                            tp[(size_t)t].st.push_back(st);
                            tp[(size_t)t].cnt.push_back(cnt[(size_t)st]);
                        }
                }
                for (int32_t st : touched) cnt[(size_t)st] = 0;
            }
        } catch (...) {
            failed = true;
        }
    });
    if (failed) throw std::bad_alloc();

    // blocks, chunks and offsets
    std::vector<int64_t> tile_b0((size_t)n_dt + 1, 0);
    for (int64_t t = 0; t < n_dt; ++t) tile_b0[(size_t)t + 1] = tile_b0[(size_t)t] + (int64_t)tp[(size_t)t].st.size();
    const int64_t nb = tile_b0[(size_t)n_dt];
    if (nb > 0x7fffffffLL - 1) throw std::bad_alloc();
    out->blk_src_tile.resize((size_t)nb);
    out->blk_e0.assign((size_t)nb + 1, 0);
    out->blk_tile.assign((size_t)nb, -1);
    std::vector<int64_t> blk_t0((size_t)nb + 1, 0);  // offsets of the finished operands' edges in dt_addr / dt_edge
    int64_t nde = 0, ndt = 0, n_tiles = 0;
    const int64_t ch = std::max<int64_t>(1, hp.max_chunk_blocks);
    for (int64_t t = 0; t < n_dt; ++t) {
        const TilePlan& p = tp[(size_t)t];
        const int64_t b0 = tile_b0[(size_t)t], k = (int64_t)p.st.size();
        for (int64_t i = 0; i < k; ++i) {
            out->blk_src_tile[(size_t)(b0 + i)] = p.st[(size_t)i];
            out->blk_e0[(size_t)(b0 + i)] = (int32_t)nde;
            blk_t0[(size_t)(b0 + i)] = ndt;
            if (p.cnt[(size_t)i] > kDenseListMax) {
                out->blk_tile[(size_t)(b0 + i)] = (int32_t)n_tiles++;
                ndt += p.cnt[(size_t)i];
            } else {
                nde += p.cnt[(size_t)i];
            }
        }
        if (k == 0) continue;
        const int64_t n_chunks = (k + ch - 1) / ch;
        for (int64_t c = 0; c < n_chunks; ++c)
            out->chunks.push_back(DenseChunk{(int32_t)t, (int32_t)(b0 + c * ch), (int32_t)std::min(b0 + k, b0 + (c + 1) * ch), (int32_t)c});
        for (int m = 0; m < kDenseM; ++m) {
            const int32_t v = out->dst_order[(size_t)t * kDenseM + m];
            if (v >= 0) out->extra_slots[(size_t)v] = (int32_t)n_chunks;
        }
    }
    if (nde > 0x7fffffffLL - 1 || ndt > 0x7fffffffLL - 1 || n_tiles * kDenseTileElems > 0x7fffffffLL - 1) throw std::bad_alloc();
    out->blk_e0[(size_t)nb] = (int32_t)nde;
    blk_t0[(size_t)nb] = ndt;
    out->n_dense_edges = nde + ndt;
    out->n_tiles = n_tiles;
    out->de_pos.resize((size_t)nde);
    out->de_edge.resize((size_t)nde);
    out->dt_addr.resize((size_t)ndt);
    out->dt_edge.resize((size_t)ndt);

    // pass 2: dense edges into their blocks; what is left of every column counted, then written
    std::vector<int64_t> rem_cnt((size_t)n, 0);
    parallel_for(n_threads, n_threads, [&](int64_t th) {
        try {
            std::vector<int32_t> blk_of((size_t)n_st, -1);
            std::vector<int32_t> cursor;
            for (int64_t t = th; t < n_dt; t += n_threads) {
                const TilePlan& p = tp[(size_t)t];
                const int64_t b0 = tile_b0[(size_t)t];
                for (size_t i = 0; i < p.st.size(); ++i) blk_of[(size_t)p.st[i]] = (int32_t)i;
                cursor.assign(p.st.size(), 0);
                for (int m = 0; m < kDenseM; ++m) {
                    const int32_t v = out->dst_order[(size_t)t * kDenseM + m];
                    if (v < 0) continue;
                    int64_t left = 0;
                    for (int64_t e = col_ptr[v]; e < col_ptr[v + 1]; ++e) {
                        const int32_t sp = spos[(size_t)row_idx[e]];
                        const int32_t bi = blk_of[(size_t)(sp / kDenseK)];
                        if (bi < 0) {
                            ++left;
                            continue;
                        }
                        const int k = sp % kDenseK;
                        // the weight's place in the block's 64 x 32 operand, in the lane order of the 16x16x32 matrix instruction:
                        // sub-tile of 16 destinations, then lane = (k / 8) * 16 + (m % 16), then k % 8
                        const int pos = (((m >> 4) * 64 + (k >> 3) * 16 + (m & 15)) << 3) + (k & 7);
                        const int32_t tile = out->blk_tile[(size_t)(b0 + bi)];
                        if (tile >= 0) {
                            const int64_t at = blk_t0[(size_t)(b0 + bi)] + cursor[(size_t)bi]++;
                            out->dt_addr[(size_t)at] = (int32_t)((int64_t)tile * kDenseTileElems + pos);
                            out->dt_edge[(size_t)at] = (int32_t)e;
                        } else {
                            const int64_t at = (int64_t)out->blk_e0[(size_t)(b0 + bi)] + cursor[(size_t)bi]++;
                            out->de_pos[(size_t)at] = (uint16_t)pos;
                            out->de_edge[(size_t)at] = (int32_t)e;
                        }
                    }
                    rem_cnt[(size_t)v] = left;
                }
                for (size_t i = 0; i < p.st.size(); ++i) blk_of[(size_t)p.st[i]] = -1;
            }
        } catch (...) {
            failed = true;
        }
    });
    if (failed) throw std::bad_alloc();
    out->rem_col_ptr.assign((size_t)n + 1, 0);
    for (int64_t v = 0; v < n; ++v) out->rem_col_ptr[(size_t)v + 1] = out->rem_col_ptr[(size_t)v] + rem_cnt[(size_t)v];
    const int64_t nrem = out->rem_col_ptr[(size_t)n];
    out->rem_row_idx.resize((size_t)nrem);
    out->rem_edge.resize((size_t)nrem);
    std::vector<int32_t> dpos((size_t)n);
    for (int64_t r = 0; r < n; ++r) dpos[(size_t)dorder[(size_t)r]] = (int32_t)r;
    parallel_for(n_threads, n_threads, [&](int64_t th) {
        // (no allocation in here: a tile's dense source tiles are looked up by binary search)
        const int64_t v0 = n * th / n_threads, v1 = n * (th + 1) / n_threads;
        for (int64_t v = v0; v < v1; ++v) {
            const TilePlan& p = tp[(size_t)(dpos[(size_t)v] / kDenseM)];
            int64_t at = out->rem_col_ptr[(size_t)v];
            for (int64_t e = col_ptr[v]; e < col_ptr[v + 1]; ++e) {
                const int32_t st = spos[(size_t)row_idx[e]] / kDenseK;
                if (!p.st.empty() && std::binary_search(p.st.begin(), p.st.end(), st)) continue;
                out->rem_row_idx[(size_t)at] = row_idx[e];
                out->rem_edge[(size_t)at] = (int32_t)e;
                ++at;
            }
        }
    });
}

namespace {

const char* kVersion = "saga-mi355x 0.1 (gfx950)";

bool tensor_ok(const saga_tensor* t)
{
    return t && t->data && t->rows >= 0 && t->cols > 0 && t->ld >= t->cols &&
           (t->dtype == SAGA_F32 || t->dtype == SAGA_BF16) && (t->mem == SAGA_MEM_DEVICE || t->mem == SAGA_MEM_HOST);
}

struct DeviceGuard {
    int prev = -1;
    explicit DeviceGuard(int dev)
    {
        if (hipGetDevice(&prev) != hipSuccess) prev = -1;
        if (prev != dev) (void)hipSetDevice(dev);
    }
    ~DeviceGuard()
    {
        if (prev >= 0) (void)hipSetDevice(prev);
    }
};

}  // namespace

// ---------------------------------------------------------------------------
// ApplyVertex on rows already on the device (used by both paths)
// ---------------------------------------------------------------------------
saga_status run_apply_vertex(saga_ctx* ctx, const void* A, int64_t lda, int32_t a_dtype, int64_t rows, int32_t F_in,
                             const saga_vertex_params* vp, const void* Xself, int64_t ld_self, int32_t F_self, void* Y,
                             int64_t ldy, int32_t y_dtype)
{
    const saga_tensor* W = vp->W;
    const int32_t F_out = (int32_t)W->cols;
    const bool self = vp->W_self != nullptr;
    int64_t n_pad, k_pad, n_pad2 = 0, k_pad2 = 0;
    bt_padded_shape(F_out, F_in, a_dtype, &n_pad, &k_pad);
    if (self) bt_padded_shape(F_out, F_self, a_dtype, &n_pad2, &k_pad2);
    const int64_t ldbt = k_pad + k_pad2;
    const size_t es = a_dtype == SAGA_F32 ? 4 : 2;
    if (saga_status st = ctx->dev_alloc(&ctx->ws_bt, (size_t)(n_pad * ldbt) * es)) return st;
    HIP_TRY(ctx, launch_zero_bytes(ctx->ws_bt.p, (size_t)(n_pad * ldbt) * es, ctx->stream));
    HIP_TRY(ctx, launch_pack_bt_transpose(W->data, W->ld, F_in, F_out, a_dtype, ctx->ws_bt.p, ldbt, 0, ctx->stream));
    if (self)
        HIP_TRY(ctx, launch_pack_bt_transpose(vp->W_self->data, vp->W_self->ld, F_self, F_out, a_dtype, ctx->ws_bt.p, ldbt,
                                              k_pad, ctx->stream));
    GemmArgs g{};
    g.A = A;
    g.lda = lda;
    if (self) {
        g.A2 = Xself;
        g.lda2 = ld_self;
        g.K2 = F_self;
    }
    g.Bt = ctx->ws_bt.p;
    g.ldbt = ldbt;
    g.bias = vp->bias ? static_cast<const float*>(vp->bias->data) : nullptr;
    g.C = Y;
    g.ldc = ldy;
    g.M = rows;
    g.N = F_out;
    g.K = F_in;
    g.dtype = a_dtype;
    g.out_dtype = y_dtype;
    g.act = vp->act;
    HIP_TRY(ctx, launch_gemm(g, ctx->stream));
    return SAGA_OK;
}

// ---------------------------------------------------------------------------
// work list of a resident graph, built for the width of the rows it will gather
// ---------------------------------------------------------------------------
static int64_t pow2_floor(int64_t x)
{
    int64_t p = 1;
    while (p * 2 <= x) p *= 2;
    return p;
}

WorkListParams work_list_params(const saga_ctx* ctx, int64_t row_bytes, int32_t width)
{
    WorkListParams p;
    p.min_edges = ctx->opt_split;
    // A piece costs one partial row written and read again (8 bytes per feature) on top of the rows it gathers. Where the
    // caller has not chosen, narrow outputs get finer pieces: measured with 128 fp32 features (512-byte partial rows, the
    // gated layer on R-MAT 20: 4.06 ms at 64 edges, 3.93 at 32, 4.01 at 16; CommNet 2.09 / 2.05 / 2.15) against 64 for
    // the 2 KiB partial rows of the R-MAT 18 workload (4.45 ms at 64, 4.57 at 48, 4.86 at 32, 4.71 at 80).
    if (!ctx->opt_split_set && width > 0 && width * 4 < 2048) p.min_edges = 32;
    p.cut_degree = ctx->opt_cut_degree > 0 ? ctx->opt_cut_degree : 2 * p.min_edges;
    p.stripe_rows = 0;
    if (ctx->opt_stripe_kb > 0) p.stripe_rows = std::max<int64_t>(64, pow2_floor(ctx->opt_stripe_kb * 1024 / std::max<int64_t>(row_bytes, 1)));
    p.team = ctx->opt_team ? 4 : 1;
    p.order = ctx->opt_piece_order;
    return p;
}

saga_status ensure_work_list(saga_ctx* ctx, saga_graph* g, int64_t row_bytes, int32_t width)
{
    // source rows that all fit the L2s together (8 x 4 MiB) are not what finer pieces are for: there is no miss to save,
    // only partial rows to add
    const bool table_in_l2 = g->n * std::max<int64_t>(row_bytes, 1) <= (32ll << 20);
    const WorkListParams p = work_list_params(ctx, row_bytes, table_in_l2 ? 0 : width);
    auto same = [](const WorkListParams& a, const WorkListParams& b) {
        return a.min_edges == b.min_edges && a.cut_degree == b.cut_degree && a.stripe_rows == b.stripe_rows && a.team == b.team && a.order == b.order;
    };
    if (same(p, g->list_params)) return SAGA_OK;
    if (ctx->arena_active)
        return ctx->fail(SAGA_ERR_UNSUPPORTED, "no work list for this row width yet: call saga_layer_forward once with the same shapes first");
    // park the current list, then look for one built earlier with these parameters
    if (g->list_params.min_edges >= 0) {
        if (g->saved_lists.size() >= 8) {
            ctx->dev_free(&g->saved_lists.front().items);
            ctx->dev_free(&g->saved_lists.front().heavy);
            g->saved_lists.erase(g->saved_lists.begin());
        }
        g->saved_lists.push_back(saga_graph::SavedList{g->list_params, g->d_items, g->d_heavy, g->n_items, g->n_team, g->n_heavy, g->n_slots});
        g->d_items = DevBuf{};
        g->d_heavy = DevBuf{};
        g->list_params = WorkListParams{-1, -1, -1, false, 1, 1};
    }
    for (size_t i = 0; i < g->saved_lists.size(); ++i) {
        if (!same(p, g->saved_lists[i].params)) continue;
        const saga_graph::SavedList sl = g->saved_lists[i];
        g->saved_lists.erase(g->saved_lists.begin() + (long)i);
        g->d_items = sl.items;
        g->d_heavy = sl.heavy;
        g->n_items = sl.n_items;
        g->n_team = sl.n_team;
        g->n_heavy = sl.n_heavy;
        g->n_slots = sl.n_slots;
        g->list_params = sl.params;
        return SAGA_OK;
    }
    std::vector<int32_t> h_row;
    WorkList wl;
    try {
        h_row.resize((size_t)std::max<int64_t>(g->nnz, 1));
    } catch (...) {
        return ctx->fail(SAGA_ERR_INTERNAL, "out of host memory");
    }
    if (g->nnz > 0) {
        HIP_TRY(ctx, hipMemcpyAsync(h_row.data(), g->d_row_idx.p, sizeof(int32_t) * (size_t)g->nnz, hipMemcpyDeviceToHost, ctx->stream));
        HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    }
    try {
        build_work_list(g->h_col_ptr.data(), h_row.data(), g->n, p, &wl);
    } catch (...) {
        return ctx->fail(SAGA_ERR_INTERNAL, "out of host memory");
    }
    if (saga_status st = ctx->dev_alloc(&g->d_items, sizeof(WorkItem) * std::max<size_t>(wl.items.size(), 1))) return st;
    if (saga_status st = ctx->dev_alloc(&g->d_heavy, sizeof(HeavyVertex) * std::max<size_t>(wl.heavy.size(), 1))) return st;
    if (!wl.items.empty())
        HIP_TRY(ctx, hipMemcpyAsync(g->d_items.p, wl.items.data(), sizeof(WorkItem) * wl.items.size(), hipMemcpyHostToDevice, ctx->stream));
    if (!wl.heavy.empty())
        HIP_TRY(ctx, hipMemcpyAsync(g->d_heavy.p, wl.heavy.data(), sizeof(HeavyVertex) * wl.heavy.size(), hipMemcpyHostToDevice, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));  // wl goes out of scope below
    g->n_items = (int64_t)wl.items.size();
    g->n_team = wl.n_team;
    g->n_heavy = (int64_t)wl.heavy.size();
    g->n_slots = wl.n_slots;
    g->list_params = p;
    return SAGA_OK;
}

void hybrid_free(saga_ctx* ctx, HybridDevice* h)
{
    for (DevBuf* b : {&h->chunks, &h->blk_src_tile, &h->blk_e0, &h->blk_tile, &h->de_pos, &h->de_edge, &h->de_w, &h->dt_addr, &h->dt_edge, &h->de_tiles,
                      &h->src_tile_ids, &h->tile_row_slot0,
                      &h->rem_row_idx, &h->rem_edge, &h->rem_w, &h->items, &h->heavy})
        ctx->dev_free(b);
    *h = HybridDevice{};
}

static HybridParams hybrid_params(const saga_ctx* ctx)
{
    HybridParams hp;
    if (ctx->opt_dense_min_edges > 0) hp.min_block_edges = ctx->opt_dense_min_edges;
    if (ctx->opt_dense_tile_gain >= 0) hp.min_tile_gain = ctx->opt_dense_tile_gain;
    if (ctx->opt_dense_chunk > 0) hp.max_chunk_blocks = (int32_t)ctx->opt_dense_chunk;
    return hp;
}

// The dense-block form of a resident graph for rows of `row_bytes` (the remainder's work list depends on the row width
// like any other): built on the host at the first call that can use it, kept in the graph handle.
saga_status ensure_hybrid(saga_ctx* ctx, saga_graph* g, int64_t row_bytes, int32_t width)
{
    HybridDevice& h = g->hyb;
    // The remainder's piece size goes by the bytes of a source row, not by the narrow-row rule of the general list: its
    // columns have lost their heavy blocks. Rows of 256 and 512 bytes keep 64 edges per piece (backward pass of the R-MAT
    // 18 workload, 128 bf16 features: 3.65 ms at 64, 3.98 at 32; 256 features: 3.42 at 64, 3.46 at 48); rows of 1 KiB take
    // fewer (forward layer of the same workload, 512 bf16 features, bands of 1 MiB: 4.11 ms at 48, 4.21 at 40, 4.23 at 56
    // and 64, 4.32 at 32, 4.73 at 80: longer pieces reach over more bands of source rows, shorter ones cost k_combine more
    // than the sparse kernel gains). Columns are cut from 128 edges on either way.
    (void)width;
    WorkListParams p = work_list_params(ctx, row_bytes, 0);
    // Rows of 1 KiB also take bands of 2 MiB of them instead of 1 MiB, and with those pieces of 40 edges: what is left of a
    // column after its well-filled blocks have gone has few edges per band, and a piece then ends at the next band
    // boundary sooner than it is worth (same workload, one session: 4.25 ms per layer with bands of 1 MiB and 48 edges;
    // with 2 MiB 4.16 at 48, 4.17 at 44, 4.11 at 40, 4.18 at 36, 4.22 at 32; with 4 MiB 4.32 at 48, 4.18 at 40, 4.17 at 32).
    const bool wide_rows = row_bytes >= 1024;
    if (!ctx->opt_split_set && wide_rows) p.min_edges = (!ctx->opt_stripe_set && p.stripe_rows > 0) ? 40 : 48;
    if (!ctx->opt_stripe_set && wide_rows && p.stripe_rows > 0) p.stripe_rows *= 2;
    const HybridParams hp = hybrid_params(ctx);
    auto same = [](const WorkListParams& a, const WorkListParams& b) {
        return a.min_edges == b.min_edges && a.cut_degree == b.cut_degree && a.stripe_rows == b.stripe_rows && a.team == b.team && a.order == b.order;
    };
    if (h.built && same(p, h.list_params) && hp.min_block_edges == h.hp.min_block_edges && hp.min_tile_gain == h.hp.min_tile_gain &&
        hp.max_chunk_blocks == h.hp.max_chunk_blocks)
        return SAGA_OK;
    if (ctx->arena_active)
        return ctx->fail(SAGA_ERR_UNSUPPORTED, "no dense-block plan for this row width yet: call saga_layer_forward once with the same shapes first");
    hybrid_free(ctx, &h);
    h.list_params = p;
    h.hp = hp;
    h.built = true;
    if (g->nnz == 0 || g->n >= (1LL << 30)) return SAGA_OK;
    std::vector<int32_t> h_row((size_t)g->nnz);
    HIP_TRY(ctx, hipMemcpyAsync(h_row.data(), g->d_row_idx.p, sizeof(int32_t) * (size_t)g->nnz, hipMemcpyDeviceToHost, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    HybridPlan plan;
    build_hybrid_plan(g->h_col_ptr.data(), h_row.data(), g->n, hp, &plan);
    if (plan.chunks.empty()) return SAGA_OK;  // nothing dense enough: the sparse kernel takes the whole graph
    WorkList wl;
    build_work_list(plan.rem_col_ptr.data(), plan.rem_row_idx.data(), g->n, p, &wl, plan.extra_slots.data());
    // first partial row of every destination that has dense blocks, by destination rank
    std::vector<int32_t> slot0_of((size_t)g->n, -1);
    for (const HeavyVertex& hv : wl.heavy) slot0_of[(size_t)hv.v] = hv.slot0;
    std::vector<int32_t> tile_row_slot0(plan.dst_order.size(), -1);
    for (size_t i = 0; i < plan.dst_order.size(); ++i) {
        const int32_t v = plan.dst_order[i];
        if (v >= 0 && plan.extra_slots[(size_t)v] > 0) tile_row_slot0[i] = slot0_of[(size_t)v];
    }
    auto up = [&](DevBuf* b, const void* src, size_t bytes) -> saga_status {
        if (saga_status st = ctx->dev_alloc(b, std::max<size_t>(bytes, 16))) return st;
        if (bytes) HIP_TRY(ctx, hipMemcpyAsync(b->p, src, bytes, hipMemcpyHostToDevice, ctx->stream));
        return SAGA_OK;
    };
    saga_status st;
    if ((st = up(&h.chunks, plan.chunks.data(), sizeof(DenseChunk) * plan.chunks.size())) ||
        (st = up(&h.blk_src_tile, plan.blk_src_tile.data(), 4 * plan.blk_src_tile.size())) ||
        (st = up(&h.blk_e0, plan.blk_e0.data(), 4 * plan.blk_e0.size())) ||
        (st = up(&h.blk_tile, plan.blk_tile.data(), 4 * plan.blk_tile.size())) ||
        (st = up(&h.de_pos, plan.de_pos.data(), 2 * plan.de_pos.size())) ||
        (st = up(&h.de_edge, plan.de_edge.data(), 4 * plan.de_edge.size())) ||
        (st = up(&h.dt_addr, plan.dt_addr.data(), 4 * plan.dt_addr.size())) ||
        (st = up(&h.dt_edge, plan.dt_edge.data(), 4 * plan.dt_edge.size())) ||
        (st = ctx->dev_alloc(&h.de_tiles, std::max<size_t>(2 * (size_t)plan.n_tiles * kDenseTileElems, 16))) ||
        (st = up(&h.src_tile_ids, plan.src_tile_ids.data(), 4 * plan.src_tile_ids.size())) ||
        (st = up(&h.tile_row_slot0, tile_row_slot0.data(), 4 * tile_row_slot0.size())) ||
        (st = up(&h.rem_row_idx, plan.rem_row_idx.data(), 4 * plan.rem_row_idx.size())) ||
        (st = up(&h.rem_edge, plan.rem_edge.data(), 4 * plan.rem_edge.size())) ||
        (st = up(&h.items, wl.items.data(), sizeof(WorkItem) * wl.items.size())) ||
        (st = up(&h.heavy, wl.heavy.data(), sizeof(HeavyVertex) * wl.heavy.size())) ||
        (st = ctx->dev_alloc(&h.de_w, std::max<size_t>(4 * plan.de_pos.size(), 16))) ||
        (st = ctx->dev_alloc(&h.rem_w, std::max<size_t>(4 * plan.rem_row_idx.size(), 16)))) {
        (void)hipStreamSynchronize(ctx->stream);
        hybrid_free(ctx, &h);
        return st;
    }
    // the finished operands start as zeros; packing the weights only ever writes the cells that hold an edge
    if (plan.n_tiles > 0) HIP_TRY(ctx, launch_zero_bytes(h.de_tiles.p, 2 * (size_t)plan.n_tiles * kDenseTileElems, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));  // the host vectors go out of scope below
    h.n_list_edges = (int64_t)plan.de_pos.size();
    h.n_tile_edges = (int64_t)plan.dt_addr.size();
    h.n_tiles = plan.n_tiles;
    h.n_chunks = (int64_t)plan.chunks.size();
    h.n_blocks = (int64_t)plan.blk_src_tile.size();
    h.n_dense_edges = plan.n_dense_edges;
    h.n_rem_edges = (int64_t)plan.rem_row_idx.size();
    h.n_items = (int64_t)wl.items.size();
    h.n_team = wl.n_team;
    h.n_heavy = (int64_t)wl.heavy.size();
    h.n_slots = wl.n_slots;
    h.weights_state = 0;
    h.usable = true;
    return SAGA_OK;
}

bool hybrid_applies(const saga_ctx* ctx, int32_t F, int64_t ld, const void* rows)
{
    return ctx->opt_dense_blocks && ctx->opt_fused && !ctx->opt_team && !ctx->opt_mma && F % 128 == 0 && ld % 8 == 0 &&
           (reinterpret_cast<uintptr_t>(rows) & 15u) == 0;
}

// The dense-block half of a bf16 sum propagation over `view` (the graph, or its edge order by source), whose plan
// ensure_hybrid has built. ga carries the rows (src, ld_src, F) and the partial rows; on return it reads the remainder's
// weights. The edge data in the two orders the kernels read them (block by block as two-part bf16, and in the
// remainder's edge order) are packed here: attached data (`w_attached`: w_src is the view's own copy, which
// saga_graph_set_edge_data invalidates) once, data passed with the call every call, COPY packs ones once.
// *forked: the kernel went to the context's second stream and the caller waits for ev_join after its own launch.
saga_status hybrid_dense_launch(saga_ctx* ctx, saga_graph* view, GatherArgs* ga, bool weighted, const float* w_src, bool w_attached,
                                saga_ctx::EventSet* es, bool* forked)
{
    hipStream_t s = ctx->stream;
    HybridDevice& h = view->hyb;
    *forked = false;
    const int want_state = !weighted ? 2 : (w_attached ? 1 : 0);
    if (want_state == 0 || h.weights_state != want_state) {
        PackArgs pa{};
        pa.w = w_src;
        pa.de_edge = static_cast<const int32_t*>(h.de_edge.p);
        pa.n_list = h.n_list_edges;
        pa.de_w = static_cast<uint32_t*>(h.de_w.p);
        pa.dt_edge = static_cast<const int32_t*>(h.dt_edge.p);
        pa.dt_addr = static_cast<const int32_t*>(h.dt_addr.p);
        pa.n_tile = h.n_tile_edges;
        pa.de_tiles = static_cast<uint16_t*>(h.de_tiles.p);
        pa.rem_edge = static_cast<const int32_t*>(h.rem_edge.p);
        pa.n_rem = weighted ? h.n_rem_edges : 0;
        pa.rem_w = static_cast<float*>(h.rem_w.p);
        HIP_TRY(ctx, launch_pack_hybrid_weights(pa, s));
        h.weights_state = want_state;
    }
    if (weighted) ga->edge_w = static_cast<const float*>(h.rem_w.p);
    DenseArgs da{};
    da.chunks = static_cast<const DenseChunk*>(h.chunks.p);
    da.n_chunks = h.n_chunks;
    da.blk_src_tile = static_cast<const int32_t*>(h.blk_src_tile.p);
    da.blk_e0 = static_cast<const int32_t*>(h.blk_e0.p);
    da.blk_tile = static_cast<const int32_t*>(h.blk_tile.p);
    da.de_tiles = static_cast<const uint16_t*>(h.de_tiles.p);
    da.de_pos = static_cast<const uint16_t*>(h.de_pos.p);
    da.de_w = static_cast<const uint32_t*>(h.de_w.p);
    da.src_tile_ids = static_cast<const int32_t*>(h.src_tile_ids.p);
    da.tile_row_slot0 = static_cast<const int32_t*>(h.tile_row_slot0.p);
    da.X = static_cast<const uint16_t*>(ga->src);
    da.ld = ga->ld_src;
    da.F = ga->F;
    da.use_low = weighted ? 1 : 0;
    da.partials = ga->partials;
    if (ctx->opt_dense_overlap && !ctx->arena_active) {
        if (!ctx->s_dense) {
            HIP_TRY(ctx, hipStreamCreateWithFlags(&ctx->s_dense, hipStreamNonBlocking));
            HIP_TRY(ctx, hipEventCreateWithFlags(&ctx->ev_fork, hipEventDisableTiming));
            HIP_TRY(ctx, hipEventCreateWithFlags(&ctx->ev_join, hipEventDisableTiming));
        }
        HIP_TRY(ctx, hipEventRecord(ctx->ev_fork, s));
        HIP_TRY(ctx, hipStreamWaitEvent(ctx->s_dense, ctx->ev_fork, 0));
        HIP_TRY(ctx, launch_dense_blocks(da, ctx->s_dense));
        HIP_TRY(ctx, hipEventRecord(ctx->ev_join, ctx->s_dense));
        *forked = true;
    } else {
        HIP_TRY(ctx, launch_dense_blocks(da, s));
        if (es) {
            HIP_TRY(ctx, hipEventRecord(es->ev_dense, s));
            es->has_dense = true;
        }
    }
    if (es) es->n_gather_launches = 2;
    return SAGA_OK;
}

// The per-vertex products of Section 3.2 are read through edges only: the source parts by an edge's source, the
// destination part by its destination. In a directed power-law graph many vertices are neither (R-MAT 20 with 32 edges
// per vertex: 38 % have no out-edge, 38 % no in-edge), so the graph keeps the two lists of vertices that are, and the
// products are taken over those rows. Built on the host at the first call that can use them.
saga_status ensure_endpoints(saga_ctx* ctx, saga_graph* g)
{
    if (g->endpoints_built || ctx->arena_active) return SAGA_OK;  // (a call that must not allocate uses them if they are there)
    const int64_t n = g->n;
    std::vector<int32_t> h_row, src_rows, dst_rows;
    try {
        h_row.resize((size_t)std::max<int64_t>(g->nnz, 1));
    } catch (...) {
        return ctx->fail(SAGA_ERR_INTERNAL, "out of host memory");
    }
    if (g->nnz > 0) {
        HIP_TRY(ctx, hipMemcpyAsync(h_row.data(), g->d_row_idx.p, sizeof(int32_t) * (size_t)g->nnz, hipMemcpyDeviceToHost, ctx->stream));
        HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    }
    try {
        std::vector<uint8_t> has_out((size_t)std::max<int64_t>(n, 1), 0);
        for (int64_t e = 0; e < g->nnz; ++e) has_out[(size_t)h_row[(size_t)e]] = 1;
        for (int64_t v = 0; v < n; ++v) {
            if (has_out[(size_t)v]) src_rows.push_back((int32_t)v);
            if (g->h_col_ptr[(size_t)v + 1] > g->h_col_ptr[(size_t)v]) dst_rows.push_back((int32_t)v);
        }
        g->n_src_rows = (int64_t)src_rows.size();
        g->n_dst_rows = (int64_t)dst_rows.size();
        for (std::vector<int32_t>* l : {&src_rows, &dst_rows})
            while (!l->empty() && l->size() % 64 != 0) l->push_back(l->back());
    } catch (...) {
        return ctx->fail(SAGA_ERR_INTERNAL, "out of host memory");
    }
    for (auto pr : {std::make_pair(&g->d_src_rows, &src_rows), std::make_pair(&g->d_dst_rows, &dst_rows)}) {
        if (saga_status st = ctx->dev_alloc(pr.first, sizeof(int32_t) * std::max<size_t>(pr.second->size(), 64))) return st;
        if (!pr.second->empty())
            HIP_TRY(ctx, hipMemcpyAsync(pr.first->p, pr.second->data(), sizeof(int32_t) * pr.second->size(), hipMemcpyHostToDevice, ctx->stream));
    }
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));  // the vectors go out of scope below
    g->endpoints_built = true;
    return SAGA_OK;
}

// The product `hg` over the graph's listed rows (sources or destinations): the arguments with the list in place if the list
// leaves out enough rows to pay for it and the product kernel takes lists for this shape, else unchanged (all hg.M rows).
static GemmArgs over_endpoints(const GemmArgs& hg, const saga_graph* g, bool source_side, bool* listed)
{
    *listed = false;
    if (!g || !g->endpoints_built) return hg;
    const int64_t rows = source_side ? g->n_src_rows : g->n_dst_rows;
    GemmArgs sub = hg;
    sub.row_ids = static_cast<const int32_t*>(source_side ? g->d_src_rows.p : g->d_dst_rows.p);
    sub.M = rows;
    if (rows * 8 > hg.M * 7 || !gemm_takes_row_list(sub)) return hg;
    *listed = true;
    return sub;
}

// Section 3.2: H = X [Wgs^T | Wm^T | Wgd^T] (+ [0 | 0 | b]) once per vertex, into ctx->ws_hoist (n x 3F fp32)
saga_status hoist_gated(saga_ctx* ctx, const saga_tensor* X, const saga_edge_params* ep, int64_t n, int32_t F, saga_graph* g)
{
    if (g)
        if (saga_status est = ensure_endpoints(ctx, g)) return est;
    hipStream_t s = ctx->stream;
    int64_t n_pad, k_pad;
    bt_padded_shape(3 * F, F, SAGA_F32, &n_pad, &k_pad);
    saga_status st;
    if ((st = ctx->dev_alloc(&ctx->ws_bt, sizeof(float) * (size_t)(n_pad * k_pad)))) return st;
    if ((st = ctx->dev_alloc(&ctx->ws_bias, sizeof(float) * (size_t)(3 * F)))) return st;
    if ((st = ctx->dev_alloc(&ctx->ws_hoist, sizeof(float) * (size_t)n * 3 * F))) return st;
    float* bt = static_cast<float*>(ctx->ws_bt.p);
    float* bias = static_cast<float*>(ctx->ws_bias.p);
    const float* Wg = static_cast<const float*>(ep->W_gate->data);
    HIP_TRY(ctx, launch_zero_bytes(bt, sizeof(float) * (size_t)(n_pad * k_pad), s));
    HIP_TRY(ctx, launch_zero_bytes(bias, sizeof(float) * (size_t)(3 * F), s));
    HIP_TRY(ctx, launch_pack_bt_rows(Wg, ep->W_gate->ld, 0, F, F, bt, k_pad, 0, s));
    HIP_TRY(ctx, launch_pack_bt_rows(ep->W_msg ? static_cast<const float*>(ep->W_msg->data) : nullptr,
                                     ep->W_msg ? ep->W_msg->ld : 0, 0, F, F, bt, k_pad, F, s));
    HIP_TRY(ctx, launch_pack_bt_rows(Wg, ep->W_gate->ld, F, F, F, bt, k_pad, 2 * (int64_t)F, s));
    if (ep->b_gate)
        HIP_TRY(ctx, hipMemcpyAsync(bias + 2 * F, ep->b_gate->data, sizeof(float) * (size_t)F, hipMemcpyDeviceToDevice, s));
    GemmArgs hg{};
    hg.A = X->data;
    hg.lda = X->ld;
    hg.Bt = bt;
    hg.ldbt = k_pad;
    hg.bias = bias;
    hg.C = ctx->ws_hoist.p;
    hg.ldc = 3 * (int64_t)F;
    hg.M = n;
    hg.N = 3 * F;
    hg.K = F;
    hg.dtype = hg.out_dtype = SAGA_F32;
    hg.act = SAGA_ACT_NONE;
    // [Ps | M] for the vertices with out-edges, Pd (+ b) for those with in-edges, as two products, where at least one of
    // them can go over a list (the product kernel that takes lists has K = 128: the packed weights then hold whole
    // 128-row groups for either product)
    GemmArgs src = hg, dst = hg;
    src.N = 2 * F;
    src.bias = nullptr;  // (its 2F entries are zeros)
    dst.N = F;
    dst.Bt = bt + 2 * (int64_t)F * k_pad;
    dst.bias = bias + 2 * F;
    dst.C = static_cast<float*>(ctx->ws_hoist.p) + 2 * F;
    bool src_listed = false, dst_listed = false;
    src = over_endpoints(src, g, true, &src_listed);
    dst = over_endpoints(dst, g, false, &dst_listed);
    if (src_listed || dst_listed) {
        HIP_TRY(ctx, launch_gemm(src, s));
        HIP_TRY(ctx, launch_gemm(dst, s));
        ctx->acc.n_hoist_row_cols = src.M * src.N + dst.M * dst.N;
        return SAGA_OK;
    }
    HIP_TRY(ctx, launch_gemm(hg, s));
    ctx->acc.n_hoist_row_cols = hg.M * hg.N;
    return SAGA_OK;
}

// Figure 11's ApplyEdge depends on the source only: H = sigmoid(X Wp^T + bp) once per vertex (Section 3.2),
// into ctx->ws_hoist (n x Fm fp32)
saga_status hoist_pool(saga_ctx* ctx, const saga_tensor* X, const saga_edge_params* ep, int64_t n, int32_t F, int32_t Fm, int32_t act,
                       saga_graph* g)
{
    if (g)
        if (saga_status est = ensure_endpoints(ctx, g)) return est;
    hipStream_t s = ctx->stream;
    int64_t n_pad, k_pad;
    bt_padded_shape(Fm, F, SAGA_F32, &n_pad, &k_pad);
    saga_status st;
    if ((st = ctx->dev_alloc(&ctx->ws_bt, sizeof(float) * (size_t)(n_pad * k_pad)))) return st;
    if ((st = ctx->dev_alloc(&ctx->ws_hoist, sizeof(float) * (size_t)n * Fm))) return st;
    float* bt = static_cast<float*>(ctx->ws_bt.p);
    HIP_TRY(ctx, launch_zero_bytes(bt, sizeof(float) * (size_t)(n_pad * k_pad), s));
    HIP_TRY(ctx, launch_pack_bt_rows(static_cast<const float*>(ep->W_pool->data), ep->W_pool->ld, 0, Fm, F, bt, k_pad, 0, s));
    GemmArgs hg{};
    hg.A = X->data;
    hg.lda = X->ld;
    hg.Bt = bt;
    hg.ldbt = k_pad;
    hg.bias = ep->b_pool ? static_cast<const float*>(ep->b_pool->data) : nullptr;
    hg.C = ctx->ws_hoist.p;
    hg.ldc = Fm;
    hg.M = n;
    hg.N = Fm;
    hg.K = F;
    hg.dtype = hg.out_dtype = SAGA_F32;
    hg.act = act;
    bool listed = false;
    hg = over_endpoints(hg, g, true, &listed);  // pooled rows are read through an edge's source
    HIP_TRY(ctx, launch_gemm(hg, s));
    ctx->acc.n_hoist_row_cols = hg.M * hg.N;
    return SAGA_OK;
}

saga_status VertexProducts::init(saga_ctx* c, const saga_tensor* x, const saga_edge_params* ep)
{
    ctx = c;
    X = x;
    F = (int32_t)x->cols;
    hipStream_t s = ctx->stream;
    const bool gated = ep->op == SAGA_EDGE_GATED;
    const int32_t n_rows = gated ? 3 * F : (int32_t)ep->W_pool->rows;
    int64_t n_pad;
    bt_padded_shape(n_rows, F, SAGA_F32, &n_pad, &k_pad);
    n_pad += 128;  // a product may start in the middle of the buffer (W_gd) and reads whole tiles of rows
    if (saga_status st = ctx->dev_alloc(&ctx->ws_prod, sizeof(float) * (size_t)(n_pad * k_pad))) return st;
    if (saga_status st = ctx->dev_alloc(&ctx->ws_bias, sizeof(float) * (size_t)n_rows)) return st;
    bt = static_cast<float*>(ctx->ws_prod.p);
    bias = static_cast<float*>(ctx->ws_bias.p);
    HIP_TRY(ctx, launch_zero_bytes(bt, sizeof(float) * (size_t)(n_pad * k_pad), s));
    HIP_TRY(ctx, launch_zero_bytes(bias, sizeof(float) * (size_t)n_rows, s));
    if (gated) {
        const float* Wg = static_cast<const float*>(ep->W_gate->data);
        HIP_TRY(ctx, launch_pack_bt_rows(Wg, ep->W_gate->ld, 0, F, F, bt, k_pad, 0, s));
        HIP_TRY(ctx, launch_pack_bt_rows(ep->W_msg ? static_cast<const float*>(ep->W_msg->data) : nullptr, ep->W_msg ? ep->W_msg->ld : 0, 0,
                                         F, F, bt, k_pad, F, s));
        HIP_TRY(ctx, launch_pack_bt_rows(Wg, ep->W_gate->ld, F, F, F, bt, k_pad, 2 * (int64_t)F, s));
        if (ep->b_gate)
            HIP_TRY(ctx, hipMemcpyAsync(bias + 2 * F, ep->b_gate->data, sizeof(float) * (size_t)F, hipMemcpyDeviceToDevice, s));
    } else {
        HIP_TRY(ctx, launch_pack_bt_rows(static_cast<const float*>(ep->W_pool->data), ep->W_pool->ld, 0, n_rows, F, bt, k_pad, 0, s));
        if (ep->b_pool) HIP_TRY(ctx, hipMemcpyAsync(bias, ep->b_pool->data, sizeof(float) * (size_t)n_rows, hipMemcpyDeviceToDevice, s));
    }
    HIP_TRY(ctx, hipStreamSynchronize(s));  // the products run on other streams of the schedule
    return SAGA_OK;
}

saga_status VertexProducts::rows(DevBuf* tmp, int64_t row0, int64_t n_rows, int32_t w0, int32_t n_cols, int32_t act, float* dst, int64_t ldc,
                                 hipStream_t on, int64_t* h2d) const
{
    if (saga_status e = ctx->dev_alloc(tmp, sizeof(float) * (size_t)n_rows * F)) return e;  // grows once: intervals do not grow
    HIP_TRY(ctx, hipMemcpy2DAsync(tmp->p, sizeof(float) * (size_t)F, static_cast<const float*>(X->data) + row0 * X->ld,
                                  sizeof(float) * (size_t)X->ld, sizeof(float) * (size_t)F, (size_t)n_rows, hipMemcpyHostToDevice, on));
    *h2d += n_rows * (int64_t)F * 4;
    GemmArgs hg{};
    hg.A = tmp->p;
    hg.lda = F;
    hg.Bt = bt + (int64_t)w0 * k_pad;
    hg.ldbt = k_pad;
    hg.bias = bias + w0;
    hg.C = dst;
    hg.ldc = ldc;
    hg.M = n_rows;
    hg.N = n_cols;
    hg.K = F;
    hg.dtype = hg.out_dtype = SAGA_F32;
    hg.act = act;
    hg.tiled_only = one_kernel ? 1 : 0;
    HIP_TRY(ctx, launch_gemm(hg, on));
    return SAGA_OK;
}

// A streamed layer of any of the four programs. Linear layers go straight to the chunk schedule. Layers whose ApplyEdge
// has a per-vertex part (Section 3.2) form those products on the device as the rows of X arrive: a source interval's
// rows of X are copied in and multiplied into the interval buffer ([Ps | M] of a gated layer, the pooled rows of a
// max-pooling one), and a gated layer's destination parts Pd_j are formed the same way from the destination
// interval's rows of X. The products therefore never cross the host link: it carries X once per destination
// interval, like in a linear layer, instead of the two to three times wider hoisted rows there and back.
static saga_status streamed_layer(saga_ctx* ctx, saga_graph* g, const saga_tensor* X, const saga_edge_params* ep, int32_t agg,
                                  const saga_vertex_params* vp, saga_tensor* Y, saga_tensor* accum_out)
{
    const int64_t n = g->n;
    const int32_t F = (int32_t)X->cols;
    const bool gated = ep->op == SAGA_EDGE_GATED, pool = ep->op == SAGA_EDGE_POOL;
    StreamExtras ex;
    bool use_ex = false;
    if (accum_out) {
        ex.accum_rows = static_cast<float*>(accum_out->data);
        ex.ld_accum = accum_out->ld;
        use_ex = true;
    }
    if (vp && vp->W_self) {
        ex.self_rows = static_cast<const float*>(X->data);
        ex.ld_self = X->ld;
        ex.F_self = F;
        use_ex = true;
    }
    if ((!gated && !pool) || n == 0) return streamed_forward(ctx, g, X, ep, agg, vp, Y, nullptr, use_ex ? &ex : nullptr);

    const int32_t Fh = gated ? 2 * F : (int32_t)ep->W_pool->rows;  // width of the rows that travel over the edges
    VertexProducts prod;
    prod.one_kernel = agg == SAGA_AGG_MAX;
    if (saga_status st = prod.init(ctx, X, ep)) return st;
    for (DevBuf* b : {&ctx->ws_accum, &ctx->ws_tile}) ctx->dev_free(b);  // sized per interval below
    VertexFeed feed;
    feed.bytes_per_row = sizeof(float) * (size_t)F;
    feed.fill = [&](int64_t row0, int64_t rows, float* dst, hipStream_t on, bool, int64_t* h2d) -> saga_status {
        return prod.rows(&ctx->ws_accum, row0, rows, 0, Fh, pool ? (int32_t)SAGA_ACT_SIGMOID : (int32_t)SAGA_ACT_NONE, dst, Fh, on, h2d);
    };
    saga_tensor hx{};  // shape of the rows that travel; the feed supplies them
    hx.data = nullptr;
    hx.rows = n;
    hx.cols = hx.ld = Fh;
    hx.dtype = SAGA_F32;
    hx.mem = SAGA_MEM_HOST;
    saga_edge_params e2 = *ep;
    if (pool) {  // the pooled rows are plain vertex data now
        e2.op = SAGA_EDGE_COPY;
    } else {     // rows [Ps | M] travel, the destination parts Pd of the resident interval are formed beside its accumulator
        ex.acc_width = F;
        ex.bytes_per_dst_row = sizeof(float) * (size_t)F;
        ex.dst_fill = [&](int64_t row0, int64_t rows, float* dst, hipStream_t on, int64_t* h2d) -> saga_status {
            return prod.rows(&ctx->ws_tile, row0, rows, 2 * F, F, SAGA_ACT_NONE, dst, F, on, h2d);
        };
        use_ex = true;
    }
    return streamed_forward(ctx, g, &hx, &e2, agg, vp, Y, &feed, use_ex ? &ex : nullptr);
}

// No C++ exception may leave an extern "C" entry point: whatever the layer code throws (host memory for a work list,
// a tiling, a vector of counts) becomes SAGA_ERR_INTERNAL, after everything the call enqueued has been waited for.
template <typename Fn>
static saga_status guarded(saga_ctx* ctx, Fn&& fn)
{
    try {
        return fn();
    } catch (const std::exception& e) {
        chunk_grid_drain(ctx);
        return ctx->fail(SAGA_ERR_INTERNAL, "%s", e.what());
    } catch (...) {
        chunk_grid_drain(ctx);
        return ctx->fail(SAGA_ERR_INTERNAL, "unknown exception");
    }
}

extern "C" {

const char* saga_version(void) { return kVersion; }

saga_status saga_plan_work_list(int64_t n, const int64_t* col_ptr, const int32_t* row_idx, int64_t min_edges,
                                int64_t cut_degree, int64_t stripe_rows, int32_t team, int32_t* items_out, int64_t capacity,
                                int64_t* n_items, int64_t* n_team_items, int64_t* n_split_vertices, int64_t* n_slots)
{
    if (n < 0 || !col_ptr || min_edges < 1 || cut_degree < 0 || stripe_rows < 0 || capacity < 0 || (team != 1 && team != 4))
        return SAGA_ERR_INVALID_ARG;
    if (col_ptr[n] > 0 && !row_idx) return SAGA_ERR_INVALID_ARG;
    WorkList wl;
    try {
        build_work_list(col_ptr, row_idx, n, WorkListParams{min_edges, cut_degree, stripe_rows, false, team}, &wl);
    } catch (...) {
        return SAGA_ERR_INTERNAL;
    }
    if (n_items) *n_items = (int64_t)wl.items.size();
    if (n_team_items) *n_team_items = wl.n_team;
    if (n_split_vertices) *n_split_vertices = (int64_t)wl.heavy.size();
    if (n_slots) *n_slots = wl.n_slots;
    if (items_out) {
        const int64_t m = std::min<int64_t>(capacity, (int64_t)wl.items.size());
        memcpy(items_out, wl.items.data(), sizeof(WorkItem) * (size_t)m);
    }
    return SAGA_OK;
}

saga_status saga_plan_dense_blocks(int64_t n, const int64_t* col_ptr, const int32_t* row_idx, int64_t min_block_edges, int64_t min_tile_gain,
                                   int32_t max_chunk_blocks, int64_t* counts, int32_t* chunks_out, int64_t chunk_capacity, int32_t* block_edges_out,
                                   int64_t block_capacity, int32_t* remainder_row_idx_out, int32_t* remainder_edge_out, int64_t* remainder_col_ptr_out,
                                   int32_t* dense_edge_out, int32_t* dense_block_of_edge_out)
{
    if (n < 0 || !col_ptr || !counts || min_block_edges < 1 || min_tile_gain < 0 || max_chunk_blocks < 1) return SAGA_ERR_INVALID_ARG;
    if (col_ptr[n] > 0 && !row_idx) return SAGA_ERR_INVALID_ARG;
    try {
        HybridPlan plan;
        HybridParams hp;
        hp.min_block_edges = min_block_edges;
        hp.min_tile_gain = min_tile_gain;
        hp.max_chunk_blocks = max_chunk_blocks;
        build_hybrid_plan(col_ptr, row_idx, n, hp, &plan);
        counts[0] = (int64_t)plan.chunks.size();
        counts[1] = (int64_t)plan.blk_src_tile.size();
        counts[2] = plan.n_dense_edges;
        counts[3] = (int64_t)plan.rem_row_idx.size();
        if (chunks_out) memcpy(chunks_out, plan.chunks.data(), sizeof(DenseChunk) * (size_t)std::min<int64_t>(chunk_capacity, counts[0]));
        if (block_edges_out)
            for (int64_t b = 0; b < std::min<int64_t>(block_capacity, counts[1]); ++b)
                block_edges_out[b] = plan.blk_tile[(size_t)b] >= 0 ? -1 : plan.blk_e0[(size_t)b + 1] - plan.blk_e0[(size_t)b];
        if (remainder_row_idx_out && counts[3] > 0) memcpy(remainder_row_idx_out, plan.rem_row_idx.data(), 4 * (size_t)counts[3]);
        if (remainder_edge_out && counts[3] > 0) memcpy(remainder_edge_out, plan.rem_edge.data(), 4 * (size_t)counts[3]);
        if (remainder_col_ptr_out) memcpy(remainder_col_ptr_out, plan.rem_col_ptr.data(), 8 * ((size_t)n + 1));
        if (dense_edge_out) {  // list edges first, then the edges of the finished operands
            if (!plan.de_edge.empty()) memcpy(dense_edge_out, plan.de_edge.data(), 4 * plan.de_edge.size());
            if (!plan.dt_edge.empty()) memcpy(dense_edge_out + plan.de_edge.size(), plan.dt_edge.data(), 4 * plan.dt_edge.size());
        }
        if (dense_block_of_edge_out) {
            for (int64_t b = 0; b < counts[1]; ++b)
                for (int32_t e = plan.blk_e0[(size_t)b]; e < plan.blk_e0[(size_t)b + 1]; ++e) dense_block_of_edge_out[e] = (int32_t)b;
            std::vector<int32_t> block_of_tile((size_t)plan.n_tiles, -1);
            for (int64_t b = 0; b < counts[1]; ++b)
                if (plan.blk_tile[(size_t)b] >= 0) block_of_tile[(size_t)plan.blk_tile[(size_t)b]] = (int32_t)b;
            for (size_t i = 0; i < plan.dt_addr.size(); ++i)
                dense_block_of_edge_out[plan.de_edge.size() + i] = block_of_tile[(size_t)(plan.dt_addr[i] / kDenseTileElems)];
        }
    } catch (...) {
        return SAGA_ERR_INTERNAL;
    }
    return SAGA_OK;
}

saga_status saga_plan_reencoding(int64_t n, const int64_t* col_ptr, const int32_t* row_idx, int32_t Q, int32_t P, uint64_t seed,
                                 int32_t* new_id, int64_t* before, int64_t* after)
{
    if (n < 1 || n > 0x7fffffffLL - 1 || !col_ptr || !new_id || Q < 1 || P < Q || P > n) return SAGA_ERR_INVALID_ARG;
    const int64_t nnz = col_ptr[n];
    if (nnz > 0 && !row_idx) return SAGA_ERR_INVALID_ARG;
    try {
        // rank by total degree, ties by a hash of (seed, id)
        std::vector<int64_t> deg((size_t)n, 0);
        for (int64_t v = 0; v < n; ++v) {
            deg[(size_t)v] += col_ptr[v + 1] - col_ptr[v];
            for (int64_t e = col_ptr[v]; e < col_ptr[v + 1]; ++e) {
                if (row_idx[e] < 0 || row_idx[e] >= n) return SAGA_ERR_BAD_GRAPH;
                ++deg[(size_t)row_idx[e]];
            }
        }
        auto mix = [](uint64_t x) {
            x += 0x9e3779b97f4a7c15ULL;
            x = (x ^ (x >> 30)) * 0xbf58476d1ce4e5b9ULL;
            x = (x ^ (x >> 27)) * 0x94d049bb133111ebULL;
            return x ^ (x >> 31);
        };
        std::vector<int32_t> order((size_t)n);
        for (int64_t v = 0; v < n; ++v) order[(size_t)v] = (int32_t)v;
        std::sort(order.begin(), order.end(), [&](int32_t a, int32_t b) {
            if (deg[(size_t)a] != deg[(size_t)b]) return deg[(size_t)a] > deg[(size_t)b];
            const uint64_t ha = mix(seed ^ mix((uint64_t)a)), hb = mix(seed ^ mix((uint64_t)b));
            return ha != hb ? ha < hb : a < b;
        });
        // deal to the P intervals of ceil(n / P) ids, forwards and backwards in turn, skipping full ones
        const int64_t Sp = (n + P - 1) / P;
        std::vector<int64_t> fill((size_t)P, 0);
        auto cap = [&](int64_t g) { return std::max<int64_t>(0, std::min<int64_t>(Sp, n - g * Sp)); };
        int64_t r = 0;
        for (int64_t round = 0; r < n; ++round) {
            for (int64_t k = 0; k < P && r < n; ++k) {
                const int64_t g = (round & 1) ? P - 1 - k : k;
                if (fill[(size_t)g] >= cap(g)) continue;
                new_id[(size_t)order[(size_t)r++]] = (int32_t)(g * Sp + fill[(size_t)g]++);
            }
        }
        // chunk edge counts of the tiling, before and after
        const int64_t Dq = (n + Q - 1) / Q;
        for (int pass = 0; pass < 2; ++pass) {
            int64_t* res = pass == 0 ? before : after;
            if (!res) continue;
            std::vector<int64_t> cnt((size_t)Q * P, 0);
            for (int64_t v = 0; v < n; ++v) {
                const int64_t j = (pass == 0 ? v : (int64_t)new_id[(size_t)v]) / Dq;
                for (int64_t e = col_ptr[v]; e < col_ptr[v + 1]; ++e) {
                    const int64_t u = row_idx[e];
                    ++cnt[(size_t)(j * P + (pass == 0 ? u : (int64_t)new_id[(size_t)u]) / Sp)];
                }
            }
            res[0] = *std::max_element(cnt.begin(), cnt.end());
            res[1] = *std::min_element(cnt.begin(), cnt.end());
            res[2] = (int64_t)cnt.size();
        }
    } catch (...) {
        return SAGA_ERR_INTERNAL;
    }
    return SAGA_OK;
}

saga_status saga_create(saga_ctx** out, int device, void* hip_stream, size_t hbm_budget_bytes)
{
    if (!out) return SAGA_ERR_INVALID_ARG;
    *out = nullptr;
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || device < 0 || device >= count) {
        (void)hipGetLastError();
        return SAGA_ERR_HIP;
    }
    saga_ctx* c = new (std::nothrow) saga_ctx();
    if (!c) return SAGA_ERR_INTERNAL;
    c->device = device;
    c->budget = hbm_budget_bytes;
    DeviceGuard guard(device);
    if (hip_stream) {
        c->stream = static_cast<hipStream_t>(hip_stream);
    } else {
        if (hipStreamCreateWithFlags(&c->stream, hipStreamNonBlocking) != hipSuccess) {
            delete c;
            return SAGA_ERR_HIP;
        }
        c->own_stream = true;
    }
    // the static scratch array has its own copy, at its own address, on every GPU: ask for this device's, with this device current
    void* sp = nullptr;
    if (hipGetSymbolAddress(&sp, HIP_SYMBOL(scratch)) != hipSuccess || !sp) {
        (void)hipGetLastError();
        if (c->own_stream) (void)hipStreamDestroy(c->stream);
        delete c;
        return SAGA_ERR_HIP;
    }
    c->scratch_ptr = static_cast<unsigned char*>(sp);
    *out = c;
    return SAGA_OK;
}

saga_status saga_destroy(saga_ctx* ctx)
{
    if (!ctx) return SAGA_ERR_INVALID_ARG;
    DeviceGuard guard(ctx->device);
    (void)hipStreamSynchronize(ctx->stream);
    for (DevBuf* b : {&ctx->ws_accum, &ctx->ws_accum16, &ctx->ws_partials, &ctx->ws_hoist, &ctx->ws_bt, &ctx->ws_bias,
                      &ctx->ws_flag, &ctx->ws_dz, &ctx->ws_grad, &ctx->ws_splitk, &ctx->ws_edge_t, &ctx->ws_dh, &ctx->ws_dz16, &ctx->ws_wt, &ctx->ws_tile, &ctx->ws_edge_msg, &ctx->ws_prod, &ctx->st_A, &ctx->st_V[0], &ctx->st_V[1],
                      &ctx->st_C[0], &ctx->st_C[1], &ctx->st_Y[0], &ctx->st_Y[1], &ctx->st_partials, &ctx->st_D, &ctx->st_S[0],
                      &ctx->st_S[1]})
        ctx->dev_free(b);
    if (ctx->h_grad) (void)hipHostFree(ctx->h_grad);
    ctx->destroy_stream_set();
    if (ctx->ev_fork) (void)hipEventDestroy(ctx->ev_fork);
    if (ctx->ev_join) (void)hipEventDestroy(ctx->ev_join);
    if (ctx->s_dense) (void)hipStreamDestroy(ctx->s_dense);
    for (auto& es : ctx->ev_pool) {
        for (auto& e : es.ev) (void)hipEventDestroy(e);
        (void)hipEventDestroy(es.ev_dense);
    }
    if (ctx->own_stream) (void)hipStreamDestroy(ctx->stream);
    delete ctx;
    return SAGA_OK;
}

const char* saga_last_error(const saga_ctx* ctx) { return ctx ? ctx->err.c_str() : "null context"; }
size_t saga_peak_device_bytes(const saga_ctx* ctx) { return ctx ? ctx->peak_bytes : 0; }

saga_status saga_set_option(saga_ctx* ctx, const char* name, int64_t value)
{
    if (!ctx || !name) return SAGA_ERR_INVALID_ARG;
    if (!strcmp(name, "split")) {
        if (value < 16 || value > (1 << 24)) return ctx->fail(SAGA_ERR_INVALID_ARG, "split must be in [16, 2^24]");
        ctx->opt_split = value;
        ctx->opt_split_set = true;
    } else if (!strcmp(name, "cut_degree")) {
        if (value < 0 || value > (1LL << 31)) return ctx->fail(SAGA_ERR_INVALID_ARG, "cut_degree must be in [0, 2^31]");
        ctx->opt_cut_degree = value;
    } else if (!strcmp(name, "stripe_kb")) {
        if (value < 0 || value > (1 << 22)) return ctx->fail(SAGA_ERR_INVALID_ARG, "stripe_kb must be in [0, 2^22]");
        ctx->opt_stripe_kb = value;
        ctx->opt_stripe_set = true;
    } else if (!strcmp(name, "piece_order")) {
        if (value != 0 && value != 1) return ctx->fail(SAGA_ERR_INVALID_ARG, "piece_order must be 0 or 1");
        ctx->opt_piece_order = (int)value;
    } else if (!strcmp(name, "team")) {
        if (value != 0 && value != 1) return ctx->fail(SAGA_ERR_INVALID_ARG, "team must be 0 or 1");
        ctx->opt_team = (int)value;
    } else if (!strcmp(name, "mma")) {
        if (value != 0 && value != 1) return ctx->fail(SAGA_ERR_INVALID_ARG, "mma must be 0 or 1");
        ctx->opt_mma = (int)value;
    } else if (!strcmp(name, "xcd_remap")) {
        if (value != 0 && value != 1) return ctx->fail(SAGA_ERR_INVALID_ARG, "xcd_remap must be 0 or 1");
        ctx->opt_xcd_remap = (int)value;
    } else if (!strcmp(name, "dst_intervals")) {
        if (value < 0 || value > 4096) return ctx->fail(SAGA_ERR_INVALID_ARG, "dst_intervals must be in [0, 4096]");
        ctx->opt_dst_intervals = (int)value;
    } else if (!strcmp(name, "schedule")) {
        if (value < 0 || value > 2) return ctx->fail(SAGA_ERR_INVALID_ARG, "schedule must be 0, 1 or 2");
        ctx->opt_schedule = (int)value;
    } else if (!strcmp(name, "overlap")) {
        if (value != 0 && value != 1) return ctx->fail(SAGA_ERR_INVALID_ARG, "overlap must be 0 or 1");
        ctx->opt_overlap = (int)value;
    } else if (!strcmp(name, "bwd_tile_rows")) {
        if (value < 0 || value > (1LL << 31)) return ctx->fail(SAGA_ERR_INVALID_ARG, "bwd_tile_rows must be in [0, 2^31]");
        ctx->opt_bwd_tile_rows = value;
    } else if (!strcmp(name, "dense_blocks")) {
        if (value != 0 && value != 1) return ctx->fail(SAGA_ERR_INVALID_ARG, "dense_blocks must be 0 or 1");
        ctx->opt_dense_blocks = (int)value;
    } else if (!strcmp(name, "dense_overlap")) {
        if (value != 0 && value != 1) return ctx->fail(SAGA_ERR_INVALID_ARG, "dense_overlap must be 0 or 1");
        ctx->opt_dense_overlap = (int)value;
    } else if (!strcmp(name, "dense_min_edges")) {
        if (value < 0 || value > kDenseM * kDenseK) return ctx->fail(SAGA_ERR_INVALID_ARG, "dense_min_edges must be in [0, 2048]");
        ctx->opt_dense_min_edges = value;
    } else if (!strcmp(name, "dense_tile_gain")) {
        if (value < -1 || value > (1LL << 40)) return ctx->fail(SAGA_ERR_INVALID_ARG, "dense_tile_gain must be in [-1, 2^40]");
        ctx->opt_dense_tile_gain = value;
    } else if (!strcmp(name, "dense_chunk")) {
        if (value < 0 || value > (1 << 20)) return ctx->fail(SAGA_ERR_INVALID_ARG, "dense_chunk must be in [0, 2^20]");
        ctx->opt_dense_chunk = value;
    } else if (!strcmp(name, "fused")) {
        if (value != 0 && value != 1) return ctx->fail(SAGA_ERR_INVALID_ARG, "fused must be 0 or 1");
        ctx->opt_fused = (int)value;
    } else if (!strcmp(name, "transform_first")) {
        if (value != 0 && value != 1) return ctx->fail(SAGA_ERR_INVALID_ARG, "transform_first must be 0 or 1");
        ctx->opt_transform_first = (int)value;
    } else if (!strcmp(name, "src_intervals")) {
        if (value < 0 || value > 4096) return ctx->fail(SAGA_ERR_INVALID_ARG, "src_intervals must be in [0, 4096]");
        ctx->opt_src_intervals = (int)value;
    } else {
        return ctx->fail(SAGA_ERR_INVALID_ARG, "unknown option '%s'", name);
    }
    return SAGA_OK;
}

saga_status saga_copy_bytes(saga_ctx* ctx, void* dst, const void* src, size_t bytes)
{
    if (!ctx) return SAGA_ERR_INVALID_ARG;
    if (!dst || !src) return ctx->fail(SAGA_ERR_INVALID_ARG, "null pointer");
    DeviceGuard guard(ctx->device);
    hipError_t e = launch_copy_bytes(dst, src, bytes, ctx->stream);
    if (e == hipErrorInvalidValue) return ctx->fail(SAGA_ERR_INVALID_ARG, "copy needs 16-byte aligned pointers and size");
    if (e != hipSuccess) return ctx->fail(SAGA_ERR_HIP, "copy kernel: %s", hipGetErrorString(e));
    return SAGA_OK;
}

saga_status saga_set_profiling(saga_ctx* ctx, int32_t on)
{
    if (!ctx) return SAGA_ERR_INVALID_ARG;
    DeviceGuard guard(ctx->device);
    if (saga_status st = ctx->drain_events()) return st;
    ctx->profiling = on != 0;
    return SAGA_OK;
}

saga_status saga_reset_timings(saga_ctx* ctx)
{
    if (!ctx) return SAGA_ERR_INVALID_ARG;
    DeviceGuard guard(ctx->device);
    if (saga_status st = ctx->drain_events()) return st;
    const saga_timings keep = ctx->acc;
    ctx->acc = saga_timings{};
    ctx->acc.n_work_items = keep.n_work_items;
    ctx->acc.n_split_vertices = keep.n_split_vertices;
    ctx->acc.n_dense_blocks = keep.n_dense_blocks;
    ctx->acc.n_dense_edges = keep.n_dense_edges;
    ctx->acc.n_partial_rows = keep.n_partial_rows;
    ctx->acc.n_hoist_row_cols = keep.n_hoist_row_cols;
    return SAGA_OK;
}

saga_status saga_get_timings(saga_ctx* ctx, saga_timings* out)
{
    if (!ctx || !out) return SAGA_ERR_INVALID_ARG;
    DeviceGuard guard(ctx->device);
    if (saga_status st = ctx->drain_events()) return st;
    *out = ctx->acc;
    return SAGA_OK;
}

// ---------------------------------------------------------------------------
// graph ingest
// ---------------------------------------------------------------------------
saga_status saga_graph_create_csc(saga_ctx* ctx, int64_t n, int64_t nnz, const int64_t* col_ptr, const int32_t* row_idx,
                                  int32_t where, saga_graph** out)
{
    if (!ctx) return SAGA_ERR_INVALID_ARG;
    if (!out) return ctx->fail(SAGA_ERR_INVALID_ARG, "out is null");
    *out = nullptr;
    if (n < 0 || nnz < 0 || !col_ptr || (nnz > 0 && !row_idx))
        return ctx->fail(SAGA_ERR_INVALID_ARG, "null array or negative size");
    if (where != SAGA_MEM_DEVICE && where != SAGA_MEM_HOST) return ctx->fail(SAGA_ERR_INVALID_ARG, "bad placement");
    if (n > 0x7fffffffLL - 1 || nnz > 0x7fffffffLL - 64)
        return ctx->fail(SAGA_ERR_UNSUPPORTED, "graph too large for 32-bit vertex ids / edge offsets");
    DeviceGuard guard(ctx->device);

    saga_graph* g = new (std::nothrow) saga_graph();
    if (!g) return ctx->fail(SAGA_ERR_INTERNAL, "out of host memory");
    g->ctx = ctx;
    g->n = n;
    g->nnz = nnz;
    g->where = where;
    auto bail = [&](saga_status st) {
        saga_graph_destroy(g);
        return st;
    };

    // column pointers are always examined on the host
    try {
        g->h_col_ptr.resize((size_t)n + 1);
    } catch (...) {
        return bail(ctx->fail(SAGA_ERR_INTERNAL, "out of host memory"));
    }
    if (where == SAGA_MEM_DEVICE) {
        hipError_t e = hipMemcpyAsync(g->h_col_ptr.data(), col_ptr, sizeof(int64_t) * ((size_t)n + 1), hipMemcpyDeviceToHost,
                                      ctx->stream);
        if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
        if (e != hipSuccess) return bail(ctx->fail(SAGA_ERR_HIP, "copying col_ptr: %s", hipGetErrorString(e)));
    } else {
        memcpy(g->h_col_ptr.data(), col_ptr, sizeof(int64_t) * ((size_t)n + 1));
    }
    const int64_t* cp = g->h_col_ptr.data();
    if (cp[0] != 0) return bail(ctx->fail(SAGA_ERR_BAD_GRAPH, "col_ptr[0] = %lld, expected 0", (long long)cp[0]));
    for (int64_t v = 0; v < n; ++v)
        if (cp[v + 1] < cp[v])
            return bail(ctx->fail(SAGA_ERR_BAD_GRAPH, "col_ptr decreases at vertex %lld", (long long)v));
    if (cp[n] != nnz)
        return bail(ctx->fail(SAGA_ERR_BAD_GRAPH, "col_ptr[n] = %lld but n_edges = %lld", (long long)cp[n], (long long)nnz));

    if (where == SAGA_MEM_HOST) {
        // streamed graphs stay on the host; validate the ids here
        try {
            g->h_row_idx.assign(row_idx, row_idx + nnz);
        } catch (...) {
            return bail(ctx->fail(SAGA_ERR_INTERNAL, "out of host memory"));
        }
        for (int64_t v = 0; v < n; ++v) {
            for (int64_t e = cp[v]; e < cp[v + 1]; ++e) {
                const int32_t u = row_idx[e];
                if (u < 0 || u >= n)
                    return bail(ctx->fail(SAGA_ERR_BAD_GRAPH, "source id %d out of range at edge %lld", u, (long long)e));
                if (e > cp[v] && row_idx[e - 1] >= u)
                    return bail(ctx->fail(SAGA_ERR_BAD_GRAPH, "column %lld is not strictly ascending at edge %lld",
                                          (long long)v, (long long)e));
            }
        }
        int64_t maxdeg = 0;
        for (int64_t v = 0; v < n; ++v) maxdeg = std::max(maxdeg, cp[v + 1] - cp[v]);
        g->max_degree = maxdeg;
        *out = g;
        return SAGA_OK;
    }

    int64_t maxdeg = 0;
    for (int64_t v = 0; v < n; ++v) maxdeg = std::max(maxdeg, cp[v + 1] - cp[v]);
    g->max_degree = maxdeg;
    saga_status st;
    if ((st = ctx->dev_alloc(&g->d_row_idx, sizeof(int32_t) * (size_t)std::max<int64_t>(nnz, 1)))) return bail(st);
    if ((st = ctx->dev_alloc(&ctx->ws_flag, 256))) return bail(st);
    hipError_t e = hipSuccess;
    if (nnz > 0) e = hipMemcpyAsync(g->d_row_idx.p, row_idx, sizeof(int32_t) * (size_t)nnz, hipMemcpyDeviceToDevice, ctx->stream);
    if (e == hipSuccess) e = launch_zero_bytes(ctx->ws_flag.p, 256, ctx->stream);
    if (e == hipSuccess)
        e = launch_validate_columns(col_ptr, n, static_cast<const int32_t*>(g->d_row_idx.p), n,
                                    static_cast<int32_t*>(ctx->ws_flag.p), ctx->stream);
    int32_t flag = 0;
    if (e == hipSuccess) e = hipMemcpyAsync(&flag, ctx->ws_flag.p, sizeof flag, hipMemcpyDeviceToHost, ctx->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
    if (e != hipSuccess) return bail(ctx->fail(SAGA_ERR_HIP, "graph upload: %s", hipGetErrorString(e)));
    if (flag) return bail(ctx->fail(SAGA_ERR_BAD_GRAPH, "row_idx has an id out of range or a column that is not strictly ascending"));
    *out = g;
    return SAGA_OK;
}

saga_status saga_graph_destroy(saga_graph* g)
{
    if (!g) return SAGA_ERR_INVALID_ARG;
    saga_ctx* ctx = g->ctx;
    DeviceGuard guard(ctx->device);
    (void)hipStreamSynchronize(ctx->stream);
    for (DevBuf* b : {&g->d_row_idx, &g->d_items, &g->d_heavy, &g->d_edge_data, &g->d_src_rows, &g->d_dst_rows}) ctx->dev_free(b);
    for (auto& sl : g->saved_lists) {
        ctx->dev_free(&sl.items);
        ctx->dev_free(&sl.heavy);
    }
    hybrid_free(ctx, &g->hyb);
    if (g->grid) chunk_grid_destroy(ctx, g->grid);
    transposed_graph_destroy(ctx, g);
    delete g;
    return SAGA_OK;
}

saga_status saga_graph_set_edge_data(saga_graph* g, const float* w)
{
    if (!g) return SAGA_ERR_INVALID_ARG;
    saga_ctx* ctx = g->ctx;
    if (!w && g->nnz > 0) return ctx->fail(SAGA_ERR_INVALID_ARG, "edge_weight is null");
    DeviceGuard guard(ctx->device);
    if (g->where == SAGA_MEM_HOST) {
        try {
            g->h_edge_data.assign(w, w + g->nnz);
        } catch (...) {
            return ctx->fail(SAGA_ERR_INTERNAL, "out of host memory");
        }
        // A tiling that exists keeps its structure: only the weights inside its pinned payloads are written again (no
        // streamed call is in flight: each one synchronises its streams before it returns). The same for the edge
        // order by source and its tiling.
        return guarded(ctx, [&] {
            chunk_grid_refresh_weights(g);
            return transposed_host_refresh_weights(ctx, g);
        });
    }
    g->tr_edge_data_valid = false;
    if (g->hyb.weights_state == 1) g->hyb.weights_state = 0;  // the dense-block form packs the new data at its next call
    if (g->tr && g->tr->hyb.weights_state == 1) g->tr->hyb.weights_state = 0;
    if (saga_status st = ctx->dev_alloc(&g->d_edge_data, sizeof(float) * (size_t)std::max<int64_t>(g->nnz, 1))) return st;
    if (g->nnz > 0) {
        HIP_TRY(ctx, hipMemcpyAsync(g->d_edge_data.p, w, sizeof(float) * (size_t)g->nnz, hipMemcpyDeviceToDevice, ctx->stream));
        HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    }
    return SAGA_OK;
}

saga_status saga_graph_info(const saga_graph* g, int64_t* max_in_degree, int64_t* n_work_items, int64_t* n_split_vertices)
{
    if (!g) return SAGA_ERR_INVALID_ARG;
    if (max_in_degree) *max_in_degree = g->max_degree;
    if (n_work_items) *n_work_items = g->n_items;
    if (n_split_vertices) *n_split_vertices = g->n_heavy;
    return SAGA_OK;
}

// ---------------------------------------------------------------------------
// one layer, everything resident in HBM
// ---------------------------------------------------------------------------
static saga_status resident_forward(saga_ctx* ctx, saga_graph* g, const saga_tensor* X, const saga_edge_params* ep,
                                    int32_t agg, const saga_vertex_params* vp, saga_tensor* Y, saga_tensor* accum_out)
{
    const int64_t n = g->n;
    const int32_t F = (int32_t)X->cols;
    const bool pool = ep->op == SAGA_EDGE_POOL;
    const int32_t Fm = pool ? (int32_t)ep->W_pool->rows : F;  // message width
    const bool bf16 = X->dtype == SAGA_BF16;
    const bool has_w = vp && vp->W;
    hipStream_t s = ctx->stream;
    // Transform first (option): for a linear ApplyEdge under the sum accumulator, W (.) sum_e w_e x_u = sum_e w_e (W (.) x_u),
    // so when the layer narrows the rows the product runs first and the propagation moves F_out values per edge
    // instead of F_in. The Gather output of the paper's order then never exists, so accum_out keeps the usual order.
    const bool tf = ctx->opt_transform_first && has_w && !vp->W_self && !accum_out && agg == SAGA_AGG_SUM &&
                    (ep->op == SAGA_EDGE_COPY || ep->op == SAGA_EDGE_MUL_WEIGHT) && vp->W->cols < F;
    const int32_t Fo_tf = tf ? (int32_t)vp->W->cols : 0;
    // bytes one edge gathers: the source row, or two hoisted fp32 rows when gated
    const int64_t row_bytes = ep->op == SAGA_EDGE_GATED ? 2 * (int64_t)F * 4 : (int64_t)(tf ? Fo_tf : Fm) * (bf16 ? 2 : 4);
    // bf16 rows summed over linear messages: the well-filled blocks of the adjacency matrix go to the matrix cores, the
    // sparse kernel keeps the remainder (rows of a multiple of 128 features, 16-byte aligned: what the dense kernel loads)
    const int32_t Fg = tf ? Fo_tf : Fm;  // width of the rows the propagation moves
    const int64_t ld_g = tf ? (int64_t)Fo_tf : X->ld;
    bool hybrid = bf16 && agg == SAGA_AGG_SUM && (ep->op == SAGA_EDGE_COPY || ep->op == SAGA_EDGE_MUL_WEIGHT) &&
                  hybrid_applies(ctx, Fg, ld_g, tf ? nullptr : X->data);
    if (hybrid) {
        if (saga_status st = ensure_hybrid(ctx, g, row_bytes, Fg)) return st;
        hybrid = g->hyb.usable;
    }
    if (!hybrid)
        if (saga_status st = ensure_work_list(ctx, g, row_bytes, Fg)) return st;

    saga_ctx::EventSet* es = nullptr;
    if (ctx->profiling && !ctx->arena_active) {
        if (ctx->ev_used == ctx->ev_pool.size()) {
            if (ctx->ev_pool.size() >= 512) {
                if (saga_status st = ctx->drain_events()) return st;
            } else {
                saga_ctx::EventSet ne{};
                for (auto& e : ne.ev) HIP_TRY(ctx, hipEventCreate(&e));
                HIP_TRY(ctx, hipEventCreate(&ne.ev_dense));
                ctx->ev_pool.push_back(ne);
            }
        }
        es = &ctx->ev_pool[ctx->ev_used];
        es->has_hoist = es->has_combine = es->has_apply = es->has_dense = false;
        es->n_gather_launches = 1;
        HIP_TRY(ctx, hipEventRecord(es->ev[0], s));
    }

    GatherArgs ga{};
    ga.items = static_cast<const WorkItem*>(hybrid ? g->hyb.items.p : g->d_items.p);
    ga.n_items = hybrid ? g->hyb.n_items : g->n_items;
    ga.n_team = hybrid ? g->hyb.n_team : g->n_team;
    ga.row_idx = static_cast<const int32_t*>(hybrid ? g->hyb.rem_row_idx.p : g->d_row_idx.p);
    const int64_t n_slots = hybrid ? g->hyb.n_slots : g->n_slots;
    const int64_t n_heavy = hybrid ? g->hyb.n_heavy : g->n_heavy;
    const HeavyVertex* heavy = static_cast<const HeavyVertex*>(hybrid ? g->hyb.heavy.p : g->d_heavy.p);
    ga.F = Fm;
    ga.agg = agg;
    ga.op = pool ? (int32_t)SAGA_EDGE_COPY : ep->op;
    ga.xcd_remap = ctx->opt_xcd_remap;
    ga.mma = ctx->opt_mma;
    ga.accumulate = 0;

    if (ep->op == SAGA_EDGE_GATED) {
        if (saga_status st = hoist_gated(ctx, X, ep, n, F, g)) return st;
        ga.src = ctx->ws_hoist.p;
        ga.ld_src = 3 * (int64_t)F;
        ga.src2 = static_cast<const float*>(ctx->ws_hoist.p) + F;
        ga.ld_src2 = 3 * (int64_t)F;
        ga.dst = static_cast<const float*>(ctx->ws_hoist.p) + 2 * F;
        ga.ld_dst = 3 * (int64_t)F;
        ga.dtype = SAGA_F32;
        if (es) es->has_hoist = true;
    } else if (pool) {
        // then the propagation kernel gathers rows of H
        if (saga_status st = hoist_pool(ctx, X, ep, n, F, Fm, SAGA_ACT_SIGMOID, g)) return st;
        ga.src = ctx->ws_hoist.p;
        ga.ld_src = Fm;
        ga.dtype = SAGA_F32;
        if (es) es->has_hoist = true;
    } else {
        ga.src = X->data;
        ga.ld_src = X->ld;
        ga.dtype = X->dtype;
        if (ep->op == SAGA_EDGE_MUL_WEIGHT)
            ga.edge_w = ep->edge_weight ? ep->edge_weight : static_cast<const float*>(g->d_edge_data.p);
        if (tf) {
            // Z = X W in X's dtype, no bias, no activation: those follow the sum
            DevBuf* zb = bf16 ? &ctx->ws_accum16 : &ctx->ws_accum;
            if (saga_status st = ctx->dev_alloc(zb, (size_t)(bf16 ? 2 : 4) * (size_t)n * Fo_tf)) return st;
            saga_vertex_params vz{};
            vz.W = vp->W;
            vz.act = SAGA_ACT_NONE;
            if (saga_status st = run_apply_vertex(ctx, X->data, X->ld, X->dtype, n, F, &vz, nullptr, 0, 0, zb->p, Fo_tf, X->dtype))
                return st;
            ga.src = zb->p;
            ga.ld_src = Fo_tf;
            ga.F = Fo_tf;
            ga.bias = vp->bias ? static_cast<const float*>(vp->bias->data) : nullptr;
            ga.act = vp->act;
            if (es) es->has_hoist = true;  // the product is timed in the slot of the per-vertex products
        }
    }
    if (es) HIP_TRY(ctx, hipEventRecord(es->ev[1], s));

    // where the Gather output goes
    //   fp32: accum_out if given, else Y itself when there is no ApplyVertex, else workspace
    //   bf16: a bf16 copy feeds the ApplyVertex product (or is Y itself without one);
    //         the fp32 rows are written only when accum_out asks for them
    if (tf) {
        if (bf16) {
            ga.out16 = static_cast<uint16_t*>(Y->data);
            ga.ld_out16 = Y->ld;
        } else {
            ga.out = static_cast<float*>(Y->data);
            ga.ld_out = Y->ld;
        }
    } else if (!bf16) {
        if (accum_out) {
            ga.out = static_cast<float*>(accum_out->data);
            ga.ld_out = accum_out->ld;
        } else if (!has_w) {
            ga.out = static_cast<float*>(Y->data);
            ga.ld_out = Y->ld;
        } else {
            if (saga_status st = ctx->dev_alloc(&ctx->ws_accum, sizeof(float) * (size_t)n * Fm)) return st;
            ga.out = static_cast<float*>(ctx->ws_accum.p);
            ga.ld_out = Fm;
        }
    } else {
        if (accum_out) {
            ga.out = static_cast<float*>(accum_out->data);
            ga.ld_out = accum_out->ld;
        }
        if (!has_w) {
            ga.out16 = static_cast<uint16_t*>(Y->data);
            ga.ld_out16 = Y->ld;
        } else {
            if (saga_status st = ctx->dev_alloc(&ctx->ws_accum16, sizeof(uint16_t) * (size_t)n * F)) return st;
            ga.out16 = static_cast<uint16_t*>(ctx->ws_accum16.p);
            ga.ld_out16 = F;
        }
    }
    if (n_slots > 0) {
        if (saga_status st = ctx->dev_alloc(&ctx->ws_partials, sizeof(float) * (size_t)n_slots * ga.F)) return st;
        ga.partials = static_cast<float*>(ctx->ws_partials.p);
    }
    bool dense_forked = false;
    if (hybrid) {
        const bool weighted = ep->op == SAGA_EDGE_MUL_WEIGHT;
        const float* w_src = !weighted ? nullptr : (ep->edge_weight ? ep->edge_weight : static_cast<const float*>(g->d_edge_data.p));
        if (saga_status st = hybrid_dense_launch(ctx, g, &ga, weighted, w_src, weighted && !ep->edge_weight, es, &dense_forked)) return st;
    }
    if (!ctx->opt_fused) {
        // the baseline of Section 6.2: the stages one by one through a materialised per-edge tensor, which the fused
        // operator exists to avoid; Gather then is the same kernel reading message e for edge e
        if (ep->op != SAGA_EDGE_COPY && ep->op != SAGA_EDGE_MUL_WEIGHT)
            return ctx->fail(SAGA_ERR_UNSUPPORTED, "option fused = 0 covers COPY and MUL_WEIGHT messages");
        const size_t msg_bytes = sizeof(float) * (size_t)std::max<int64_t>(g->nnz, 1) * ga.F;
        const size_t all_bytes = (msg_bytes + 255) / 256 * 256 + sizeof(int32_t) * (size_t)std::max<int64_t>(g->nnz, 1);
        if (all_bytes > ((size_t)128 << 30) || (ctx->budget > 0 && ctx->cur_bytes + all_bytes > ctx->budget))
            return ctx->fail(SAGA_ERR_BUDGET, "the per-edge tensor of the unfused stages needs %zu bytes", all_bytes);
        if (saga_status st = ctx->dev_alloc(&ctx->ws_edge_msg, all_bytes)) return st;
        float* msg = static_cast<float*>(ctx->ws_edge_msg.p);
        int32_t* iota = reinterpret_cast<int32_t*>(static_cast<char*>(ctx->ws_edge_msg.p) + (msg_bytes + 255) / 256 * 256);
        HIP_TRY(ctx, launch_stage_scatter_apply(ga.src, ga.ld_src, ga.dtype, ga.row_idx, ga.edge_w, msg, iota, ga.F, g->nnz, s));
        ga.src = msg;
        ga.ld_src = ga.F;
        ga.dtype = SAGA_F32;
        ga.row_idx = iota;
        ga.edge_w = nullptr;
        ga.op = SAGA_EDGE_COPY;
        ga.mma = 0;
    }
    HIP_TRY(ctx, launch_gather(ga, s));
    if (dense_forked) HIP_TRY(ctx, hipStreamWaitEvent(s, ctx->ev_join, 0));
    if (es) HIP_TRY(ctx, hipEventRecord(es->ev[2], s));

    if (n_heavy > 0) {
        CombineArgs ca{};
        ca.heavy = heavy;
        ca.n_heavy = n_heavy;
        ca.partials = ga.partials;
        ca.F = ga.F;
        ca.agg = agg;
        ca.out = ga.out;
        ca.ld_out = ga.ld_out;
        ca.out16 = ga.out16;
        ca.ld_out16 = ga.ld_out16;
        ca.accumulate = 0;
        ca.bias = ga.bias;
        ca.act = ga.act;
        HIP_TRY(ctx, launch_combine(ca, s));
        if (es) es->has_combine = true;
    }
    if (es) HIP_TRY(ctx, hipEventRecord(es->ev[3], s));

    if (has_w && !tf) {
        const void* A = bf16 ? static_cast<const void*>(ga.out16) : static_cast<const void*>(ga.out);
        const int64_t lda = bf16 ? ga.ld_out16 : ga.ld_out;
        if (saga_status st = run_apply_vertex(ctx, A, lda, X->dtype, n, Fm, vp, X->data, X->ld, F, Y->data, Y->ld, Y->dtype))
            return st;
        if (es) es->has_apply = true;
    }
    if (es) {
        HIP_TRY(ctx, hipEventRecord(es->ev[4], s));
        ctx->ev_used += 1;
    }
    ctx->acc.n_work_items = hybrid ? g->hyb.n_items : g->n_items;
    ctx->acc.n_split_vertices = n_heavy;
    ctx->acc.n_dense_blocks = hybrid ? g->hyb.n_blocks : 0;
    ctx->acc.n_dense_edges = hybrid ? g->hyb.n_dense_edges : 0;
    ctx->acc.n_partial_rows = n_slots;
    ctx->acc.plan_dst_intervals = ctx->acc.plan_src_intervals = 0;
    return SAGA_OK;
}

saga_status saga_layer_forward_noalloc(saga_ctx* ctx, const saga_graph* g, const saga_tensor* X, const saga_edge_params* ep,
                                       int32_t agg, const saga_vertex_params* vp, saga_tensor* Y, saga_tensor* accum_out)
{
    if (!ctx) return SAGA_ERR_INVALID_ARG;
    if (!g || !X) return ctx->fail(SAGA_ERR_INVALID_ARG, "null argument");
    if (X->mem != SAGA_MEM_DEVICE || g->where != SAGA_MEM_DEVICE)
        return ctx->fail(SAGA_ERR_UNSUPPORTED, "saga_layer_forward_noalloc covers resident layers (device tensors, device graph)");
    if (ctx->arena_active) return ctx->fail(SAGA_ERR_INVALID_ARG, "saga_layer_forward_noalloc is not re-entrant");
    // The workspaces an ordinary call would grow are set aside; while arena_active every request is carved from the
    // static array (or refused), so the layer code below runs unchanged and reaches no allocator.
    DevBuf* const ws[] = {&ctx->ws_accum, &ctx->ws_accum16, &ctx->ws_partials, &ctx->ws_hoist, &ctx->ws_bt, &ctx->ws_bias, &ctx->ws_edge_msg};
    DevBuf saved[sizeof(ws) / sizeof(ws[0])];
    for (size_t i = 0; i < sizeof(ws) / sizeof(ws[0]); ++i) {
        saved[i] = *ws[i];
        *ws[i] = DevBuf{};
    }
    ctx->arena_used = 0;
    ctx->arena_active = true;
    const saga_status st = saga_layer_forward(ctx, g, X, ep, agg, vp, Y, accum_out);
    ctx->arena_active = false;
    for (size_t i = 0; i < sizeof(ws) / sizeof(ws[0]); ++i) *ws[i] = saved[i];
    return st;
}

saga_status saga_layer_forward(saga_ctx* ctx, const saga_graph* g, const saga_tensor* X, const saga_edge_params* ep,
                               int32_t agg, const saga_vertex_params* vp, saga_tensor* Y, saga_tensor* accum_out)
{
    if (!ctx) return SAGA_ERR_INVALID_ARG;
    if (!g || !X || !ep || !Y) return ctx->fail(SAGA_ERR_INVALID_ARG, "null argument");
    if (g->ctx != ctx) return ctx->fail(SAGA_ERR_INVALID_ARG, "graph belongs to another context");
    if (!tensor_ok(X) || !tensor_ok(Y)) return ctx->fail(SAGA_ERR_INVALID_ARG, "malformed X or Y tensor");
    if (agg != SAGA_AGG_SUM && agg != SAGA_AGG_MAX) return ctx->fail(SAGA_ERR_INVALID_ARG, "bad accumulator");
    if (ep->op < SAGA_EDGE_COPY || ep->op > SAGA_EDGE_POOL) return ctx->fail(SAGA_ERR_INVALID_ARG, "bad edge op");
    if (X->rows != g->n || Y->rows != g->n)
        return ctx->fail(SAGA_ERR_INVALID_ARG, "X/Y have %lld/%lld rows, graph has %lld vertices", (long long)X->rows,
                         (long long)Y->rows, (long long)g->n);
    if (X->cols > (1 << 20)) return ctx->fail(SAGA_ERR_UNSUPPORTED, "feature width above 2^20");
    const int64_t F = X->cols;
    const bool has_w = vp && vp->W;
    if (vp && (vp->act < SAGA_ACT_NONE || vp->act > SAGA_ACT_SIGMOID)) return ctx->fail(SAGA_ERR_INVALID_ARG, "bad activation");
    int64_t Fm = F;  // message width
    if (ep->op == SAGA_EDGE_POOL) {
        if (X->dtype != SAGA_F32) return ctx->fail(SAGA_ERR_UNSUPPORTED, "max-pooling ApplyEdge is fp32 only");
        const saga_tensor* Wp = ep->W_pool;
        if (!tensor_ok(Wp) || Wp->mem != SAGA_MEM_DEVICE || Wp->dtype != SAGA_F32 || Wp->cols != F || Wp->rows < 1 ||
            Wp->rows > (1 << 20))
            return ctx->fail(SAGA_ERR_INVALID_ARG, "W_pool must be a device F_pool x F fp32 tensor");
        if (ep->b_pool && (!tensor_ok(ep->b_pool) || ep->b_pool->mem != SAGA_MEM_DEVICE || ep->b_pool->dtype != SAGA_F32 ||
                           ep->b_pool->rows * ep->b_pool->cols != Wp->rows))
            return ctx->fail(SAGA_ERR_INVALID_ARG, "b_pool must be F_pool fp32 values on the device");
        Fm = Wp->rows;
    }
    if (has_w) {
        const saga_tensor* W = vp->W;
        if (!tensor_ok(W) || W->mem != SAGA_MEM_DEVICE || W->rows != Fm || W->dtype != X->dtype)
            return ctx->fail(SAGA_ERR_INVALID_ARG, "W must be a device Fm x F_out tensor of X's dtype");
        if (vp->W_self && (!tensor_ok(vp->W_self) || vp->W_self->mem != SAGA_MEM_DEVICE || vp->W_self->rows != F ||
                           vp->W_self->cols != W->cols || vp->W_self->dtype != X->dtype))
            return ctx->fail(SAGA_ERR_INVALID_ARG, "W_self must be a device F_in x F_out tensor of X's dtype");
        if (vp->bias && (!tensor_ok(vp->bias) || vp->bias->mem != SAGA_MEM_DEVICE || vp->bias->dtype != SAGA_F32 ||
                         vp->bias->rows * vp->bias->cols != W->cols))
            return ctx->fail(SAGA_ERR_INVALID_ARG, "bias must be F_out fp32 values on the device");
        if (Y->cols != W->cols) return ctx->fail(SAGA_ERR_INVALID_ARG, "Y has %lld columns, W has %lld", (long long)Y->cols, (long long)W->cols);
    } else {
        if (Y->cols != Fm) return ctx->fail(SAGA_ERR_INVALID_ARG, "without W, Y must be n x Fm");
        if (vp && (vp->bias || vp->act != SAGA_ACT_NONE || vp->W_self))
            return ctx->fail(SAGA_ERR_UNSUPPORTED, "bias, activation or W_self without W");
    }
    if (Y->dtype != X->dtype) return ctx->fail(SAGA_ERR_INVALID_ARG, "Y must have X's dtype");
    if (ep->op == SAGA_EDGE_GATED) {
        if (X->dtype != SAGA_F32) return ctx->fail(SAGA_ERR_UNSUPPORTED, "gated ApplyEdge is fp32 only");
        const saga_tensor* Wg = ep->W_gate;
        if (!tensor_ok(Wg) || Wg->mem != SAGA_MEM_DEVICE || Wg->dtype != SAGA_F32 || Wg->rows != F || Wg->cols != 2 * F)
            return ctx->fail(SAGA_ERR_INVALID_ARG, "W_gate must be a device F x 2F fp32 tensor");
        if (ep->b_gate && (!tensor_ok(ep->b_gate) || ep->b_gate->mem != SAGA_MEM_DEVICE || ep->b_gate->dtype != SAGA_F32 ||
                           ep->b_gate->rows * ep->b_gate->cols != F))
            return ctx->fail(SAGA_ERR_INVALID_ARG, "b_gate must be F fp32 values on the device");
        if (ep->W_msg && (!tensor_ok(ep->W_msg) || ep->W_msg->mem != SAGA_MEM_DEVICE || ep->W_msg->dtype != SAGA_F32 ||
                          ep->W_msg->rows != F || ep->W_msg->cols != F))
            return ctx->fail(SAGA_ERR_INVALID_ARG, "W_msg must be a device F x F fp32 tensor");
    }
    DeviceGuard guard(ctx->device);

    const bool streamed = X->mem == SAGA_MEM_HOST;
    if (streamed) {
        if (Y->mem != SAGA_MEM_HOST || g->where != SAGA_MEM_HOST)
            return ctx->fail(SAGA_ERR_INVALID_ARG, "streamed calls need X, Y and the graph in host memory");
        if (accum_out && (!tensor_ok(accum_out) || accum_out->mem != SAGA_MEM_HOST || accum_out->dtype != SAGA_F32 ||
                          accum_out->rows != g->n || accum_out->cols != Fm))
            return ctx->fail(SAGA_ERR_INVALID_ARG, "accum_out of a streamed call must be a host n x Fm fp32 tensor");
        if (X->dtype != SAGA_F32) return ctx->fail(SAGA_ERR_UNSUPPORTED, "the streamed path is fp32 only");
        if (ep->op == SAGA_EDGE_MUL_WEIGHT && g->h_edge_data.empty() && g->nnz > 0)
            return ctx->fail(SAGA_ERR_INVALID_ARG, "streamed MUL_WEIGHT needs saga_graph_set_edge_data");
        const saga_status sst = guarded(ctx, [&] { return streamed_layer(ctx, const_cast<saga_graph*>(g), X, ep, agg, vp, Y, accum_out); });
        if (sst != SAGA_OK) chunk_grid_drain(ctx);  // host tensors are the caller's again when this returns
        return sst;
    }
    if (Y->mem != SAGA_MEM_DEVICE || g->where != SAGA_MEM_DEVICE)
        return ctx->fail(SAGA_ERR_INVALID_ARG, "resident calls need X, Y and the graph in device memory");
    if (accum_out && (!tensor_ok(accum_out) || accum_out->mem != SAGA_MEM_DEVICE || accum_out->dtype != SAGA_F32 ||
                      accum_out->rows != g->n || accum_out->cols != Fm))
        return ctx->fail(SAGA_ERR_INVALID_ARG, "accum_out must be a device n x Fm fp32 tensor");
    if (ep->op == SAGA_EDGE_MUL_WEIGHT && !ep->edge_weight && !g->d_edge_data.p && g->nnz > 0)
        return ctx->fail(SAGA_ERR_INVALID_ARG, "MUL_WEIGHT needs edge_weight or saga_graph_set_edge_data");
    if (g->n == 0) return SAGA_OK;
    return guarded(ctx, [&] { return resident_forward(ctx, const_cast<saga_graph*>(g), X, ep, agg, vp, Y, accum_out); });
}

saga_status saga_layer_backward(saga_ctx* ctx, const saga_graph* g, const saga_tensor* X, const saga_tensor* A,
                                const saga_tensor* Y, const saga_tensor* dY, const saga_edge_params* ep, int32_t agg,
                                const saga_vertex_params* vp, const saga_layer_grads* grads)
{
    if (!ctx) return SAGA_ERR_INVALID_ARG;
    if (!g || !A || !dY || !ep || !vp || !grads) return ctx->fail(SAGA_ERR_INVALID_ARG, "null argument");
    if (g->ctx != ctx) return ctx->fail(SAGA_ERR_INVALID_ARG, "graph belongs to another context");
    if (g->where == SAGA_MEM_HOST) {
        // streamed: the layer's tensors live in host memory, parameters and their gradients on the device
        auto f32_at = [](const saga_tensor* t, int32_t mem) { return tensor_ok(t) && t->mem == mem && t->dtype == SAGA_F32; };
        if (agg != SAGA_AGG_SUM && agg != SAGA_AGG_MAX) return ctx->fail(SAGA_ERR_INVALID_ARG, "bad accumulator");
        const bool pool_h = ep->op == SAGA_EDGE_POOL, gated_h = ep->op == SAGA_EDGE_GATED;
        if (ep->op < SAGA_EDGE_COPY || ep->op > SAGA_EDGE_POOL) return ctx->fail(SAGA_ERR_INVALID_ARG, "bad edge op");
        const bool max_or_pool = pool_h || (agg == SAGA_AGG_MAX && !gated_h);
        if (vp->act != SAGA_ACT_NONE && vp->act != SAGA_ACT_RELU && vp->act != SAGA_ACT_SIGMOID)
            return ctx->fail(SAGA_ERR_INVALID_ARG, "bad activation");
        const saga_tensor* W = vp->W;
        if (!W || !f32_at(W, SAGA_MEM_DEVICE) || W->rows > (1 << 20) || W->cols > (1 << 20))
            return ctx->fail(SAGA_ERR_INVALID_ARG, "W must be a device F_in x F_out fp32 tensor");
        const int64_t n = g->n, Fmh = W->rows, Fo = W->cols;  // Fmh: message width (rows of W, columns of A)
        int64_t F = Fmh;                                       // F: width of X and dX
        if (pool_h) {
            const saga_tensor* Wp = ep->W_pool;
            if (!Wp || !f32_at(Wp, SAGA_MEM_DEVICE) || Wp->rows != Fmh || Wp->cols < 1 || Wp->cols > (1 << 20))
                return ctx->fail(SAGA_ERR_INVALID_ARG, "W_pool must be a device F_pool x F fp32 tensor with F_pool = rows of W");
            F = Wp->cols;
            if (ep->b_pool && (!f32_at(ep->b_pool, SAGA_MEM_DEVICE) || ep->b_pool->rows * ep->b_pool->cols != Fmh))
                return ctx->fail(SAGA_ERR_INVALID_ARG, "b_pool must be F_pool fp32 values on the device");
            if (!grads->dW_pool || !f32_at(grads->dW_pool, SAGA_MEM_DEVICE) || grads->dW_pool->rows != Fmh || grads->dW_pool->cols != F)
                return ctx->fail(SAGA_ERR_INVALID_ARG, "grads->dW_pool must be a device F_pool x F fp32 tensor");
            if (grads->db_pool && (!f32_at(grads->db_pool, SAGA_MEM_DEVICE) || grads->db_pool->rows * grads->db_pool->cols != Fmh))
                return ctx->fail(SAGA_ERR_INVALID_ARG, "grads->db_pool must be F_pool fp32 values on the device");
        } else if (grads->dW_pool || grads->db_pool) {
            return ctx->fail(SAGA_ERR_INVALID_ARG, "pool gradients are for POOL layers only");
        }
        if ((max_or_pool || gated_h) && (!X || !f32_at(X, SAGA_MEM_HOST) || X->rows != n || X->cols != F))
            return ctx->fail(SAGA_ERR_INVALID_ARG, "this layer needs X as a host n x F fp32 tensor");
        if (gated_h) {
            if (!ep->W_gate || !f32_at(ep->W_gate, SAGA_MEM_DEVICE) || ep->W_gate->rows != F || ep->W_gate->cols != 2 * F)
                return ctx->fail(SAGA_ERR_INVALID_ARG, "W_gate must be a device F x 2F fp32 tensor");
            if (ep->b_gate && (!f32_at(ep->b_gate, SAGA_MEM_DEVICE) || ep->b_gate->rows * ep->b_gate->cols != F))
                return ctx->fail(SAGA_ERR_INVALID_ARG, "b_gate must be F fp32 values on the device");
            if (ep->W_msg && (!f32_at(ep->W_msg, SAGA_MEM_DEVICE) || ep->W_msg->rows != F || ep->W_msg->cols != F))
                return ctx->fail(SAGA_ERR_INVALID_ARG, "W_msg must be a device F x F fp32 tensor");
            if (!grads->dW_gate || !f32_at(grads->dW_gate, SAGA_MEM_DEVICE) || grads->dW_gate->rows != F || grads->dW_gate->cols != 2 * F)
                return ctx->fail(SAGA_ERR_INVALID_ARG, "grads->dW_gate must be a device F x 2F fp32 tensor");
            if (grads->db_gate && (!f32_at(grads->db_gate, SAGA_MEM_DEVICE) || grads->db_gate->rows * grads->db_gate->cols != F))
                return ctx->fail(SAGA_ERR_INVALID_ARG, "grads->db_gate must be F fp32 values on the device");
            if (grads->dW_msg && (!ep->W_msg || !f32_at(grads->dW_msg, SAGA_MEM_DEVICE) || grads->dW_msg->rows != F || grads->dW_msg->cols != F))
                return ctx->fail(SAGA_ERR_INVALID_ARG, "grads->dW_msg must be a device F x F fp32 tensor, and needs W_msg");
        } else if (grads->dW_gate || grads->db_gate || grads->dW_msg) {
            return ctx->fail(SAGA_ERR_INVALID_ARG, "gate gradients are for GATED layers only");
        }
        if (!f32_at(A, SAGA_MEM_HOST) || A->rows != n || A->cols != Fmh)
            return ctx->fail(SAGA_ERR_INVALID_ARG, "streamed calls need A as a host n x Fm fp32 tensor");
        if (!f32_at(dY, SAGA_MEM_HOST) || dY->rows != n || dY->cols != Fo)
            return ctx->fail(SAGA_ERR_INVALID_ARG, "streamed calls need dY as a host n x F_out fp32 tensor");
        if (vp->act != SAGA_ACT_NONE && (!Y || !f32_at(Y, SAGA_MEM_HOST) || Y->rows != n || Y->cols != Fo))
            return ctx->fail(SAGA_ERR_INVALID_ARG, "an activation needs Y as a host n x F_out fp32 tensor");
        if (!grads->dW || !f32_at(grads->dW, SAGA_MEM_DEVICE) || grads->dW->rows != Fmh || grads->dW->cols != Fo)
            return ctx->fail(SAGA_ERR_INVALID_ARG, "grads->dW must be a device Fm x F_out fp32 tensor");
        if (grads->dbias && (!f32_at(grads->dbias, SAGA_MEM_DEVICE) || grads->dbias->rows * grads->dbias->cols != Fo))
            return ctx->fail(SAGA_ERR_INVALID_ARG, "grads->dbias must be F_out fp32 values on the device");
        if (grads->dX && (!f32_at(grads->dX, SAGA_MEM_HOST) || grads->dX->rows != n || grads->dX->cols != F))
            return ctx->fail(SAGA_ERR_INVALID_ARG, "streamed calls need grads->dX as a host n x F fp32 tensor");
        if (vp->W_self) {
            if (!f32_at(vp->W_self, SAGA_MEM_DEVICE) || vp->W_self->rows != F || vp->W_self->cols != Fo)
                return ctx->fail(SAGA_ERR_INVALID_ARG, "W_self must be a device F_in x F_out fp32 tensor");
            if (!grads->dW_self || !f32_at(grads->dW_self, SAGA_MEM_DEVICE) || grads->dW_self->rows != F || grads->dW_self->cols != Fo)
                return ctx->fail(SAGA_ERR_INVALID_ARG, "W_self is given: grads->dW_self must be a device F_in x F_out fp32 tensor");
            if (!X || !f32_at(X, SAGA_MEM_HOST) || X->rows != n || X->cols != F)
                return ctx->fail(SAGA_ERR_INVALID_ARG, "W_self needs X as a host n x F_in fp32 tensor");
        } else if (grads->dW_self) {
            return ctx->fail(SAGA_ERR_INVALID_ARG, "grads->dW_self is given but W_self is not");
        }
        if (ep->op == SAGA_EDGE_MUL_WEIGHT && g->h_edge_data.empty() && g->nnz > 0)
            return ctx->fail(SAGA_ERR_INVALID_ARG, "streamed MUL_WEIGHT needs saga_graph_set_edge_data");
        DeviceGuard guard_h(ctx->device);
        const saga_status sst = guarded(ctx, [&] {
            return gated_h ? streamed_gated_backward(ctx, const_cast<saga_graph*>(g), X, A, Y, dY, ep, agg, vp, grads)
                   : max_or_pool ? streamed_max_pool_backward(ctx, const_cast<saga_graph*>(g), X, A, Y, dY, ep, agg, vp, grads)
                                 : streamed_backward(ctx, const_cast<saga_graph*>(g), X, A, Y, dY, ep, vp, grads);
        });
        if (sst != SAGA_OK) chunk_grid_drain(ctx);  // host tensors are the caller's again when this returns
        return sst;
    }
    if (agg != SAGA_AGG_SUM && agg != SAGA_AGG_MAX) return ctx->fail(SAGA_ERR_INVALID_ARG, "bad accumulator");
    const bool gated = ep->op == SAGA_EDGE_GATED, pool = ep->op == SAGA_EDGE_POOL;
    if (ep->op < SAGA_EDGE_COPY || ep->op > SAGA_EDGE_POOL) return ctx->fail(SAGA_ERR_INVALID_ARG, "bad edge op");
    if (vp->act != SAGA_ACT_NONE && vp->act != SAGA_ACT_RELU && vp->act != SAGA_ACT_SIGMOID)
        return ctx->fail(SAGA_ERR_INVALID_ARG, "bad activation");
    auto dev_f32 = [](const saga_tensor* t) { return tensor_ok(t) && t->mem == SAGA_MEM_DEVICE && t->dtype == SAGA_F32; };
    const saga_tensor* W = vp->W;
    if (!W) return ctx->fail(SAGA_ERR_UNSUPPORTED, "the backward pass needs an ApplyVertex product (vp->W)");
    if (tensor_ok(W) && W->dtype == SAGA_BF16) {
        // bf16 layers: X, W, Y, dY, dX in bf16; A and the parameter gradients in fp32
        auto dev_bf16 = [](const saga_tensor* t) { return tensor_ok(t) && t->mem == SAGA_MEM_DEVICE && t->dtype == SAGA_BF16; };
        if (agg != SAGA_AGG_SUM || (ep->op != SAGA_EDGE_COPY && ep->op != SAGA_EDGE_MUL_WEIGHT))
            return ctx->fail(SAGA_ERR_UNSUPPORTED, "the bf16 backward pass covers sum over COPY / MUL_WEIGHT messages");
        if (vp->act == SAGA_ACT_SIGMOID)  // a derivative y (1 - y) from an 8-bit y is not worth having
            return ctx->fail(SAGA_ERR_UNSUPPORTED, "the bf16 backward pass covers activations NONE and RELU only");
        if (!dev_bf16(W) || W->rows > (1 << 20) || W->cols > (1 << 20)) return ctx->fail(SAGA_ERR_INVALID_ARG, "malformed W");
        const int64_t n = g->n, F = W->rows, Fo = W->cols;
        if (!dev_f32(A) || A->rows != n || A->cols != F) return ctx->fail(SAGA_ERR_INVALID_ARG, "A must be a device n x F_in fp32 tensor");
        if (!dev_bf16(dY) || dY->rows != n || dY->cols != Fo)
            return ctx->fail(SAGA_ERR_INVALID_ARG, "dY must be a device n x F_out bf16 tensor, like W");
        if (vp->act == SAGA_ACT_RELU && (!Y || !dev_bf16(Y) || Y->rows != n || Y->cols != Fo))
            return ctx->fail(SAGA_ERR_INVALID_ARG, "RELU needs Y as a device n x F_out bf16 tensor");
        if (!grads->dW || !dev_f32(grads->dW) || grads->dW->rows != F || grads->dW->cols != Fo)
            return ctx->fail(SAGA_ERR_INVALID_ARG, "grads->dW must be a device F_in x F_out fp32 tensor");
        if (grads->dbias && (!dev_f32(grads->dbias) || grads->dbias->rows * grads->dbias->cols != Fo))
            return ctx->fail(SAGA_ERR_INVALID_ARG, "grads->dbias must be F_out fp32 values on the device");
        if (grads->dX && (!dev_bf16(grads->dX) || grads->dX->rows != n || grads->dX->cols != F))
            return ctx->fail(SAGA_ERR_INVALID_ARG, "grads->dX must be a device n x F_in bf16 tensor");
        if (vp->W_self) {
            if (!dev_bf16(vp->W_self) || vp->W_self->rows != F || vp->W_self->cols != Fo)
                return ctx->fail(SAGA_ERR_INVALID_ARG, "W_self must be a device F_in x F_out bf16 tensor, like W");
            if (!X || !dev_bf16(X) || X->rows != n || X->cols != F)
                return ctx->fail(SAGA_ERR_INVALID_ARG, "W_self needs X as a device n x F_in bf16 tensor");
            if (!grads->dW_self || !dev_f32(grads->dW_self) || grads->dW_self->rows != F || grads->dW_self->cols != Fo)
                return ctx->fail(SAGA_ERR_INVALID_ARG, "W_self is given: grads->dW_self must be a device F_in x F_out fp32 tensor");
        } else if (grads->dW_self) {
            return ctx->fail(SAGA_ERR_INVALID_ARG, "grads->dW_self is given but W_self is not");
        }
        if (grads->dW_gate || grads->db_gate || grads->dW_msg || grads->dW_pool || grads->db_pool)
            return ctx->fail(SAGA_ERR_INVALID_ARG, "this layer has no such parameter gradients");
        if (ep->op == SAGA_EDGE_MUL_WEIGHT && !ep->edge_weight && !g->d_edge_data.p && g->nnz > 0)
            return ctx->fail(SAGA_ERR_INVALID_ARG, "MUL_WEIGHT needs edge_weight or saga_graph_set_edge_data");
        DeviceGuard guard16(ctx->device);
        return guarded(ctx, [&] { return resident_backward_bf16(ctx, const_cast<saga_graph*>(g), X, A, Y, dY, ep, vp, grads); });
    }
    if (!dev_f32(W) || W->rows > (1 << 20) || W->cols > (1 << 20))
        return ctx->fail(SAGA_ERR_INVALID_ARG, "W must be a device Fm x F_out fp32 tensor");
    // Fm: message width (rows of W, columns of A); F: width of X and dX
    const int64_t n = g->n, Fm = W->rows, Fo = W->cols;
    int64_t F = Fm;
    if (pool) {
        const saga_tensor* Wp = ep->W_pool;
        if (!Wp || !dev_f32(Wp) || Wp->rows != Fm || Wp->cols < 1 || Wp->cols > (1 << 20))
            return ctx->fail(SAGA_ERR_INVALID_ARG, "W_pool must be a device F_pool x F fp32 tensor with F_pool = rows of W");
        F = Wp->cols;
        if (ep->b_pool && (!dev_f32(ep->b_pool) || ep->b_pool->rows * ep->b_pool->cols != Fm))
            return ctx->fail(SAGA_ERR_INVALID_ARG, "b_pool must be F_pool fp32 values on the device");
        if (!grads->dW_pool || !dev_f32(grads->dW_pool) || grads->dW_pool->rows != Fm || grads->dW_pool->cols != F)
            return ctx->fail(SAGA_ERR_INVALID_ARG, "grads->dW_pool must be a device F_pool x F fp32 tensor");
        if (grads->db_pool && (!dev_f32(grads->db_pool) || grads->db_pool->rows * grads->db_pool->cols != Fm))
            return ctx->fail(SAGA_ERR_INVALID_ARG, "grads->db_pool must be F_pool fp32 values on the device");
    } else if (grads->dW_pool || grads->db_pool) {
        return ctx->fail(SAGA_ERR_INVALID_ARG, "pool gradients are for POOL layers only");
    }
    if (!dev_f32(A) || A->rows != n || A->cols != Fm) return ctx->fail(SAGA_ERR_INVALID_ARG, "A must be a device n x Fm fp32 tensor");
    if (!dev_f32(dY) || dY->rows != n || dY->cols != Fo)
        return ctx->fail(SAGA_ERR_INVALID_ARG, "dY must be a device n x F_out fp32 tensor");
    if (vp->act != SAGA_ACT_NONE && (!Y || !dev_f32(Y) || Y->rows != n || Y->cols != Fo))
        return ctx->fail(SAGA_ERR_INVALID_ARG, "an activation needs Y as a device n x F_out fp32 tensor");
    const bool needs_x = vp->W_self || gated || pool || agg == SAGA_AGG_MAX;
    if (needs_x && (!X || !dev_f32(X) || X->rows != n || X->cols != F))
        return ctx->fail(SAGA_ERR_INVALID_ARG, "this layer needs X as a device n x F fp32 tensor");
    if (vp->W_self) {
        if (!dev_f32(vp->W_self) || vp->W_self->rows != F || vp->W_self->cols != Fo)
            return ctx->fail(SAGA_ERR_INVALID_ARG, "W_self must be a device F_in x F_out fp32 tensor");
        if (!grads->dW_self) return ctx->fail(SAGA_ERR_INVALID_ARG, "W_self is given but grads->dW_self is not");
    } else if (grads->dW_self) {
        return ctx->fail(SAGA_ERR_INVALID_ARG, "grads->dW_self is given but W_self is not");
    }
    if (!grads->dW || !dev_f32(grads->dW) || grads->dW->rows != Fm || grads->dW->cols != Fo)
        return ctx->fail(SAGA_ERR_INVALID_ARG, "grads->dW must be a device Fm x F_out fp32 tensor");
    if (grads->dW_self && (!dev_f32(grads->dW_self) || grads->dW_self->rows != F || grads->dW_self->cols != Fo))
        return ctx->fail(SAGA_ERR_INVALID_ARG, "grads->dW_self must be a device F_in x F_out fp32 tensor");
    if (grads->dbias && (!dev_f32(grads->dbias) || grads->dbias->rows * grads->dbias->cols != Fo))
        return ctx->fail(SAGA_ERR_INVALID_ARG, "grads->dbias must be F_out fp32 values on the device");
    if (grads->dX && (!dev_f32(grads->dX) || grads->dX->rows != n || grads->dX->cols != F))
        return ctx->fail(SAGA_ERR_INVALID_ARG, "grads->dX must be a device n x F fp32 tensor");
    if (ep->op == SAGA_EDGE_MUL_WEIGHT && !ep->edge_weight && !g->d_edge_data.p && g->nnz > 0)
        return ctx->fail(SAGA_ERR_INVALID_ARG, "MUL_WEIGHT needs edge_weight or saga_graph_set_edge_data");
    if (gated) {
        if (!ep->W_gate || !dev_f32(ep->W_gate) || ep->W_gate->rows != F || ep->W_gate->cols != 2 * F)
            return ctx->fail(SAGA_ERR_INVALID_ARG, "W_gate must be a device F x 2F fp32 tensor");
        if (ep->b_gate && (!dev_f32(ep->b_gate) || ep->b_gate->rows * ep->b_gate->cols != F))
            return ctx->fail(SAGA_ERR_INVALID_ARG, "b_gate must be F fp32 values on the device");
        if (ep->W_msg && (!dev_f32(ep->W_msg) || ep->W_msg->rows != F || ep->W_msg->cols != F))
            return ctx->fail(SAGA_ERR_INVALID_ARG, "W_msg must be a device F x F fp32 tensor");
        if (!grads->dW_gate || !dev_f32(grads->dW_gate) || grads->dW_gate->rows != F || grads->dW_gate->cols != 2 * F)
            return ctx->fail(SAGA_ERR_INVALID_ARG, "grads->dW_gate must be a device F x 2F fp32 tensor");
        if (grads->db_gate && (!dev_f32(grads->db_gate) || grads->db_gate->rows * grads->db_gate->cols != F))
            return ctx->fail(SAGA_ERR_INVALID_ARG, "grads->db_gate must be F fp32 values on the device");
        if (grads->dW_msg && (!ep->W_msg || !dev_f32(grads->dW_msg) || grads->dW_msg->rows != F || grads->dW_msg->cols != F))
            return ctx->fail(SAGA_ERR_INVALID_ARG, "grads->dW_msg must be a device F x F fp32 tensor, and needs W_msg");
    } else if (grads->dW_gate || grads->db_gate || grads->dW_msg) {
        return ctx->fail(SAGA_ERR_INVALID_ARG, "gate gradients are for GATED layers only");
    }
    DeviceGuard guard(ctx->device);
    return guarded(ctx, [&] { return resident_backward(ctx, const_cast<saga_graph*>(g), X, A, Y, dY, ep, agg, vp, grads); });
}

}  // extern "C"

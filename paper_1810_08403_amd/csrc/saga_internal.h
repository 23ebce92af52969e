// Internal declarations shared by the translation units of libsaga.
#pragma once

#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <functional>
#include <string>
#include <thread>
#include <vector>

#include "../../include/saga.h"

// fn(i) for i in [0, n) on up to max_threads threads. fn must not throw. If a thread cannot be started the threads that
// did start (or the caller alone) do all the work: nothing is thrown from here.
template <typename Fn>
inline void parallel_for(int64_t n, int max_threads, Fn fn)
{
    const int nt = (int)std::max<int64_t>(1, std::min<int64_t>(std::min<int64_t>(n, max_threads), std::thread::hardware_concurrency()));
    if (nt <= 1) {
        for (int64_t i = 0; i < n; ++i) fn(i);
        return;
    }
    std::atomic<int64_t> next{0};
    auto work = [&] {
        for (;;) {
            const int64_t i = next.fetch_add(1);
            if (i >= n) break;
            fn(i);
        }
    };
    std::vector<std::thread> th;
    try {
        th.reserve((size_t)nt);
        for (int t = 1; t < nt; ++t) th.emplace_back(work);
    } catch (...) {
        // out of threads or memory: carry on with what there is
    }
    work();
    for (auto& t : th) t.join();
}

// ---------------------------------------------------------------------------
// work list: the unit a wavefront of the propagation kernel processes
// ---------------------------------------------------------------------------
// One item is a run of consecutive in-edges of one destination vertex
// (Section 3.3: a vertex's in-edge group, cut into consecutive sub-groups when
// the in-degree is large). slot < 0: the item covers the whole column and its
// result is the vertex's row. slot >= 0: the item writes a partial row
// `slot`, and a combine pass reduces a vertex's partial rows in slot order.
struct WorkItem {
    int32_t v;     // destination vertex (local to the output interval)
    int32_t e0;    // first edge
    int32_t e1;    // one past the last edge
    int32_t slot;  // partial-row index, or -1
};
struct HeavyVertex {
    int32_t v;
    int32_t slot0;
    int32_t nslots;
    int32_t pad;
};

struct WorkList {
    std::vector<WorkItem> items;  // team items first (one workgroup each), then solo items (one wavefront each)
    std::vector<HeavyVertex> heavy;
    int64_t n_team = 0;
    int64_t n_slots = 0;
    int64_t max_degree = 0;
};

struct WorkListParams {
    int64_t min_edges;    // a piece of a cut column holds at least this many edges
    int64_t cut_degree;   // columns with more in-edges than this are cut
    int64_t stripe_rows;  // pieces end on multiples of this many source rows (0: cut by count only)
    bool skip_empty = false;  // leave columns without edges out (streamed chunks: nothing to add)
    int32_t team = 1;         // wavefronts that share one piece of a cut column (1 or 4)
    int32_t order = 1;        // pieces in the list: 0 by first band and column, 1 by first band, last band and column
};
// Build the work list of a CSC block whose arrays are on the host
// (col_ptr[0] = 0; vertex ids and edge offsets are local to the block).
// extra_slots (nullable, one per column): partial rows that another kernel writes for the column ahead of
// its own pieces (the dense blocks below). Such a column is always combined from partial rows: slots
// [slot0, slot0 + extra) are reserved for the other kernel, its pieces (all of them, even a single one) follow.
struct saga_ctx;
// width: features of the rows the propagation writes (0: not known), see the definition
WorkListParams work_list_params(const saga_ctx* ctx, int64_t row_bytes, int32_t width = 0);
void build_work_list(const int64_t* col_ptr, const int32_t* row_idx, int64_t n_cols, const WorkListParams& p,
                     WorkList* out, const int32_t* extra_slots = nullptr);

// ---------------------------------------------------------------------------
// dense blocks: the part of the adjacency matrix that is a dense contraction
// ---------------------------------------------------------------------------
// Destinations ranked by in-degree and sources ranked by out-degree, grouped 64 and 32 at a time, cut the
// adjacency matrix into 64 x 32 blocks. In a power-law graph the blocks of heavy destinations and heavy
// sources are well filled: there the sum over in-edges is a dense product A_block (64 x 32 edge weights)
// times X_block (32 source rows), which the matrix cores do at a cost that does not depend on how many of
// the 2,048 cells hold an edge, and every source row is read once for 64 destinations instead of once per
// edge. Blocks with at least min_block_edges edges go that way (in destination tiles where that pays for
// the partial rows it costs); all other edges stay with the sparse propagation kernel as a remainder CSC.
constexpr int kDenseM = 64, kDenseK = 32;
struct HybridParams {
    // A block costs the matrix cores the same whatever its fill (64 MFMAs per wavefront: about a microsecond of one compute
    // unit with two-part weights), an edge whose source row hits in the L2 costs the sparse kernel about 0.02 ns of the whole
    // chip. Measured on the R-MAT 18 workload (512 bf16 features) the layer takes 4.11 ms with blocks from 200 edges on
    // (a tenth full), 4.14 at 192, 4.16 at 208, 4.27 at 160, 4.36 at 144, 4.48 at 256; the backward pass of the same layer
    // (256 features) 3.43 ms at 192, 3.51 at 208, 3.66 at 256.
    int64_t min_block_edges = 200;
    int64_t min_tile_gain = 512;    // edges beyond min_block_edges, summed over a destination tile's blocks, that pay for its partial rows
    int32_t max_chunk_blocks = 128; // blocks of one destination tile worked by one workgroup (one partial row per destination each)
};
// A block's weights reach the kernel in one of two forms: as a list of (cell, weight) pairs that the workgroup scatters
// into a cleared LDS operand (blocks of up to kDenseListMax edges: one pair per thread), or, for fuller blocks, as the
// finished 64 x 32 operand itself (two bf16 parts, 8 KiB), which is copied into LDS as it is.
constexpr int kDenseListMax = 256;
constexpr int kDenseTileElems = 2 * kDenseM * kDenseK;  // bf16 values of a finished operand: high parts, then low parts
struct DenseChunk {
    int32_t tile;   // destination tile
    int32_t b0, b1; // its blocks [b0, b1)
    int32_t cidx;   // which of the tile's chunks this is: the partial row written for a destination is slot0 + cidx
};
struct HybridPlan {
    int64_t n_dst_tiles = 0, n_src_tiles = 0, n_dense_edges = 0;
    std::vector<int32_t> dst_order;      // n_dst_tiles * 64: the vertex at each destination rank (-1: none)
    std::vector<int32_t> src_tile_ids;   // n_src_tiles * 32: the vertex at each source rank (0 where there is none: a valid row, never weighted)
    std::vector<int32_t> blk_src_tile;   // per block
    std::vector<int32_t> blk_e0;         // per block + 1: its edges in de_pos / de_edge (none for a block kept as a finished operand)
    std::vector<int32_t> blk_tile;       // per block: which finished operand is its own, or -1 for a block kept as a list
    int64_t n_tiles = 0;                 // finished operands
    std::vector<uint16_t> de_pos;        // list blocks: where the edge's weight sits in the block's 64 x 32 operand (matrix-core lane order)
    std::vector<int32_t> de_edge;        // the edge's number in the caller's edge order
    std::vector<int32_t> dt_addr;        // edges of finished operands: operand * kDenseTileElems + cell (the high part; the low part is kDenseM * kDenseK further)
    std::vector<int32_t> dt_edge;
    std::vector<DenseChunk> chunks;
    std::vector<int32_t> extra_slots;    // per vertex: chunks of its destination tile (0: the tile has no dense blocks)
    std::vector<int64_t> rem_col_ptr;    // the remainder as a CSC of its own (sources ascending inside a column)
    std::vector<int32_t> rem_row_idx, rem_edge;
};
void build_hybrid_plan(const int64_t* col_ptr, const int32_t* row_idx, int64_t n, const HybridParams& hp, HybridPlan* out);

// ---------------------------------------------------------------------------
// device buffers with accounting
// ---------------------------------------------------------------------------
struct saga_ctx;

struct DevBuf {
    void* p = nullptr;
    size_t bytes = 0;
};

struct saga_ctx {
    int device = 0;
    hipStream_t stream = nullptr;
    bool own_stream = false;
    size_t budget = 0;
    size_t cur_bytes = 0, peak_bytes = 0;
    std::string err;

    // tunables
    int64_t opt_split = 64;        // minimum edges per piece of a cut column
    bool opt_split_set = false;    // the caller has chosen it (narrow rows otherwise get finer pieces, see work_list_params)
    int64_t opt_cut_degree = 0;    // 0 = 2 * split
    int64_t opt_stripe_kb = 1024;  // source-row band one piece may span, in KiB of feature rows (0 = cut by count)
    bool opt_stripe_set = false;   // the caller has chosen it (the remainder of the dense-block path otherwise takes wider bands for 1 KiB rows)
    int opt_piece_order = 1;       // see WorkListParams::order
    int opt_xcd_remap = 1;
    int opt_mma = 0;               // 1: bf16 sum propagation with the multiply-accumulate on the matrix unit (measured: a tie)
    int opt_team = 0;              // 1: a piece of a cut column is worked by a whole workgroup (measured slower)
    int opt_dst_intervals = 0, opt_src_intervals = 0;
    int opt_schedule = 0;  // streamed path: 0 the paper's schedule, 1 stage by stage, 2 destination order innermost
    int opt_overlap = 1;   // streamed path: copies on their own streams
    int64_t opt_bwd_tile_rows = 0;  // streamed backward: rows per tile of backward-ApplyVertex (0 = about 64 MiB)
    int opt_transform_first = 0;  // resident linear sum layers with F_out < F_in: Y = act(gather(X W) + bias)
    int opt_fused = 1;            // 0: resident linear layers run Scatter, ApplyEdge and Gather as separate stages (baseline)
    int opt_dense_blocks = 1;     // bf16 sum layers over COPY / MUL_WEIGHT edges: well-filled blocks of the adjacency matrix on the matrix cores
    int64_t opt_dense_min_edges = 0, opt_dense_tile_gain = -1, opt_dense_chunk = 0;  // 0 / -1: the defaults of HybridParams

    // reusable workspace (grown on demand, never shrunk until destroy)
    DevBuf ws_accum;     // Gather output A (fp32 or bf16) when the caller gives no accum_out
    DevBuf ws_accum16;   // bf16 copy of A for the bf16 ApplyVertex product
    DevBuf ws_partials;  // partial rows of split vertices
    DevBuf ws_hoist;     // [Ps | M | Pd] per vertex (gated)
    DevBuf ws_bt;        // packed, transposed weights
    DevBuf ws_bias;      // packed bias for the hoisted product
    DevBuf ws_flag;      // validation flag
    // backward pass
    DevBuf ws_dz;        // gradient of the pre-activation (ReLU layers)
    DevBuf ws_grad;      // gradient rows between the dense product and the propagation kernel
    DevBuf ws_splitk;    // per-split partials of the parameter gradients and of the bias column sums
    DevBuf ws_edge_t;    // per-call edge weights in the order of the transposed graph
    DevBuf ws_dh;        // gated layers: per-vertex gradients [dPs | dM | dPd]
    DevBuf ws_dz16;      // bf16 layers: the gradient of the pre-activation in bf16
    // streamed calls: accumulator interval, two vertex intervals, two chunk payloads, two output tiles, partial rows
    DevBuf st_A, st_V[2], st_C[2], st_Y[2], st_partials;
    DevBuf st_D, st_S[2];  // gated: destination parts of the resident interval; W_self: tiles of the interval's own rows
    float* h_grad = nullptr;   // streamed backward of max / pooled layers: the gradient of accum of all vertices, pinned
    size_t h_grad_bytes = 0;
    // The copy-in and copy-out streams and the events of the chunk schedule. They belong to the context, are made at the
    // first streamed call and live until saga_destroy: one streamed call runs at a time, and tilings come and go with
    // the row width of a call, which must not cost a stream and fourteen events each time.
    struct StreamSet {
        hipStream_t s_in = nullptr, s_out = nullptr;
        hipEvent_t ev_ready[2] = {nullptr, nullptr}, ev_free[2] = {nullptr, nullptr};
        hipEvent_t ev_y_ready[2] = {nullptr, nullptr}, ev_y_free[2] = {nullptr, nullptr};
        hipEvent_t ev_a_done = nullptr, ev_a_ready = nullptr, ev_a_in = nullptr;
        hipEvent_t ev_d_free = nullptr, ev_s_ready[2] = {nullptr, nullptr};  // destination parts / own-row tiles (gated, W_self)
        bool ready = false;
    } st;
    saga_status ensure_stream_set();
    void destroy_stream_set();
    // a second compute stream for the dense-block kernel, which runs beside the sparse propagation kernel (the two are
    // bound by different things: the matrix cores and memory latency, and the traffic below the L2), with the events that
    // fork it from and join it to the context's stream; made at the first call that needs it
    hipStream_t s_dense = nullptr;
    hipEvent_t ev_fork = nullptr, ev_join = nullptr;
    int opt_dense_overlap = 0;  // measured: no gain, the two kernels fill the chip one after the other
    DevBuf ws_wt;        // streamed backward: W transposed, the "ApplyVertex" matrix of the backward propagation
    DevBuf ws_prod;      // streamed gated / pooled layers: packed weights of the per-vertex products (VertexProducts)
    DevBuf ws_edge_msg;  // stage-by-stage baseline: the per-edge tensor (n_edges x F fp32) and the edge numbers behind it
    DevBuf ws_tile;      // streamed backward of max / pooled layers: a tile of the gradient of accum, rows of X of an interval

    // profiling
    bool profiling = false;
    struct EventSet {
        hipEvent_t ev[5];
        hipEvent_t ev_dense;  // after the dense-block kernel, before the sparse one (same stream)
        bool has_hoist, has_combine, has_apply, has_dense;
        int n_gather_launches;
    };
    std::vector<EventSet> ev_pool;
    size_t ev_used = 0;
    saga_timings acc{};

    // saga_layer_forward_noalloc: while arena_active, dev_alloc carves from the library's static device array instead of
    // calling the allocator, dev_free does nothing, and a missing work list is an error instead of being built
    unsigned char* scratch_ptr = nullptr;  // device address of the static array on this context's device
    size_t arena_used = 0;
    bool arena_active = false;

    saga_status fail(saga_status s, const char* fmt, ...);
    saga_status dev_alloc(DevBuf* b, size_t bytes);  // frees and reallocates when too small
    void dev_free(DevBuf* b);
    saga_status drain_events();
    // Before `bytes` more device bytes are taken outside the streamed schedule: if they would not fit the budget beside the
    // schedule's buffers of an earlier call, those are given up (the next streamed call allocates what its plan needs).
    void make_room(size_t bytes);
};

struct ChunkGrid;  // streamed representation (chunked.hip)

// The dense-block form of a resident graph on the device (built at the first call that can use it).
struct HybridDevice {
    bool built = false, usable = false;   // usable: the graph has dense blocks worth taking
    WorkListParams list_params{-1, -1, -1, false, 1};
    HybridParams hp;
    int64_t n_chunks = 0, n_blocks = 0, n_dense_edges = 0, n_rem_edges = 0;
    DevBuf chunks, blk_src_tile, blk_e0, blk_tile, de_pos, de_edge, de_w, dt_addr, dt_edge, de_tiles, src_tile_ids, tile_row_slot0;
    int64_t n_list_edges = 0, n_tile_edges = 0, n_tiles = 0;
    DevBuf rem_row_idx, rem_edge, rem_w, items, heavy;
    int64_t n_items = 0, n_team = 0, n_heavy = 0, n_slots = 0;
    int weights_state = 0;                // 0: de_w / rem_w not packed; 1: packed from the attached edge data; 2: packed as all ones (COPY)
};

struct saga_graph {
    saga_ctx* ctx = nullptr;
    int64_t n = 0, nnz = 0;
    int32_t where = SAGA_MEM_DEVICE;
    // resident form; the work list is built at the first call for a given
    // (split, cut_degree, stripe_rows) and rebuilt when those change
    DevBuf d_row_idx, d_items, d_heavy, d_edge_data;
    int64_t n_items = 0, n_team = 0, n_heavy = 0, n_slots = 0, max_degree = 0;
    WorkListParams list_params{-1, -1, -1, false, 1};
    // work lists built earlier for other row widths (layers of different width alternate between them)
    struct SavedList {
        WorkListParams params;
        DevBuf items, heavy;
        int64_t n_items, n_team, n_heavy, n_slots;
    };
    std::vector<SavedList> saved_lists;
    // host form (streamed)
    std::vector<int64_t> h_col_ptr;
    std::vector<int32_t> h_row_idx;
    std::vector<float> h_edge_data;
    ChunkGrid* grid = nullptr;
    // the same edges grouped by source (backward-Scatter gathers over out-edges): built at the
    // first backward call. tr's columns are this graph's sources; perm[e'] is the position in
    // this graph's edge order of the transposed graph's edge e'.
    // the vertices with out-edges and those with in-edges, ascending, each list padded to a multiple of 64 entries with its
    // last one: the per-vertex products of a gated or pooled ApplyEdge (Section 3.2) are needed for edge endpoints only
    // (ensure_endpoints; built at the first call that can use them)
    DevBuf d_src_rows, d_dst_rows;
    int64_t n_src_rows = 0, n_dst_rows = 0;
    bool endpoints_built = false;
    HybridDevice hyb;
    saga_graph* tr = nullptr;
    DevBuf d_perm;
    bool tr_edge_data_valid = false;  // tr->d_edge_data holds d_edge_data permuted
};

#define HIP_TRY(ctx, call)                                                                   \
    do {                                                                                     \
        hipError_t e__ = (call);                                                             \
        if (e__ != hipSuccess)                                                               \
            return (ctx)->fail(SAGA_ERR_HIP, "%s failed: %s (%s:%d)", #call,                \
                               hipGetErrorString(e__), __FILE__, __LINE__);                  \
    } while (0)

// ---------------------------------------------------------------------------
// kernel launchers (each validates nothing: callers check shapes first)
// ---------------------------------------------------------------------------
// internal ApplyEdge code beside the public saga_edge_op values: the gradient of a gated message with
// respect to the gate's argument (see the edge functions in gather.hip)
constexpr int32_t kGatherOpGateGrad = 100;
// ... and that gradient together with the message-part gradient, from one pass, into out / out2
constexpr int32_t kGatherOpGateBoth = 101;
// gradient of a max Gather: a vertex receives w_e * (gradient at the other end) over the edges whose maximum it supplied
constexpr int32_t kGatherOpMaxGrad = 102;
// the two gate gradients of a gated layer under the max accumulator: only where the edge's message is the maximum that
// was gathered at its destination (kGatherOpGateGrad with a third constant row `dst3` = that maximum; kGatherOpGateBoth
// with a third row per edge `src3`)
constexpr int32_t kGatherOpGateGradMax = 103;
constexpr int32_t kGatherOpGateBothMax = 104;

struct GatherArgs {
    const WorkItem* items;
    int64_t n_items;
    int64_t n_team;          // items [0, n_team) are processed by a whole workgroup each
    const int32_t* row_idx;  // source ids, local to the rows of `src`
    const float* edge_w;     // nullable (COPY)
    // LINEAR ops: src = X (dtype), ld_src elements between rows, F features.
    // Gated forms (fp32): per edge, row u of `src` (x) and of `src2` (m); per item, row v of `dst` (c1)
    // and, for kGatherOpGateGrad, of `dst2` (c2). Forward: src = Ps, src2 = M, dst = Pd, all inside the
    // hoisted rows [Ps | M | Pd] with ld 3F.
    const void* src;
    int64_t ld_src;
    const void* src2;        // gated forms only
    int64_t ld_src2;
    const float* dst;        // gated forms only
    int64_t ld_dst;
    const float* dst2;       // kGatherOpGateGrad only
    int64_t ld_dst2;
    const float* dst3;       // kGatherOpGateGradMax only
    int64_t ld_dst3;
    const void* src3;        // kGatherOpGateBothMax only
    int64_t ld_src3;
    int32_t F;
    int32_t dtype;           // saga_dtype of src (GATED: F32)
    int32_t op;              // saga_edge_op
    int32_t agg;             // saga_agg
    float* out;              // fp32 rows of the output interval (nullable if out16 given)
    int64_t ld_out;
    uint16_t* out16;         // optional bf16 copy of the rows (nullable)
    int64_t ld_out16;
    float* out2;             // kGatherOpGateBoth only: the second row (fp32), with its own partial rows
    int64_t ld_out2;
    float* partials2;
    float* partials;         // n_slots x F fp32
    int32_t accumulate;      // 1: combine with what `out` already holds (streamed, chunk i > 0)
    int32_t xcd_remap;
    int32_t mma;             // 1: bf16 sums over linear messages may run their multiply-accumulate on the matrix unit
    int32_t dst_sigmoid;     // kGatherOpMaxGrad: `dst` holds pre-activations, the item's own row is their sigmoid (pooled rows)
    // transform-first layers: the gathered rows are already X W, so ApplyVertex's bias and activation are applied
    // to every finished row (whole-column items here, cut columns in the combine pass); not with `accumulate`
    const float* bias;       // [F] fp32, nullable
    int32_t act;             // saga_act
};
hipError_t launch_gather(const GatherArgs& a, hipStream_t s);

struct CombineArgs {
    const HeavyVertex* heavy;
    int64_t n_heavy;
    const float* partials;
    int32_t F;
    int32_t agg;
    float* out;
    int64_t ld_out;
    uint16_t* out16;
    int64_t ld_out16;
    int32_t accumulate;
    const float* bias;       // as in GatherArgs
    int32_t act;
};
hipError_t launch_combine(const CombineArgs& a, hipStream_t s);

// The dense blocks of a bf16 sum layer on the matrix cores (hybrid.hip): one workgroup per chunk of blocks of one
// destination tile; each of its four wavefronts owns 128 of the features; partial rows go to `partials`.
struct DenseArgs {
    const DenseChunk* chunks;
    int64_t n_chunks;
    const int32_t* blk_src_tile;
    const int32_t* blk_e0;
    const int32_t* blk_tile;        // per block: index of its finished operand in de_tiles, or -1 (edge list)
    const uint16_t* de_tiles;       // finished operands, kDenseTileElems bf16 values each (16-byte aligned)
    const uint16_t* de_pos;
    const uint32_t* de_w;           // per list edge: the weight as two bf16 parts, high | low << 16 (w = high + low to 2^-17)
    const int32_t* src_tile_ids;
    const int32_t* tile_row_slot0;  // 64 per destination tile: first partial row of that destination, -1 where the tile has no vertex
    const uint16_t* X;              // bf16 rows
    int64_t ld;
    int32_t F;                      // a multiple of 128
    int32_t use_low;                // 0: the low parts are all zero (COPY) and their products are skipped
    float* partials;
};
hipError_t launch_dense_blocks(const DenseArgs& a, hipStream_t s);
// de_w[i] = two-part bf16 of w[de_edge[i]], de_tiles[dt_addr[i]] (and kDenseM * kDenseK further) = the two parts of
// w[dt_edge[i]], rem_w[i] = w[rem_edge[i]]; w NULL stands for all ones (and leaves rem_w alone)
struct PackArgs {
    const float* w;
    const int32_t* de_edge;
    int64_t n_list;
    uint32_t* de_w;
    const int32_t* dt_edge;
    const int32_t* dt_addr;
    int64_t n_tile;
    uint16_t* de_tiles;
    const int32_t* rem_edge;
    int64_t n_rem;
    float* rem_w;
};
hipError_t launch_pack_hybrid_weights(const PackArgs& a, hipStream_t s);

// rows x cols fp32 fill / max-identity fix-up for streamed max-Gather
hipError_t launch_fill_f32(float* p, int64_t count, float value, hipStream_t s);
hipError_t launch_neg_inf_to_zero(float* p, int64_t count, hipStream_t s);
hipError_t launch_f32_to_bf16(const float* in, uint16_t* out, int64_t count, hipStream_t s);

// Validate row_idx column by column: ids in [0, n_src), strictly ascending inside each
// column. *flag (device int32, pre-zeroed) is set nonzero on violation.
hipError_t launch_validate_columns(const int64_t* col_ptr, int64_t n_cols, const int32_t* row_idx,
                                   int64_t n_src, int32_t* flag, hipStream_t s);

// C[M x N] = act(A[M x K] * Bt[N x K]^T + bias), fp32 accumulation on MFMA.
// Bt must be padded: rows to a multiple of 128 and K to a multiple of 16 bytes
// worth of elements * 4 (see pack_*), zero-filled.
struct GemmArgs {
    const void* A;      // M x K, dtype
    int64_t lda;
    const void* A2;     // optional second operand, M x K2: C = act(A Bt[:, :Kp]^T + A2 Bt[:, Kp:]^T + bias),
    int64_t lda2;       // Kp = K padded to the K tile (bt_padded_shape)
    int32_t K2;
    int32_t tiled_only;  // 1: always k_gemm_nt, whatever M: rows of one product formed in calls of different sizes are then the same bits
    const void* Bt;     // Npad x Kpad, dtype, row n = column n of the weight matrix
    int64_t ldbt;       // = Kpad
    const float* bias;  // [N] fp32, nullable
    void* C;            // M x N, out_dtype
    int64_t ldc;
    int64_t M;
    int32_t N, K;
    int32_t dtype;      // of A and Bt
    int32_t out_dtype;  // of C
    int32_t act;
    // optional: the product over a list of M rows. Row i of the product reads row row_ids[i] of A and writes row
    // row_ids[i] of C. The list is 16-byte aligned device memory of M rounded up to a multiple of 64 entries, the last
    // entry repeated. Only where gemm_takes_row_list says so (the fp32 kernel with the weights resident in LDS).
    const int32_t* row_ids;
};
hipError_t launch_gemm(const GemmArgs& a, hipStream_t s);
bool gemm_takes_row_list(const GemmArgs& a);  // a with row_ids set: would launch_gemm run it?
// The dense-block form of a bf16 sum propagation (hybrid.hip) over one edge order of a graph: the plan and its device
// copy (ensure_hybrid; view->hyb.usable says whether the graph has blocks worth it), whether a call qualifies
// (hybrid_applies: options, rows of a multiple of 128 bf16 values, 16-byte aligned), the launch of the dense half
// (hybrid_dense_launch) and the release of the plan.
saga_status ensure_hybrid(saga_ctx* ctx, saga_graph* view, int64_t row_bytes, int32_t width = 0);
bool hybrid_applies(const saga_ctx* ctx, int32_t F, int64_t ld, const void* rows);
saga_status hybrid_dense_launch(saga_ctx* ctx, saga_graph* view, GatherArgs* ga, bool weighted, const float* w_src, bool w_attached,
                                saga_ctx::EventSet* es, bool* forked);
void hybrid_free(saga_ctx* ctx, HybridDevice* h);

// Size (elements) of a padded Bt for N x K.
void bt_padded_shape(int32_t N, int32_t K, int32_t dtype, int64_t* n_pad, int64_t* k_pad);
// Bt[n][col0 + k] = W[k][n] for n < N, k < K (W is K x N row-major with ldw). Writes only those
// entries: zero the padded Bt first. dtype in = dtype out.
hipError_t launch_pack_bt_transpose(const void* W, int64_t ldw, int32_t K, int32_t N, int32_t dtype,
                                    void* Bt, int64_t ldbt, int64_t col0, hipStream_t s);
// Bt rows [row0, row0 + R) = Wsrc[r][col0 .. col0 + K) (already output-channel major); Wsrc NULL = identity.
hipError_t launch_pack_bt_rows(const float* Wsrc, int64_t ldw, int64_t col0, int32_t R, int32_t K,
                               float* Bt, int64_t ldbt, int64_t row0, hipStream_t s);
// Bt rows [0, R) = Wsrc[r][0 .. K), bf16
hipError_t launch_pack_bt_rows_bf16(const uint16_t* Wsrc, int64_t ldw, int32_t R, int32_t K, uint16_t* Bt, int64_t ldbt, hipStream_t s);
// Stage-by-stage baseline: S[e] = fp32(X[src e]) (Scatter), S[e] *= w_e (ApplyEdge, skipped without weights), iota[e] = e
hipError_t launch_stage_scatter_apply(const void* X, int64_t ldx, int32_t dtype, const int32_t* src, const float* edge_w, float* S,
                                      int32_t* iota, int32_t F, int64_t n_edges, hipStream_t s);
hipError_t launch_zero_bytes(void* p, size_t bytes, hipStream_t s);

// C[FP x FQ] = P^T Q over n rows (fp32), the rows divided over n_split ranges of
// rows_per_split (a multiple of 16) whose partials land in `part` (n_split x FP x FQ floats)
// and are then added in order into C. gemm_tn_plan picks the division.
struct GemmTnArgs {
    const float* P;
    int64_t ldp;
    const float* Q;
    int64_t ldq;
    int64_t n;
    int64_t rows_per_split;
    float* part;
    int32_t FP, FQ;
    int32_t n_split;
    int32_t pad_;
};
void gemm_tn_plan(int64_t n, int32_t FP, int32_t FQ, int64_t* rows_per_split, int32_t* n_split);
hipError_t launch_gemm_tn(const GemmTnArgs& a, float* C, int64_t ldc, int accumulate, hipStream_t s);  // accumulate: C += P^T Q
// One pass over the gradient rows: dZ (rows x F, row stride lddz, 0 = compact) = dY times the derivative of activation
// `act` taken from the layer's output Y (ReLU: 1 where Y > 0; sigmoid: Y (1 - Y); SAGA_ACT_NONE: Y is not read, nothing
// is stored, dZ is dY); with part (colsum_slabs(rows) x F floats), dbias[c] = sum over rows of dZ[r][c].
int64_t colsum_slabs(int64_t rows);
hipError_t launch_dz_colsum(const float* dY, int64_t lddy, const float* Y, int64_t ldy, int32_t act, float* dZ, int64_t rows, int32_t F,
                            float* part, float* dbias, int accumulate, hipStream_t s, int64_t lddz = 0);  // accumulate: dbias += the sums
// bf16 layers: dZ (rows x F, compact) = dY where Y > 0 (Y NULL: dY), as fp32 and as bf16
hipError_t launch_dz_bf16(const uint16_t* dY, int64_t lddy, const uint16_t* Y, int64_t ldy, float* dZ32, uint16_t* dZ16, int64_t rows,
                          int32_t F, hipStream_t s);
hipError_t launch_permute_f32(const float* in, const int32_t* perm, float* out, int64_t count, hipStream_t s);
// d[i] *= h[i] * (1 - h[i]): a gradient taken through a sigmoid whose outputs are h (both compact, count elements)
hipError_t launch_sigmoid_grad(float* d, const float* z, int64_t count, hipStream_t s);  // d *= sigmoid'(z)
hipError_t launch_copy_bytes(void* dst, const void* src, size_t bytes, hipStream_t s);

// resident graph: make the work list for rows of `row_bytes` current (saga_api.hip)
saga_status ensure_work_list(saga_ctx* ctx, saga_graph* g, int64_t row_bytes, int32_t width = 0);
// per-vertex products of a gated ApplyEdge into ctx->ws_hoist, rows [Ps | M | Pd (+ b)] (saga_api.hip)
// g (nullable): the resident graph whose edges will read the rows; with it, rows of vertices that are no edge's endpoint
// are left unwritten where the product kernel can take a list of rows
saga_status hoist_gated(saga_ctx* ctx, const saga_tensor* X, const saga_edge_params* ep, int64_t n, int32_t F, saga_graph* g = nullptr);
saga_status ensure_endpoints(saga_ctx* ctx, saga_graph* g);
// per-vertex messages of a max-pooling ApplyEdge into ctx->ws_hoist, n x Fm (saga_api.hip)
// act: SAGA_ACT_SIGMOID for the pooled rows themselves, SAGA_ACT_NONE for their pre-activations (backward pass)
saga_status hoist_pool(saga_ctx* ctx, const saga_tensor* X, const saga_edge_params* ep, int64_t n, int32_t F, int32_t Fm,
                       int32_t act = SAGA_ACT_SIGMOID, saga_graph* g = nullptr);
// backward pass of a resident layer (backward.hip)
saga_status resident_backward(saga_ctx* ctx, saga_graph* g, const saga_tensor* X, const saga_tensor* A, const saga_tensor* Y,
                              const saga_tensor* dY, const saga_edge_params* ep, int32_t agg, const saga_vertex_params* vp,
                              const saga_layer_grads* grads);
saga_status resident_backward_bf16(saga_ctx* ctx, saga_graph* g, const saga_tensor* X, const saga_tensor* A, const saga_tensor* Y, const saga_tensor* dY,
                                   const saga_edge_params* ep, const saga_vertex_params* vp, const saga_layer_grads* grads);
// backward pass of a streamed layer: tensors in host memory, host graph (backward.hip)
saga_status streamed_gated_backward(saga_ctx* ctx, saga_graph* g, const saga_tensor* X, const saga_tensor* A, const saga_tensor* Y,
                                    const saga_tensor* dY, const saga_edge_params* ep, int32_t agg, const saga_vertex_params* vp,
                                    const saga_layer_grads* grads);
saga_status streamed_max_pool_backward(saga_ctx* ctx, saga_graph* g, const saga_tensor* X, const saga_tensor* A, const saga_tensor* Y,
                                       const saga_tensor* dY, const saga_edge_params* ep, int32_t agg, const saga_vertex_params* vp,
                                       const saga_layer_grads* grads);
saga_status streamed_backward(saga_ctx* ctx, saga_graph* g, const saga_tensor* X, const saga_tensor* A, const saga_tensor* Y,
                              const saga_tensor* dY, const saga_edge_params* ep, const saga_vertex_params* vp, const saga_layer_grads* grads);
void transposed_graph_destroy(saga_ctx* ctx, saga_graph* g);
// new edge data on a host graph: carried over into the edge order by source (if it exists) and into that order's tiling
saga_status transposed_host_refresh_weights(saga_ctx* ctx, saga_graph* g);

// streamed path (chunked.hip)
// A VertexFeed replaces the plain host-to-device copy of a source interval's rows: fill() enqueues on `s` whatever leaves
// rows [row0, row0 + rows) of the vertex data in dst (rows x F, compact). It is called once per (destination interval,
// source interval) pair in schedule order, also for pairs without edges the first time an interval is seen
// (first_visit), and adds the bytes it copies to *h2d. bytes_per_row: device bytes it holds per row of an interval,
// for the planner. With a feed, X only supplies the shape and the paper's schedule is used.
struct VertexFeed {
    std::function<saga_status(int64_t row0, int64_t rows, float* dst, hipStream_t s, bool first_visit, int64_t* h2d)> fill;
    size_t bytes_per_row = 0;
};
// What the streamed schedule needs beyond a linear layer. Gated layers: the rows that travel are the hoisted rows
// [Ps | M] (2F wide; X gives their shape, a feed or a host array the values), the accumulator rows are acc_width = F
// wide, and the destination parts Pd of every destination interval are made resident from dst_rows, or by dst_fill,
// while the interval is worked on. W_self layers: the interval's own rows of the
// layer input are copied in tile by tile for the second operand of the ApplyVertex product.
struct StreamExtras {
    int32_t acc_width = 0;             // 0: as wide as X's rows
    const float* dst_rows = nullptr;   // host, n rows of acc_width values, ld_dst elements apart: per-destination rows kept
    int64_t ld_dst = 0;                // beside the accumulators of the resident interval (gated; backward of a max Gather)
    int32_t op = 0;                    // 0: ep->op; else an internal edge function of the propagation kernel whose rows
                                       // [x | m] travel (2 * acc_width wide) and whose constant row is dst_rows
    // the gate-gradient edge functions take two constant rows per destination: dst_width = 2 * acc_width makes the
    // resident rows [c1 | c2]; they come from dst_rows alone (its rows are then 2 * acc_width wide) or, with dst2_rows,
    // c1 from dst_rows and c2 from dst2_rows
    int32_t dst_width = 0;             // 0: acc_width
    const float* dst2_rows = nullptr;  // host, n rows of acc_width values, ld_dst2 elements apart
    int64_t ld_dst2 = 0;
    // instead of dst_rows: produces the constant rows of destinations [row0, row0 + rows) in dst (dst_width wide,
    // compact) on stream s and adds the bytes it copies to *h2d (a gated layer forms Pd of the interval from its rows of X)
    std::function<saga_status(int64_t row0, int64_t rows, float* dst, hipStream_t s, int64_t* h2d)> dst_fill;
    bool dst_sigmoid = false;          // the constant rows are pre-activations of pooled rows (GatherArgs::dst_sigmoid)
    int32_t n_out = 1;                 // 2: the edge function has two outputs; accumulator rows are [out | out2]
    // called once per destination interval after its last chunk, before ApplyVertex, with the interval's accumulator
    // rows on the device (compute stream s): the backward pass of pooled messages goes through the sigmoid there
    std::function<saga_status(int64_t row0, int64_t rows, float* acc, hipStream_t s, int64_t* h2d)> after_gather;
    size_t bytes_per_dst_row = 0;      // device bytes after_gather holds per row of a destination interval, for the planner
    const float* self_rows = nullptr;  // host, n rows of F_self, ld_self elements apart (W_self)
    int64_t ld_self = 0;
    int32_t F_self = 0;
    // instead of self_rows: produces rows [row0, row0 + rows) of the second operand (F_self wide, compact) in dst on
    // stream s and adds the bytes it copies to *h2d (the streamed backward pass forms the interval's own dZ there)
    std::function<saga_status(int64_t row0, int64_t rows, float* dst, hipStream_t s, int64_t* h2d)> self_fill;
    // the caller's accum_out: host, n rows of acc_width values, ld_accum elements apart; every destination interval's Gather
    // output is copied there on the outbound stream once its ApplyVertex products have been enqueued
    float* accum_rows = nullptr;
    int64_t ld_accum = 0;
};
saga_status streamed_forward(saga_ctx* ctx, saga_graph* g, const saga_tensor* X, const saga_edge_params* ep,
                             int32_t agg, const saga_vertex_params* vp, saga_tensor* Y, const VertexFeed* feed = nullptr,
                             const StreamExtras* extras = nullptr);
void chunk_grid_destroy(saga_ctx* ctx, ChunkGrid* grid);
// The per-vertex products of a gated or pooled ApplyEdge (Section 3.2) formed on the device from rows of a host X, for
// the streamed calls: init packs the weights (gated: rows [W_gs ; W_m ; W_gd] and the gate bias behind W_gd's rows;
// pooled: W_pool and its bias) into buffers of the context and waits for that; rows copies rows [row0, row0 + rows) of
// X into *tmp (grown to rows x F floats once) and writes tmp x (n_cols rows of the packed weights from row w0 on)^T
// + bias, through `act`, to dst with row stride ldc, all on stream `on`.
struct VertexProducts {
    saga_ctx* ctx = nullptr;
    const saga_tensor* X = nullptr;
    int32_t F = 0;
    float* bt = nullptr;
    float* bias = nullptr;
    int64_t k_pad = 0;
    // under the max accumulator: one product kernel for every interval size, because the backward pass forms these rows
    // again, in intervals of its own, and compares the messages made from them with the forward pass's maxima bit for bit
    bool one_kernel = false;
    saga_status init(saga_ctx* c, const saga_tensor* x, const saga_edge_params* ep);
    saga_status rows(DevBuf* tmp, int64_t row0, int64_t n_rows, int32_t w0, int32_t n_cols, int32_t act, float* dst, int64_t ldc,
                     hipStream_t on, int64_t* h2d) const;
};
void chunk_grid_drain(saga_ctx* ctx);  // wait for everything a (failed) streamed call enqueued
// new edge data on a host graph whose tiling exists: the weights inside the tiling's pinned payloads are written again
void chunk_grid_refresh_weights(saga_graph* g);

// shared by api and chunked: ApplyVertex on a block of rows already on the device
// Xself / ld_self / F_self: the vertices' own rows for vp->W_self (ignored when that is NULL)
saga_status run_apply_vertex(saga_ctx* ctx, const void* A, int64_t lda, int32_t a_dtype, int64_t rows,
                             int32_t F_in, const saga_vertex_params* vp, const void* Xself, int64_t ld_self,
                             int32_t F_self, void* Y, int64_t ldy, int32_t y_dtype);

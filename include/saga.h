/*
 * saga.h - C ABI of the MI355X (gfx950) SAGA-NN layer library.
 *
 * One call computes the forward pass (saga_layer_forward) or the backward pass
 * (saga_layer_backward) of one GNN layer in the SAGA-NN model of the NGra paper
 * (arXiv 1810.08403, Section 2.1-2.2):
 *
 *   Scatter     every edge u -> v receives [src = X[u], dest = X[v], data = w_e]
 *   ApplyEdge   per-edge function of that tuple (closed set below)
 *   Gather      per destination vertex, sum or element-wise max of the edge
 *               outputs ("commutative and associative accumulate", Section 2.2)
 *   ApplyVertex Y[v] = act(A[v] W [+ X[v] W_self] + bias)   (Figures 2, 9 and 10)
 *
 * Scatter, ApplyEdge and Gather run as one fused propagation kernel (the
 * fused-gather operator of Section 3.2); vertex-only matrix products inside a
 * gated ApplyEdge are hoisted to one product per vertex (Section 3.2); graphs
 * whose data live in host memory are streamed through a fixed device budget
 * as vertex intervals x edge chunks (Section 3.1). The backward stages
 * (backward-ApplyVertex, -Gather, -ApplyEdge, -Scatter, Section 2.2) run the
 * same propagation kernel over the edges grouped by source.
 *
 * The paper does not let users supply Scatter/Gather functions or accumulators
 * (Section 2.2, last paragraphs); accordingly everything here is a closed enum.
 *
 * Conventions
 *   - Edge direction: u = source, v = destination. The graph is CSC sorted by
 *     destination (Section 3.1: "edges clustered by destination vertex id"):
 *     the in-edges of v are row_idx[col_ptr[v] .. col_ptr[v+1]), source ids
 *     strictly ascending. Duplicate edges are therefore not representable.
 *   - All matrices are row-major; ld counts elements between rows.
 *   - Pointers marked "device" must be device memory of the context's GPU;
 *     "host" pointers are ordinary or pinned host memory. The caller owns every
 *     buffer it passes; the library never frees or resizes caller memory and
 *     owns only what its handles allocate (released by the *_destroy calls).
 *   - Device-path calls enqueue work on the context's stream and return without
 *     waiting; host-path (streamed) calls return after the output is in host
 *     memory.
 *   - No call throws or aborts; every failure is a saga_status, with text in
 *     saga_last_error().
 *   - A context and the handles made from it are not thread-safe.
 */
#ifndef SAGA_H
#define SAGA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct saga_ctx saga_ctx;     /* device, stream, workspace, budget, timers */
typedef struct saga_graph saga_graph; /* validated CSC, degree bins, work list, chunk grid */

typedef enum {
    SAGA_OK = 0,
    SAGA_ERR_INVALID_ARG = 1, /* null pointer, shape/dtype/placement mismatch */
    SAGA_ERR_BAD_GRAPH = 2,   /* malformed CSC */
    SAGA_ERR_UNSUPPORTED = 3, /* a combination this build does not implement */
    SAGA_ERR_BUDGET = 4,      /* no chunk plan fits the device-memory budget */
    SAGA_ERR_HIP = 5,         /* a HIP runtime call failed */
    SAGA_ERR_INTERNAL = 6
} saga_status;

typedef enum { SAGA_F32 = 0, SAGA_BF16 = 1 } saga_dtype;
typedef enum { SAGA_AGG_SUM = 0, SAGA_AGG_MAX = 1 } saga_agg;
typedef enum { SAGA_ACT_NONE = 0, SAGA_ACT_RELU = 1, SAGA_ACT_SIGMOID = 2 } saga_act;
typedef enum { SAGA_MEM_DEVICE = 0, SAGA_MEM_HOST = 1 } saga_mem;

/*
 * ApplyEdge functions (m = message of edge u -> v, per feature f):
 *   COPY        m = x_u                                   (CommNet, Figure 9)
 *   MUL_WEIGHT  m = w_e * x_u, one fp32 multiply          (GCN, Figure 10)
 *   GATED       m = sigmoid(Wg [x_u ; x_v] + b) (.) (Wm x_u)
 *               (Example 2.1 / Figure 2; b and Wm optional, so that b = NULL,
 *               Wm = NULL is exactly Example 2.1)
 *   POOL        m = sigmoid(Wp x_u + bp), F_pool values per edge (max-pooling GCN,
 *               Figure 11, whose sigma is read as the logistic sigmoid); it depends on
 *               the source only, so it is computed once per vertex (Section 3.2)
 * The message width Fm is F_pool for POOL and F_in otherwise: Gather output, accum_out and
 * the rows of W have that width.
 */
typedef enum { SAGA_EDGE_COPY = 0, SAGA_EDGE_MUL_WEIGHT = 1, SAGA_EDGE_GATED = 2, SAGA_EDGE_POOL = 3 } saga_edge_op;

/* Row-major matrix view. dtype is a saga_dtype, mem a saga_mem. */
typedef struct saga_tensor {
    void* data;
    int64_t rows, cols, ld;
    int32_t dtype;
    int32_t mem;
} saga_tensor;

typedef struct saga_edge_params {
    int32_t op;               /* saga_edge_op */
    const float* edge_weight; /* MUL_WEIGHT: [nnz] fp32 in CSC edge order, same placement as the
                                 graph; NULL = use the data attached by saga_graph_set_edge_data */
    const saga_tensor* W_gate; /* GATED: F x 2F fp32; columns [0,F) act on the source row,
                                  [F,2F) on the destination row */
    const saga_tensor* b_gate; /* GATED: 1 x F fp32, nullable */
    const saga_tensor* W_msg;  /* GATED: F x F fp32 (row = output channel), nullable = identity */
    const saga_tensor* W_pool; /* POOL: F_pool x F fp32 (row = output channel) */
    const saga_tensor* b_pool; /* POOL: 1 x F_pool fp32, nullable */
} saga_edge_params;

typedef struct saga_vertex_params {
    const saga_tensor* W;    /* Fm x F_out, dtype of X; NULL skips ApplyVertex (Y = Gather output) */
    const saga_tensor* bias; /* 1 x F_out fp32, nullable */
    int32_t act;             /* saga_act */
    int32_t reserved;
    const saga_tensor* W_self; /* F_in x F_out, dtype of X, nullable: Y = act(A W + X W_self + bias), the
                                  ApplyVertex of CommNet, ReLU(W_H (x) vertex + W_C (x) accum) (Figure 9),
                                  with W_self = W_H and W = W_C */
} saga_vertex_params;

/* Accumulated since saga_reset_timings(); stage times come from events on the context's stream. */
typedef struct saga_timings {
    int64_t n_calls;         /* saga_layer_forward calls accumulated */
    double ms_total;         /* first to last event of each call, summed */
    double ms_hoist;         /* per-vertex gate/message products (gated only) */
    double ms_gather;        /* fused Scatter-ApplyEdge-Gather kernels */
    double ms_combine;       /* combining the partial rows of split heavy vertices */
    double ms_apply_vertex;  /* ApplyVertex product + activation */
    int64_t n_gather_launches;
    int64_t bytes_h2d, bytes_d2h; /* streamed path only */
    double ms_wall_streamed;      /* host wall time of streamed calls */
    int32_t plan_dst_intervals, plan_src_intervals; /* last streamed plan (0 = resident) */
    int32_t reserved;
    int64_t n_work_items, n_split_vertices; /* of the last graph used */
    double ms_dense_blocks;  /* the part of ms_gather spent in the dense-block kernel (option "dense_blocks") */
    int64_t n_dense_blocks, n_dense_edges; /* of the last layer that used the dense-block path, else 0 */
    int64_t n_partial_rows;  /* partial rows (of the row width, fp32) the last layer wrote and combined */
    int64_t n_hoist_row_cols; /* rows x columns of per-vertex products (Section 3.2) the last gated or pooled resident layer
                                 formed: below n x 3F (n x F_pool) where rows of vertices that are no edge's endpoint were left out */
} saga_timings;

/*
 * Create a context on GPU `device`. hip_stream is a hipStream_t to enqueue on
 * (NULL: the library creates its own, default priority). hbm_budget_bytes caps
 * every device byte the library holds for streamed calls (0 = no cap).
 */
saga_status saga_create(saga_ctx** out, int device, void* hip_stream, size_t hbm_budget_bytes);
saga_status saga_destroy(saga_ctx* ctx);

/*
 * Ingest a CSC graph (Section 3.1). col_ptr is int64 [n_vertices + 1], row_idx
 * int32 [n_edges]; `where` says where both live. The library copies what it
 * needs, so the caller may free the arrays after return. It validates the
 * arrays (monotone col_ptr from 0 to n_edges, ids in range, strictly ascending
 * within a column) and returns SAGA_ERR_BAD_GRAPH otherwise. The work list
 * (light columns whole, heavy columns cut into consecutive sub-groups as in
 * Section 3.3's Scatter kernel) is built at the first call that uses the graph,
 * because the cuts depend on the width of the rows to gather.
 * SAGA_MEM_DEVICE graphs serve device-resident calls; SAGA_MEM_HOST graphs
 * serve streamed calls and are tiled into the chunk grid at the first call.
 * Synchronises the stream.
 */
saga_status saga_graph_create_csc(saga_ctx* ctx, int64_t n_vertices, int64_t n_edges,
                                  const int64_t* col_ptr, const int32_t* row_idx, int32_t where,
                                  saga_graph** out);
saga_status saga_graph_destroy(saga_graph* g);

/*
 * Attach the static edge data (edge.data of Section 2.1, e.g. GCN's degree
 * weights): [n_edges] fp32 in CSC edge order, same placement as the graph.
 * Copied. Used when saga_edge_params.edge_weight is NULL; required for
 * streamed MUL_WEIGHT calls, where it is stored chunk by chunk with the edges.
 * May be called again at any time between layer calls: a host graph that
 * already has its tiling (and its edge order by source) keeps both and only the
 * weights inside their pinned payloads are written again, in place.
 */
saga_status saga_graph_set_edge_data(saga_graph* g, const float* edge_weight);

/*
 * One layer forward. X is n x F_in (SAGA_F32, or SAGA_BF16 for COPY /
 * MUL_WEIGHT). Y is n x F_out in X's dtype (n x Fm when vp->W is NULL).
 * accum_out, if given, receives the Gather output A as n x Fm fp32 before
 * ApplyVertex: a SAGA_MEM_DEVICE tensor on the resident path, a SAGA_MEM_HOST one on the
 * streamed path (every destination interval's rows are copied out after the interval's
 * ApplyVertex products have been enqueued; the call then follows the paper's schedule whatever
 * the "schedule" option says).
 *
 * Placement selects the path: all tensors SAGA_MEM_DEVICE with a device graph
 * -> resident; X and Y SAGA_MEM_HOST (pinned recommended) with a host graph ->
 * streamed through the context's budget, parameters still on the device. Streamed calls
 * cover all four layer programs in fp32: for GATED and POOL the per-vertex products
 * (Section 3.2) are formed on the device as the rows of X arrive (a source interval's rows
 * of X are multiplied into the interval buffer: [Ps | M], or the pooled rows; for GATED the
 * destination parts Pd of the resident interval are formed beside its accumulator from the
 * interval's own rows of X), so the host link carries X only; with W_self the interval's own
 * rows of X are copied in tile by tile for the second operand of the ApplyVertex product.
 * Resident calls form the per-vertex products for edge endpoints only where that saves at least
 * an eighth of them (the source parts for vertices with out-edges, the destination part for
 * vertices with in-edges; the lists are built at the first GATED or POOL call on the graph,
 * which synchronises the stream).
 *
 * Arithmetic: fp32 accumulation everywhere. BF16: X, W bf16; A is rounded to
 * bf16 (nearest even) once before the ApplyVertex product; Y is rounded to
 * bf16. Gather over an empty in-edge set gives 0 for both accumulators.
 * max over MUL_WEIGHT / COPY messages is exact (bitwise reproducible);
 * sums are deterministic run to run (no floating-point atomics).
 */
saga_status saga_layer_forward(saga_ctx* ctx, const saga_graph* g, const saga_tensor* X,
                               const saga_edge_params* ep, int32_t agg,
                               const saga_vertex_params* vp, saga_tensor* Y, saga_tensor* accum_out);

/*
 * The resident forward layer for callers that must not allocate: code under HIP graph
 * capture, tight serving loops, harnesses that forbid it. Same arguments, same kernels
 * and same results as saga_layer_forward, but everything the layer needs beyond its inputs
 * and outputs (the Gather output, the partial rows of cut columns, the packed weights, the
 * per-vertex products of gated and pooled layers) lives in one static device array of
 * 64 MiB (67,108,864 bytes) that the library holds on every GPU it runs on until the
 * process ends. The call reaches no hipMalloc / hipFree and no other allocating routine,
 * and records no stage timings.
 *   - Device tensors and a device graph only (SAGA_ERR_UNSUPPORTED otherwise).
 *   - The work list for this row width must exist already: call saga_layer_forward once with
 *     the same shapes first, else SAGA_ERR_UNSUPPORTED (building it allocates).
 *   - A layer whose scratch needs exceed 64 MiB is refused with SAGA_ERR_BUDGET and a
 *     message; nothing has been enqueued then.
 *   - Every call on one GPU, from any context, uses that GPU's one array and finds the last
 *     call's contents in it (the call overwrites what it reads): calls that overlap on one
 *     GPU race. Enqueue them on one stream, or wait between them.
 */
saga_status saga_layer_forward_noalloc(saga_ctx* ctx, const saga_graph* g, const saga_tensor* X,
                                       const saga_edge_params* ep, int32_t agg,
                                       const saga_vertex_params* vp, saga_tensor* Y, saga_tensor* accum_out);

/*
 * Gradients a backward call writes (each overwritten, not added to). All fp32, device.
 */
typedef struct saga_layer_grads {
    saga_tensor* dX;      /* n x F_in: gradient of the layer's input; NULL = not wanted (first layer) */
    saga_tensor* dW;      /* F_in x F_out: required */
    saga_tensor* dbias;   /* F_out values; NULL = not wanted */
    saga_tensor* dW_self; /* F_in x F_out: required exactly when vp->W_self is given */
    /* GATED layers only (NULL otherwise) */
    saga_tensor* dW_gate; /* F x 2F, laid out like W_gate: required */
    saga_tensor* db_gate; /* F values; NULL = not wanted */
    saga_tensor* dW_msg;  /* F x F, laid out like W_msg; NULL = not wanted; only when W_msg is given */
    /* POOL layers only (NULL otherwise) */
    saga_tensor* dW_pool; /* F_pool x F, laid out like W_pool: required */
    saga_tensor* db_pool; /* F_pool values; NULL = not wanted */
} saga_layer_grads;

/*
 * One layer backward (the backward stages of Section 2.2, run in reverse order of the
 * forward ones): fp32, ApplyVertex Y = act(A W + X W_self + bias) with act NONE, RELU or
 * SIGMOID, everything device-resident. Covered: sum and max accumulator, each with COPY,
 * MUL_WEIGHT, GATED or POOL messages, each with or without W_self. Under the max accumulator
 * an edge carries gradient for the features whose maximum it supplied (every maximal edge
 * on a tie, the whole gradient each); the messages are recomputed by the forward pass's own
 * expressions and compared with A bit for bit, so A must be that pass's accum_out: of a
 * resident forward call for a resident backward call, of a streamed one for a streamed one
 * (the per-vertex products of GATED and POOL layers are formed by different kernels on the two
 * paths, whose sums may differ in the last bit).
 *
 *   backward-ApplyVertex   dZ = dY (.) act'(Z), the derivative taken from the stored output
 *                          (ReLU: 1 where Y > 0; sigmoid: Y (1 - Y), whose error is that of
 *                          the fp32 Y it is formed from: about 2^-24 |dY| Y |1 - 2Y|),
 *                          dW = A^T dZ, dW_self = X^T dZ,  dbias = column sums of dZ,
 *                          gradient of accum = dZ W^T, own partial gradient = dZ W_self^T
 *   backward-Gather, backward-ApplyEdge, backward-Scatter, fused the way the forward
 *   propagation is: dX[u] = sum over out-edges u -> v of w_e * (gradient of accum)[v]
 *                           + own partial gradient[u]
 *
 * A is the Gather output of the forward call (its accum_out), kept by the caller as the
 * intermediate feature data back-propagation needs (Section 3.1). X is read only for
 * dW_self and may be NULL without W_self; Y is read only for the activation's derivative and
 * may be NULL with SAGA_ACT_NONE.
 * The transposed edge order (out-edges grouped by source) and its work list are built at
 * the first backward call on a graph, which synchronises the stream. Because the
 * propagation is linear, it runs at the narrower of F_in and F_out: when F_out <= F_in the
 * rows of dZ are propagated first and multiplied by W^T afterwards (the operator motion of
 * Section 3.2 applied to the backward pass); the result is the same up to rounding order.
 *
 * What the propagation part does, by layer (u -> v an edge, dA = gradient of accum):
 *
 *   layer                  per edge                                    passes over the edges          then, per vertex                          needs
 *   ---------------------  ------------------------------------------  -----------------------------  ----------------------------------------  ---------
 *   sum, COPY/MUL_WEIGHT   dX[u] += w_e dA[v]                          out-edges, once                (own partial gradient joins dX)           A
 *   sum, GATED             s_e = W_gs x_u + W_gd x_v + b, g_e =        in-edges: dPd[v] += ds_e;      dX = [dPs|dM|dPd] [W_gs;W_m;W_gd]         A, X
 *   (Example 2.1, Fig. 2)  sigmoid(s_e), t_u = W_m x_u;                out-edges: dPs[u] += ds_e and  (+ dZ W_self^T as a second operand        
 *                          dt_e = g_e (.) dA[v],                       dM[u] += dt_e in one pass;     pair), dW_gate = [dPs^T X | dPd^T X],     
 *                          ds_e = dA[v] (.) t_u (.) g_e (.) (1 - g_e)  gates recomputed from the      db_gate = column sums of dPd,             
 *                                                                      hoisted products (Sec. 3.2)    dW_msg = dM^T X                           
 *   max, COPY/MUL_WEIGHT   dX[u][f] += w_e dA[v][f] where the message  out-edges, once                (own partial gradient written into dX     A, X
 *   (Figure 11's Gather)   w_e x_u[f], one fp32 multiply as in the                                    before the propagation adds to it)        
 *                          forward pass, equals A[v][f]                                                                                          
 *   max or sum, POOL       as above on the pooled rows h_u =           out-edges, once                dPre = dS (.) sigmoid'(z), slope formed   A, X
 *   (Figure 11)            sigmoid(z_u); z_u = W_pool x_u + b is                                      from z (a saturated unit keeps its        
 *                          recomputed per vertex by the forward                                       relative accuracy); dX = dPre W_pool      
 *                          pass's product and sigmoid                                                 (+ dZ W_self^T), dW_pool = dPre^T X,      
 *                                                                                                     db_pool = column sums of dPre             
 *   max, GATED             the GATED rows, only for the features f     as sum, GATED; A[v] travels    as sum, GATED                             A, X
 *                          where g_e[f] t_u[f] equals A[v][f]          as a third row                                                           
 *
 * Under the max accumulator a tie gives every maximal edge the whole gradient, and A must be
 * the accum_out of the forward call on the same inputs, or no message will compare equal.
 *
 * Streamed calls (a SAGA_MEM_HOST graph, fp32; every layer of the table): A, Y, dY, grads->dX (and X, where the resident call reads it) are SAGA_MEM_HOST
 * tensors (pinned recommended), the parameters and their gradients stay on the device. Every
 * transfer goes through the context's device budget like in saga_layer_forward. The passes:
 *
 *   layer                  passes
 *   ---------------------  --------------------------------------------------------------------------------------------
 *   sum, COPY/MUL_WEIGHT   one: the forward chunk schedule of Section 3.1 on the chunks of edges clustered by source
 *                          (the CSR side of the paper's chunk layout, built at the first such call), dZ as vertex data,
 *                          W^T as the ApplyVertex matrix. dZ is formed on the way in (an interval's rows of dY, and of Y
 *                          with an activation, turned into dZ in place); the first time an interval comes by, its rows
 *                          of A (and of X with W_self) come too and its share of dW, dbias (dW_self) is added, interval
 *                          by interval in a fixed order; dZ W_self^T is the second operand pair of the last product.
 *                          Without grads->dX only this backward-ApplyVertex part runs, over tiles of rows.
 *   max; POOL              three: tiles of rows for backward-ApplyVertex, which also send dA out to pinned host memory of
 *                          the library's own; the schedule over the edges clustered by source, in which rows [A | dA]
 *                          travel and the vertex's own row (x_u, or its pooled row formed on the device from the
 *                          interval's rows of X) sits beside the accumulator for the max decision (sum over pooled rows:
 *                          dA travels as plain vertex data); per interval, while its sums are on the device, the
 *                          sigmoid's slope, dW_pool, db_pool and dX = dPre W_pool.
 *   sum, GATED             three: the tile pass; the schedule over the in-edges (rows [Ps | M] travel, [Pd | dA] of the
 *                          resident interval are the constants: dPd, and per interval its share of dW_gate's right half
 *                          and of db_gate); the schedule over the edges clustered by source (rows [Pd | dA] travel,
 *                          [Ps | M] are the constants, both source-side sums at once; per interval the shares of
 *                          dW_gate's left half and of dW_msg; the last product is dX = [dPs | dM] [W_gs ; W_m] + dPd W_gd).
 *                          Ps, M, Pd are formed on the device from the rows of X of the interval that needs them.
 *   max, GATED             as sum, GATED, with the rows of A beside the rows of dA wherever those go: [Pd | dA | A] of the
 *                          resident interval over the in-edges, [Pd | dA | A] travelling over the out-edges. Ps, M, Pd
 *                          come from the same product kernel as in the streamed forward call, whatever the interval
 *                          size, so the messages formed again are that call's bits.
 *   W_self in the above    dW_self is added tile by tile with dW; dZ W_self^T is a second operand pair of the product
 *                          that ends the last pass (beside the identity for a plain max Gather, W_pool for pooled rows,
 *                          appended to dPd W_gd for gated ones).
 *
 * BF16 layers (W in SAGA_BF16; sum over COPY / MUL_WEIGHT messages, with or without W_self,
 * act NONE or RELU): X is needed only with W_self (bf16, like W_self); Y, dY and grads->dX are
 * bf16 like W, A stays the fp32 accum_out of the forward call, parameter gradients are fp32
 * (dW_self = X^T dZ from the rows of X widened to fp32; dZ W_self^T is a second operand pair of
 * the bf16 product that makes dX, which then always follows the propagation). dZ's bf16 values
 * are used as they are; the rows that travel over the edges and the product that makes dX are
 * bf16 with fp32 accumulation and one rounding to bf16 each, like the forward pass; dW and
 * dbias are fp32 products and sums.
 * Sums are deterministic run to run.
 */
saga_status saga_layer_backward(saga_ctx* ctx, const saga_graph* g, const saga_tensor* X,
                                const saga_tensor* A, const saga_tensor* Y, const saga_tensor* dY,
                                const saga_edge_params* ep, int32_t agg, const saga_vertex_params* vp,
                                const saga_layer_grads* grads);

/* Stage timers. Off by default (no events recorded). */
saga_status saga_set_profiling(saga_ctx* ctx, int32_t on);
saga_status saga_reset_timings(saga_ctx* ctx);
saga_status saga_get_timings(saga_ctx* ctx, saga_timings* out); /* synchronises the stream */

/* Tunables, for measurement. They shape the work list, which is (re)built at the next
 * saga_layer_forward that finds them changed:
 *   "split"      minimum edges in one piece of a cut column (default 64; until the caller sets it, layers whose
 *                propagation writes rows of fewer than 512 features, and whose source rows do not all fit the L2s,
 *                use 32, and the sparse remainder of the
 *                dense-block path uses 48 for source rows of 1 KiB or more)
 *   "cut_degree" columns with more in-edges than this are cut (default 0 = 2 * split)
 *   "stripe_kb"  pieces end where the source rows cross a multiple of this many KiB of
 *                feature rows, and pieces are processed band by band (default 1024;
 *                0 = cut by edge count only)
 *   "piece_order" 0/1 (default 1): the order of the pieces inside the list. 0: by the band of a piece's
 *                first source, then by column. 1: by the band of its first source, then the band of its last
 *                one, then by column, so that the pieces that run at the same time reach over the same rows.
 *                Results do not depend on it.
 *   "team"       0/1, a piece of a cut column is worked by a whole workgroup whose four
 *                wavefronts reduce through LDS, and holds at least 4 * split edges (default 0:
 *                fewer partial rows, but measured slower than one wavefront per piece)
 *   "xcd_remap"  0/1, keep neighbouring work items on one XCD (default 1)
 *   "mma"        0/1 (default 0): sums over COPY / MUL_WEIGHT messages of bf16 rows of 264..512 features
 *                form `acc += w_e * x` on the matrix unit instead of the vector ALUs. Edge weights enter
 *                as two bf16 parts (w = hi + lo to 2^-18 relative); products and sums stay fp32. A
 *                non-finite feature then turns up to 32 features of the destination row into NaN, not one.
 *                Measured: 40 % fewer vector-ALU instructions, the same time (the kernel waits for the L2).
 *   "dst_intervals" / "src_intervals"  streamed plan override, 0 = automatic. k intervals hold
 *                ceil(n / k) vertices each; where that leaves the last ones empty (7 vertices,
 *                k = 5) the plan has only the intervals that hold vertices (4), and
 *                saga_get_timings reports that number. More intervals than vertices:
 *                SAGA_ERR_INVALID_ARG.
 *   "schedule"   streamed calls: 0 = the paper's schedule (Section 3.1: an accumulator chunk
 *                stays on the device until its ApplyVertex has consumed it); the two baselines
 *                the paper measures against (Section 6.2): 1 = stage by stage (all Gather
 *                first, accumulators swapped out to the host and back for ApplyVertex),
 *                2 = destination order innermost (a source chunk stays, accumulators are
 *                swapped in and out around every edge chunk)
 *   "transform_first"  0/1 (default 0): device-resident layers with a linear ApplyEdge (COPY, MUL_WEIGHT), the
 *                sum accumulator, an ApplyVertex product that narrows the rows (F_out < F_in), no W_self and no
 *                accum_out compute Y = act(sum_e w_e (x_u W) + bias): the product first, then the propagation
 *                at F_out values per edge. The same function (the linear stages commute; the operator motion
 *                of Section 3.2 taken one step further), with a different rounding order: sums are taken over
 *                rows of X W rounded to X's dtype. Off by default because it leaves the paper's stage order.
 *   "fused"      0/1 (default 1): 0 runs Scatter, ApplyEdge and Gather of device-resident COPY / MUL_WEIGHT layers
 *                as separate stages through a per-edge tensor of n_edges x F fp32 values held by the context
 *                (the propagation without the fused operator of Section 3.2, the baseline of Section 6.2); other
 *                messages return SAGA_ERR_UNSUPPORTED in this mode, a tensor above 128 GiB or the budget
 *                SAGA_ERR_BUDGET. Max results are the same bits as the fused ones, sums differ in rounding order.
 *   "dense_blocks"  0/1 (default 1): device-resident sum layers over COPY / MUL_WEIGHT messages of bf16 rows of a multiple
 *                of 128 features. Destinations ranked by in-degree and sources by out-degree cut the adjacency matrix
 *                into 64 x 32 blocks; the well-filled ones (the heavy corner of a power-law graph) are multiplied as
 *                dense products on the matrix cores, each source row read once per block instead of once per edge, the
 *                weights as two bf16 parts (2^-17 relative); the other edges stay with the sparse propagation kernel.
 *                Same function, another rounding order; sums stay reproducible run to run. The plan is built at the
 *                first call that can use it. The resident backward pass does not use it.
 *   "dense_min_edges"  edges from which a block goes to the matrix cores (0 = default 200; at most 2048)
 *   "dense_tile_gain"  edges beyond dense_min_edges, summed over the blocks of a destination tile, from which the tile
 *                uses the dense path at all (it costs a partial row per destination; -1 = default 512)
 *   "dense_chunk"  blocks of one destination tile worked by one workgroup (0 = default 128)
 *   "dense_overlap"  0/1 (default 0): 1 runs the dense kernel on a second stream beside the sparse kernel (measured:
 *                no gain, the two fill the chip one after the other)
 *   "bwd_tile_rows"  streamed backward calls: rows per tile of the backward-ApplyVertex pass (default 0 = as
 *                many as make the widest tile about 64 MiB)
 *   "overlap"    streamed calls: 1 = copies on their own streams, overlapping the kernels
 *                (default); 0 = everything on one stream (streaming off)
 * Returns INVALID_ARG for unknown names or values. */
saga_status saga_set_option(saga_ctx* ctx, const char* name, int64_t value);

/* High-water mark of device bytes held by the library (workspace, graph copies, stream buffers). */
size_t saga_peak_device_bytes(const saga_ctx* ctx);
/* Text of the last failure on this context; owned by the context, valid until its next call. */
const char* saga_last_error(const saga_ctx* ctx);
/* Facts about an ingested graph: *max_in_degree, and *n_work_items, *n_split_vertices of the
 * work list built by the last call that used the graph (0 before any). Any may be NULL. */
saga_status saga_graph_info(const saga_graph* g, int64_t* max_in_degree, int64_t* n_work_items,
                            int64_t* n_split_vertices);
/*
 * Plain device-to-device copy kernel (16 bytes per lane, each byte read once and written
 * once), enqueued on the context's stream. It exists to calibrate memory-traffic counters:
 * what a profiler reads for a copy of known size is the scale for what it reads for the
 * layer's kernels. bytes must be a multiple of 16, pointers 16-byte aligned device memory.
 */
saga_status saga_copy_bytes(saga_ctx* ctx, void* dst, const void* src, size_t bytes);

/*
 * Host-only planning call (no GPU needed): build the work list of a host CSC the way
 * saga_layer_forward would for the given parameters, and copy up to `capacity` items into
 * items_out as (vertex, first edge, one-past-last edge, partial-row slot or -1) int32
 * quadruples. team = 4: the first *n_team_items items are pieces of cut columns, each worked
 * by the four wavefronts of one workgroup; team = 1: every item is worked by one wavefront.
 * Counts are always returned. Used to test and to inspect the plan.
 */
saga_status saga_plan_work_list(int64_t n_vertices, const int64_t* col_ptr, const int32_t* row_idx,
                                int64_t min_edges, int64_t cut_degree, int64_t stripe_rows, int32_t team,
                                int32_t* items_out, int64_t capacity, int64_t* n_items,
                                int64_t* n_team_items, int64_t* n_split_vertices, int64_t* n_slots);
/*
 * Host-only planning call (no GPU needed): a re-encoding of the vertex ids that evens out the
 * numbers of edges in the edge chunks of a dst_intervals x src_intervals tiling (Section 3.1
 * re-encodes ids, best effort, for that purpose; it does not say how). Here: vertices are ranked
 * by in-degree + out-degree, heaviest first, ties in an order drawn from `seed`, and dealt to the
 * src_intervals id intervals in alternating (boustrophedon) order, so that every interval
 * receives about the same total degree and the runs of heavy vertices that a skewed graph has at
 * neighbouring ids are spread over all intervals. new_id[v] (int32 [n], a permutation of 0..n-1)
 * is the id vertex v gets; the caller relabels its graph, features and edge data. before / after
 * (int64 [3] each, nullable) receive the largest and smallest chunk edge counts and the number of
 * chunks of the tiling with equal intervals, for the given and for the re-encoded ids.
 * Requires 1 <= dst_intervals <= src_intervals <= n.
 */
saga_status saga_plan_reencoding(int64_t n_vertices, const int64_t* col_ptr, const int32_t* row_idx,
                                 int32_t dst_intervals, int32_t src_intervals, uint64_t seed,
                                 int32_t* new_id, int64_t* before, int64_t* after);
const char* saga_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SAGA_H */

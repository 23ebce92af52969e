// Backward pass of one layer (the backward stages of Section 2.2 in reverse order of the
// forward ones). backward-Gather / backward-ApplyEdge / backward-Scatter fuse exactly like
// the forward propagation (Section 3.3): vertex u's gradient is a sum, over its out-edges
// u -> v, of rows taken at v. That is the forward propagation kernel run on the same edges
// grouped by source instead of by destination, so this file builds that second edge order
// and strings the kernels together:
//   - linear ApplyEdge (COPY, MUL_WEIGHT) under the sum accumulator, fp32 and bf16: one
//     propagation at the narrower of the layer's two widths;
//   - gated ApplyEdge: gates recomputed from the hoisted per-vertex products, one
//     propagation by destination and one (two outputs) by source;
//   - max accumulator and pooled messages: the gradient goes to the sources that supplied
//     the maxima, found by recomputing the messages;
//   - streamed layers (tensors in host memory): the chunk schedule of Section 3.1 on the
//     chunks of edges clustered by source, with dZ formed on the way in (linear ApplyEdge,
//     with or without W_self), or, for the max accumulator and pooled messages, with the
//     gradient of accum passing through pinned host memory between a tile pass and the
//     schedule, and a per-interval finish on the device; gated layers run the schedule
//     twice (in-edges, then edges by source), their per-vertex gradients passing through
//     pinned memory as well; the per-vertex products of gated and pooled layers are formed
//     again on the device from the rows of X. In all of them a W_self term adds its
//     gradient tile by tile and its share of dX inside the schedule's last product.
#include <cstring>

#include "saga_internal.h"

void transposed_graph_destroy(saga_ctx* ctx, saga_graph* g)
{
    ctx->dev_free(&g->d_perm);
    if (!g->tr) return;
    saga_graph* t = g->tr;
    if (t->grid) chunk_grid_destroy(ctx, t->grid);
    for (DevBuf* b : {&t->d_row_idx, &t->d_items, &t->d_heavy, &t->d_edge_data}) ctx->dev_free(b);
    hybrid_free(ctx, &t->hyb);
    for (auto& sl : t->saved_lists) {
        ctx->dev_free(&sl.items);
        ctx->dev_free(&sl.heavy);
    }
    delete t;
    g->tr = nullptr;
    g->tr_edge_data_valid = false;
}

// Out-edges grouped by source: a counting sort of the CSC edge list by source id. Walking
// the columns in order keeps every group ascending in destination id, which is the order
// the propagation kernel and the work-list builder expect.
static saga_status ensure_transposed(saga_ctx* ctx, saga_graph* g)
{
    if (g->tr) return SAGA_OK;
    const int64_t n = g->n, nnz = g->nnz;
    saga_graph* t = new (std::nothrow) saga_graph();
    if (!t) return ctx->fail(SAGA_ERR_INTERNAL, "out of host memory");
    t->ctx = ctx;
    t->n = n;
    t->nnz = nnz;
    t->where = SAGA_MEM_DEVICE;
    g->tr = t;
    auto bail = [&](saga_status st) {
        transposed_graph_destroy(ctx, g);
        return st;
    };
    std::vector<int32_t> src, dst, perm;
    try {
        src.resize((size_t)std::max<int64_t>(nnz, 1));
        dst.resize((size_t)std::max<int64_t>(nnz, 1));
        perm.resize((size_t)std::max<int64_t>(nnz, 1));
        t->h_col_ptr.assign((size_t)n + 1, 0);
    } catch (...) {
        return bail(ctx->fail(SAGA_ERR_INTERNAL, "out of host memory"));
    }
    if (nnz > 0) {
        hipError_t e = hipMemcpyAsync(src.data(), g->d_row_idx.p, sizeof(int32_t) * (size_t)nnz, hipMemcpyDeviceToHost, ctx->stream);
        if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
        if (e != hipSuccess) return bail(ctx->fail(SAGA_ERR_HIP, "reading the edge list: %s", hipGetErrorString(e)));
    }
    int64_t* rp = t->h_col_ptr.data();
    for (int64_t e = 0; e < nnz; ++e) ++rp[src[(size_t)e] + 1];
    int64_t maxdeg = 0;
    for (int64_t u = 0; u < n; ++u) {
        maxdeg = std::max(maxdeg, rp[u + 1]);
        rp[u + 1] += rp[u];
    }
    t->max_degree = maxdeg;
    {
        std::vector<int64_t> fill(rp, rp + n);
        const int64_t* cp = g->h_col_ptr.data();
        for (int64_t v = 0; v < n; ++v)
            for (int64_t e = cp[v]; e < cp[v + 1]; ++e) {
                const int64_t pos = fill[(size_t)src[(size_t)e]]++;
                dst[(size_t)pos] = (int32_t)v;
                perm[(size_t)pos] = (int32_t)e;
            }
    }
    saga_status st;
    if ((st = ctx->dev_alloc(&t->d_row_idx, sizeof(int32_t) * (size_t)std::max<int64_t>(nnz, 1)))) return bail(st);
    if ((st = ctx->dev_alloc(&g->d_perm, sizeof(int32_t) * (size_t)std::max<int64_t>(nnz, 1)))) return bail(st);
    if (nnz > 0) {
        hipError_t e = hipMemcpyAsync(t->d_row_idx.p, dst.data(), sizeof(int32_t) * (size_t)nnz, hipMemcpyHostToDevice, ctx->stream);
        if (e == hipSuccess) e = hipMemcpyAsync(g->d_perm.p, perm.data(), sizeof(int32_t) * (size_t)nnz, hipMemcpyHostToDevice, ctx->stream);
        if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);  // the host vectors go out of scope below
        if (e != hipSuccess) return bail(ctx->fail(SAGA_ERR_HIP, "uploading the transposed edge list: %s", hipGetErrorString(e)));
    }
    return SAGA_OK;
}

// Run the propagation kernel (and the combine pass for cut groups) over one edge order of the graph:
// `view` is the graph itself (edges grouped by destination) or its transposed twin (grouped by source).
// ga carries the sources, constants, edge function, width and output; the work list, ids, partial rows
// and launch options are filled in here.
static saga_status run_propagation(saga_ctx* ctx, saga_graph* view, GatherArgs ga, int64_t row_bytes)
{
    hipStream_t s = ctx->stream;
    if (saga_status st = ensure_work_list(ctx, view, row_bytes, ga.F)) return st;
    ga.items = static_cast<const WorkItem*>(view->d_items.p);
    ga.n_items = view->n_items;
    ga.n_team = view->n_team;
    ga.row_idx = static_cast<const int32_t*>(view->d_row_idx.p);
    ga.dtype = SAGA_F32;
    ga.agg = SAGA_AGG_SUM;
    ga.xcd_remap = ctx->opt_xcd_remap;
    ga.mma = ctx->opt_mma;
    const bool two = ga.op == kGatherOpGateBoth || ga.op == kGatherOpGateBothMax;
    if (view->n_slots > 0) {
        if (saga_status st = ctx->dev_alloc(&ctx->ws_partials, sizeof(float) * (size_t)view->n_slots * ga.F * (two ? 2 : 1))) return st;
        ga.partials = static_cast<float*>(ctx->ws_partials.p);
        if (two) ga.partials2 = ga.partials + (size_t)view->n_slots * ga.F;
    }
    HIP_TRY(ctx, launch_gather(ga, s));
    if (view->n_heavy > 0) {
        CombineArgs ca{};
        ca.heavy = static_cast<const HeavyVertex*>(view->d_heavy.p);
        ca.n_heavy = view->n_heavy;
        ca.partials = ga.partials;
        ca.F = ga.F;
        ca.agg = SAGA_AGG_SUM;
        ca.out = ga.out;
        ca.ld_out = ga.ld_out;
        ca.accumulate = ga.accumulate;
        HIP_TRY(ctx, launch_combine(ca, s));
        if (two) {
            ca.partials = ga.partials2;
            ca.out = ga.out2;
            ca.ld_out = ga.ld_out2;
            HIP_TRY(ctx, launch_combine(ca, s));
        }
    }
    return SAGA_OK;
}

// rows of `src` (n x F fp32) propagated backwards over the edges into `out`:
// out[u] (+)= sum over out-edges u -> v of w_e * src[v]
static saga_status propagate_transposed(saga_ctx* ctx, saga_graph* g, const float* edge_w_t, const float* src, int64_t ld_src,
                                        int32_t F, float* out, int64_t ld_out, int32_t accumulate)
{
    GatherArgs ga{};
    ga.edge_w = edge_w_t;
    ga.src = src;
    ga.ld_src = ld_src;
    ga.F = F;
    ga.op = edge_w_t ? SAGA_EDGE_MUL_WEIGHT : SAGA_EDGE_COPY;
    ga.out = out;
    ga.ld_out = ld_out;
    ga.accumulate = accumulate;
    return run_propagation(ctx, g->tr, ga, (int64_t)F * 4);
}

// C[rows x N] = Arows[rows x K] * Wm[N x K]^T (+ A2 * W2[N x K2]^T): weights given with the output
// channel as the row, which is how W (F_in x F_out) looks from dA = dZ W^T
static saga_status rows_times_wt(saga_ctx* ctx, const float* Arows, int64_t lda, int32_t K, const saga_tensor* Wm, const float* A2,
                                 int64_t lda2, int32_t K2, const saga_tensor* W2, int64_t rows, int32_t N, float* C, int64_t ldc)
{
    hipStream_t s = ctx->stream;
    int64_t n_pad, k_pad, k_pad2 = 0;
    bt_padded_shape(N, K, SAGA_F32, &n_pad, &k_pad);
    if (A2) {
        int64_t np2;
        bt_padded_shape(N, K2, SAGA_F32, &np2, &k_pad2);
    }
    const int64_t ldbt = k_pad + k_pad2;
    if (saga_status st = ctx->dev_alloc(&ctx->ws_bt, sizeof(float) * (size_t)(n_pad * ldbt))) return st;
    float* bt = static_cast<float*>(ctx->ws_bt.p);
    HIP_TRY(ctx, launch_zero_bytes(bt, sizeof(float) * (size_t)(n_pad * ldbt), s));
    HIP_TRY(ctx, launch_pack_bt_rows(static_cast<const float*>(Wm->data), Wm->ld, 0, N, K, bt, ldbt, 0, s));
    if (A2) HIP_TRY(ctx, launch_pack_bt_rows(static_cast<const float*>(W2->data), W2->ld, 0, N, K2, bt + k_pad, ldbt, 0, s));
    GemmArgs ga{};
    ga.A = Arows;
    ga.lda = lda;
    ga.A2 = A2;
    ga.lda2 = lda2;
    ga.K2 = K2;
    ga.Bt = bt;
    ga.ldbt = ldbt;
    ga.C = C;
    ga.ldc = ldc;
    ga.M = rows;
    ga.N = N;
    ga.K = K;
    ga.dtype = ga.out_dtype = SAGA_F32;
    ga.act = SAGA_ACT_NONE;
    HIP_TRY(ctx, launch_gemm(ga, s));
    return SAGA_OK;
}

static saga_status param_grad(saga_ctx* ctx, const float* P, int64_t ldp, int32_t FP, const float* Q, int64_t ldq, int32_t FQ,
                              int64_t n, float* C, int64_t ldc, int accumulate = 0, hipStream_t on = nullptr, bool grow = true)
{
    GemmTnArgs ta{};
    ta.P = P;
    ta.ldp = ldp;
    ta.Q = Q;
    ta.ldq = ldq;
    ta.n = n;
    ta.FP = FP;
    ta.FQ = FQ;
    gemm_tn_plan(n, FP, FQ, &ta.rows_per_split, &ta.n_split);
    const size_t need = sizeof(float) * (size_t)ta.n_split * FP * FQ;
    if (grow) {
        if (saga_status st = ctx->dev_alloc(&ctx->ws_splitk, need)) return st;
    } else if (ctx->ws_splitk.bytes < need) {  // inside a pipeline: the caller sized the workspace beforehand
        return ctx->fail(SAGA_ERR_INTERNAL, "split workspace too small");
    }
    ta.part = static_cast<float*>(ctx->ws_splitk.p);
    HIP_TRY(ctx, launch_gemm_tn(ta, C, ldc, accumulate, on ? on : ctx->stream));
    return SAGA_OK;
}

// Everything of a gated layer's backward pass after backward-ApplyVertex's parameter gradients: the gradient of
// accum, the three per-vertex sums of backward-ApplyEdge (gates recomputed from the hoisted products), and the dense
// products that turn them into dX and the ApplyEdge parameter gradients.
// With the max accumulator (`A_max` = the forward Gather output, else NULL) an edge carries gradient only for the
// features whose maximum at its destination it supplied: the two propagation passes then also compare the recomputed
// message with that maximum (a third constant row in the pass over the in-edges, a third row per edge in the pass
// over the out-edges).
static saga_status gated_backward_rest(saga_ctx* ctx, saga_graph* g, const saga_tensor* X, const float* dZ, int64_t lddz,
                                       const saga_edge_params* ep, const saga_vertex_params* vp, const saga_layer_grads* grads,
                                       const saga_tensor* A_max)
{
    const int64_t n = g->n;
    const int32_t F = (int32_t)vp->W->rows, Fo = (int32_t)vp->W->cols;
    hipStream_t s = ctx->stream;
    if (n == 0) {  // sums over nothing: the parameter gradients are zero (the products below write them for zero rows)
        float* dWg0 = static_cast<float*>(grads->dW_gate->data);
        if (saga_status st = param_grad(ctx, nullptr, 3 * (int64_t)F, F, nullptr, F, F, 0, dWg0, grads->dW_gate->ld)) return st;
        if (saga_status st = param_grad(ctx, nullptr, 3 * (int64_t)F, F, nullptr, F, F, 0, dWg0 + F, grads->dW_gate->ld)) return st;
        if (grads->dW_msg)
            if (saga_status st = param_grad(ctx, nullptr, 3 * (int64_t)F, F, nullptr, F, F, 0, static_cast<float*>(grads->dW_msg->data),
                                            grads->dW_msg->ld))
                return st;
        if (grads->db_gate) HIP_TRY(ctx, launch_fill_f32(static_cast<float*>(grads->db_gate->data), F, 0.f, s));
        return SAGA_OK;
    }
    saga_status st;
    // gradient of accum
    if ((st = ctx->dev_alloc(&ctx->ws_grad, sizeof(float) * (size_t)n * F))) return st;
    float* dA = static_cast<float*>(ctx->ws_grad.p);
    if ((st = rows_times_wt(ctx, dZ, lddz, Fo, vp->W, nullptr, 0, 0, nullptr, n, F, dA, F))) return st;
    // the per-vertex products the gates are made of
    if ((st = hoist_gated(ctx, X, ep, n, F, g))) return st;
    if ((st = ctx->dev_alloc(&ctx->ws_dh, sizeof(float) * (size_t)n * 3 * F))) return st;
    const float* H = static_cast<const float*>(ctx->ws_hoist.p);
    float* dH = static_cast<float*>(ctx->ws_dh.p);
    const int64_t ldh = 3 * (int64_t)F;
    const int64_t row_bytes = 2 * (int64_t)F * 4;
    if ((st = ensure_transposed(ctx, g))) return st;

    GatherArgs ga{};
    ga.F = F;
    ga.ld_src = ga.ld_dst = ga.ld_out = ldh;
    // destination part: dPd[v] = sum over in-edges of dA[v] (.) M[u] (.) g (1 - g), g = sigmoid(Ps[u] + Pd[v])
    ga.op = A_max ? kGatherOpGateGradMax : kGatherOpGateGrad;
    ga.src = H;
    ga.src2 = H + F;
    ga.ld_src2 = ldh;
    ga.dst = H + 2 * F;
    ga.dst2 = dA;
    ga.ld_dst2 = F;
    if (A_max) {
        ga.dst3 = static_cast<const float*>(A_max->data);
        ga.ld_dst3 = A_max->ld;
    }
    ga.out = dH + 2 * F;
    if ((st = run_propagation(ctx, g, ga, row_bytes))) return st;
    // source parts, both from one pass over the out-edges (the same two rows are loaded per edge):
    //   dPs[u] = sum of dA[v] (.) M[u] (.) g (1 - g),  dM[u] = sum of g (.) dA[v],  g = sigmoid(Pd[v] + Ps[u])
    ga.op = A_max ? kGatherOpGateBothMax : kGatherOpGateBoth;
    ga.dst3 = nullptr;
    ga.src = H + 2 * F;
    ga.src2 = dA;
    ga.ld_src2 = F;
    if (A_max) {
        ga.src3 = A_max->data;
        ga.ld_src3 = A_max->ld;
    }
    ga.dst = H;
    ga.dst2 = H + F;
    ga.ld_dst2 = ldh;
    ga.out = dH;
    ga.out2 = dH + F;
    ga.ld_out2 = ldh;
    if ((st = run_propagation(ctx, g->tr, ga, row_bytes))) return st;

    // ApplyEdge parameter gradients: [dPs | dM | dPd]^T X in one product (X is read once instead of three times);
    // its three F x F blocks are dW_gate's left half, dW_msg and dW_gate's right half
    const float* Xp = static_cast<const float*>(X->data);
    float* dWg = static_cast<float*>(grads->dW_gate->data);
    if ((st = ctx->dev_alloc(&ctx->ws_tile, sizeof(float) * 3 * (size_t)F * F))) return st;
    float* blocks = static_cast<float*>(ctx->ws_tile.p);
    if ((st = param_grad(ctx, dH, ldh, 3 * F, Xp, X->ld, F, n, blocks, F))) return st;
    const size_t row = sizeof(float) * (size_t)F;
    HIP_TRY(ctx, hipMemcpy2DAsync(dWg, sizeof(float) * (size_t)grads->dW_gate->ld, blocks, row, row, (size_t)F, hipMemcpyDeviceToDevice, s));
    HIP_TRY(ctx, hipMemcpy2DAsync(dWg + F, sizeof(float) * (size_t)grads->dW_gate->ld, blocks + 2 * (size_t)F * F, row, row, (size_t)F,
                                  hipMemcpyDeviceToDevice, s));
    if (grads->dW_msg)
        HIP_TRY(ctx, hipMemcpy2DAsync(grads->dW_msg->data, sizeof(float) * (size_t)grads->dW_msg->ld, blocks + (size_t)F * F, row, row,
                                      (size_t)F, hipMemcpyDeviceToDevice, s));
    if (grads->db_gate) {
        if ((st = ctx->dev_alloc(&ctx->ws_splitk, sizeof(float) * (size_t)colsum_slabs(n) * F))) return st;
        HIP_TRY(ctx, launch_dz_colsum(dH + 2 * F, ldh, nullptr, 0, SAGA_ACT_NONE, nullptr, n, F, static_cast<float*>(ctx->ws_splitk.p),
                                      static_cast<float*>(grads->db_gate->data), 0, s));
    }
    if (!grads->dX) return SAGA_OK;

    // dX = [dPs | dM | dPd] [W_gs ; W_m ; W_gd] (+ dZ W_self^T, the vertex's own partial gradient, as a second operand
    // pair of the same product): one product over 3F (+ F_out)
    int64_t n_pad, k_pad, k_pad2 = 0;
    bt_padded_shape(F, 3 * F, SAGA_F32, &n_pad, &k_pad);
    if (vp->W_self) {
        int64_t np2;
        bt_padded_shape(F, (int32_t)vp->W->cols, SAGA_F32, &np2, &k_pad2);
    }
    const int64_t ldbt = k_pad + k_pad2;
    if ((st = ctx->dev_alloc(&ctx->ws_bt, sizeof(float) * (size_t)(n_pad * ldbt)))) return st;
    float* bt = static_cast<float*>(ctx->ws_bt.p);
    const float* Wg = static_cast<const float*>(ep->W_gate->data);
    HIP_TRY(ctx, launch_zero_bytes(bt, sizeof(float) * (size_t)(n_pad * ldbt), s));
    HIP_TRY(ctx, launch_pack_bt_transpose(Wg, ep->W_gate->ld, F, F, SAGA_F32, bt, ldbt, 0, s));
    if (ep->W_msg)
        HIP_TRY(ctx, launch_pack_bt_transpose(ep->W_msg->data, ep->W_msg->ld, F, F, SAGA_F32, bt, ldbt, F, s));
    else
        HIP_TRY(ctx, launch_pack_bt_rows(nullptr, 0, 0, F, F, bt + F, ldbt, 0, s));
    HIP_TRY(ctx, launch_pack_bt_transpose(Wg + F, ep->W_gate->ld, F, F, SAGA_F32, bt, ldbt, 2 * (int64_t)F, s));
    GemmArgs gm{};
    if (vp->W_self) {
        HIP_TRY(ctx, launch_pack_bt_rows(static_cast<const float*>(vp->W_self->data), vp->W_self->ld, 0, F, (int32_t)vp->W->cols, bt + k_pad,
                                         ldbt, 0, s));
        gm.A2 = dZ;
        gm.lda2 = lddz;
        gm.K2 = (int32_t)vp->W->cols;
    }
    gm.A = dH;
    gm.lda = ldh;
    gm.Bt = bt;
    gm.ldbt = ldbt;
    gm.C = grads->dX->data;
    gm.ldc = grads->dX->ld;
    gm.M = n;
    gm.N = F;
    gm.K = 3 * F;
    gm.dtype = gm.out_dtype = SAGA_F32;
    gm.act = SAGA_ACT_NONE;
    HIP_TRY(ctx, launch_gemm(gm, s));
    return SAGA_OK;
}

// The edge data in the order of the transposed graph: *w_t is NULL for unweighted layers.
static saga_status transposed_weights(saga_ctx* ctx, saga_graph* g, const saga_edge_params* ep, const float** w_t)
{
    *w_t = nullptr;
    if (ep->op != SAGA_EDGE_MUL_WEIGHT || g->nnz == 0) return SAGA_OK;
    hipStream_t s = ctx->stream;
    const int32_t* perm = static_cast<const int32_t*>(g->d_perm.p);
    if (ep->edge_weight) {
        if (saga_status st = ctx->dev_alloc(&ctx->ws_edge_t, sizeof(float) * (size_t)g->nnz)) return st;
        HIP_TRY(ctx, launch_permute_f32(ep->edge_weight, perm, static_cast<float*>(ctx->ws_edge_t.p), g->nnz, s));
        *w_t = static_cast<const float*>(ctx->ws_edge_t.p);
        return SAGA_OK;
    }
    if (!g->tr_edge_data_valid) {
        if (saga_status st = ctx->dev_alloc(&g->tr->d_edge_data, sizeof(float) * (size_t)g->nnz)) return st;
        HIP_TRY(ctx, launch_permute_f32(static_cast<const float*>(g->d_edge_data.p), perm, static_cast<float*>(g->tr->d_edge_data.p),
                                        g->nnz, s));
        g->tr_edge_data_valid = true;
    }
    *w_t = static_cast<const float*>(g->tr->d_edge_data.p);
    return SAGA_OK;
}

// Max accumulator and / or max-pooling messages, after backward-ApplyVertex's parameter gradients: the gradient of
// accum, its way back over the edges (to the sources that supplied the maxima, or, for a sum, to all of them), and for
// pooled messages the way through the per-vertex sigmoid and product.
static saga_status max_pool_backward_rest(saga_ctx* ctx, saga_graph* g, const saga_tensor* X, const saga_tensor* A, const float* dZ,
                                          int64_t lddz, const saga_edge_params* ep, int32_t agg, const saga_vertex_params* vp,
                                          const saga_layer_grads* grads)
{
    const int64_t n = g->n;
    const bool pool = ep->op == SAGA_EDGE_POOL;
    const int32_t Fm = (int32_t)vp->W->rows, Fo = (int32_t)vp->W->cols;
    const int32_t F = pool ? (int32_t)ep->W_pool->cols : Fm;
    hipStream_t s = ctx->stream;
    saga_status st;
    if (n == 0) {
        if (pool) {
            if ((st = param_grad(ctx, nullptr, Fm, Fm, nullptr, F, F, 0, static_cast<float*>(grads->dW_pool->data), grads->dW_pool->ld))) return st;
            if (grads->db_pool) HIP_TRY(ctx, launch_fill_f32(static_cast<float*>(grads->db_pool->data), Fm, 0.f, s));
        }
        return SAGA_OK;
    }
    if (!pool && !grads->dX) return SAGA_OK;

    if ((st = ctx->dev_alloc(&ctx->ws_grad, sizeof(float) * (size_t)n * Fm))) return st;
    float* dA = static_cast<float*>(ctx->ws_grad.p);
    if ((st = rows_times_wt(ctx, dZ, lddz, Fo, vp->W, nullptr, 0, 0, nullptr, n, Fm, dA, Fm))) return st;
    if ((st = ensure_transposed(ctx, g))) return st;
    const float* w_t = nullptr;
    if ((st = transposed_weights(ctx, g, ep, &w_t))) return st;

    // the per-vertex part of the message, and where the gradient with respect to it goes
    const float* S = static_cast<const float*>(X->data);
    int64_t lds = X->ld;
    float* dS = grads->dX ? static_cast<float*>(grads->dX->data) : nullptr;
    int64_t ldds = grads->dX ? grads->dX->ld : 0;
    if (pool) {
        // the pre-activations z = X W_pool^T + b of the pooled rows: the max Gather's way back forms a vertex's pooled row
        // from them (once per work item), and the slope of the sigmoid comes from them further down
        if ((st = hoist_pool(ctx, X, ep, n, F, Fm, SAGA_ACT_NONE))) return st;
        if ((st = ctx->dev_alloc(&ctx->ws_dh, sizeof(float) * (size_t)n * Fm))) return st;
        S = static_cast<const float*>(ctx->ws_hoist.p);
        lds = Fm;
        dS = static_cast<float*>(ctx->ws_dh.p);
        ldds = Fm;
    }
    // without pooling the propagation writes dX itself: the vertex's own partial gradient dZ W_self^T goes in first
    const int32_t own_first = (!pool && vp->W_self) ? 1 : 0;
    if (own_first)
        if ((st = rows_times_wt(ctx, dZ, lddz, Fo, vp->W_self, nullptr, 0, 0, nullptr, n, F, dS, ldds))) return st;
    if (agg == SAGA_AGG_MAX) {
        GatherArgs ga{};
        ga.accumulate = own_first;
        ga.op = kGatherOpMaxGrad;
        ga.F = Fm;
        ga.src = A->data;      // per edge: the maximum gathered at the destination ...
        ga.ld_src = A->ld;
        ga.src2 = dA;          // ... and its gradient
        ga.ld_src2 = Fm;
        ga.dst = S;            // per item: this vertex's own row (pooled: its pre-activations)
        ga.ld_dst = lds;
        ga.dst_sigmoid = pool ? 1 : 0;
        ga.edge_w = w_t;
        ga.out = dS;
        ga.ld_out = ldds;
        if ((st = run_propagation(ctx, g->tr, ga, 2 * (int64_t)Fm * 4))) return st;
    } else {
        if ((st = propagate_transposed(ctx, g, w_t, dA, Fm, Fm, dS, ldds, own_first))) return st;
    }
    if (!pool) return SAGA_OK;

    // through the sigmoid, then the per-vertex product: dPre = dS (.) sigmoid'(z), dW_pool = dPre^T X, db_pool, dX = dPre W_pool.
    // The slope comes from the pre-activations: h (1 - h) from an fp32 h has lost the slope of a saturated unit.
    HIP_TRY(ctx, launch_sigmoid_grad(dS, S, n * (int64_t)Fm, s));
    const float* Xp = static_cast<const float*>(X->data);
    if ((st = param_grad(ctx, dS, Fm, Fm, Xp, X->ld, F, n, static_cast<float*>(grads->dW_pool->data), grads->dW_pool->ld))) return st;
    if (grads->db_pool) {
        if ((st = ctx->dev_alloc(&ctx->ws_splitk, sizeof(float) * (size_t)colsum_slabs(n) * Fm))) return st;
        HIP_TRY(ctx, launch_dz_colsum(dS, Fm, nullptr, 0, SAGA_ACT_NONE, nullptr, n, Fm, static_cast<float*>(ctx->ws_splitk.p),
                                      static_cast<float*>(grads->db_pool->data), 0, s));
    }
    if (!grads->dX) return SAGA_OK;
    // dX = dPre W_pool (+ dZ W_self^T as a second operand pair of the same product)
    int64_t n_pad, k_pad, k_pad2 = 0;
    bt_padded_shape(F, Fm, SAGA_F32, &n_pad, &k_pad);
    if (vp->W_self) {
        int64_t np2;
        bt_padded_shape(F, Fo, SAGA_F32, &np2, &k_pad2);
    }
    const int64_t ldbt = k_pad + k_pad2;
    if ((st = ctx->dev_alloc(&ctx->ws_bt, sizeof(float) * (size_t)(n_pad * ldbt)))) return st;
    float* bt = static_cast<float*>(ctx->ws_bt.p);
    HIP_TRY(ctx, launch_zero_bytes(bt, sizeof(float) * (size_t)(n_pad * ldbt), s));
    HIP_TRY(ctx, launch_pack_bt_transpose(ep->W_pool->data, ep->W_pool->ld, Fm, F, SAGA_F32, bt, ldbt, 0, s));
    GemmArgs gm{};
    if (vp->W_self) {
        HIP_TRY(ctx, launch_pack_bt_rows(static_cast<const float*>(vp->W_self->data), vp->W_self->ld, 0, F, Fo, bt + k_pad, ldbt, 0, s));
        gm.A2 = dZ;
        gm.lda2 = lddz;
        gm.K2 = Fo;
    }
    gm.A = dS;
    gm.lda = Fm;
    gm.Bt = bt;
    gm.ldbt = ldbt;
    gm.C = grads->dX->data;
    gm.ldc = grads->dX->ld;
    gm.M = n;
    gm.N = F;
    gm.K = Fm;
    gm.dtype = gm.out_dtype = SAGA_F32;
    gm.act = SAGA_ACT_NONE;
    HIP_TRY(ctx, launch_gemm(gm, s));
    return SAGA_OK;
}

saga_status resident_backward(saga_ctx* ctx, saga_graph* g, const saga_tensor* X, const saga_tensor* A, const saga_tensor* Y,
                              const saga_tensor* dY, const saga_edge_params* ep, int32_t agg, const saga_vertex_params* vp,
                              const saga_layer_grads* grads)
{
    const int64_t n = g->n;
    const int32_t F = (int32_t)vp->W->rows, Fo = (int32_t)vp->W->cols;  // F: message width (equals X's width except for POOL)
    hipStream_t s = ctx->stream;

    // backward-ApplyVertex: the activation's derivative and the bias gradient in one pass over the rows
    const float* dZ = static_cast<const float*>(dY->data);
    int64_t lddz = dY->ld;
    const bool use_y = vp->act != SAGA_ACT_NONE;  // the activation's derivative is taken from the layer's output
    if (use_y || grads->dbias) {
        float* part = nullptr;
        if (grads->dbias) {
            if (saga_status st = ctx->dev_alloc(&ctx->ws_splitk, sizeof(float) * (size_t)colsum_slabs(n) * Fo)) return st;
            part = static_cast<float*>(ctx->ws_splitk.p);
        }
        if (use_y)
            if (saga_status st = ctx->dev_alloc(&ctx->ws_dz, sizeof(float) * (size_t)std::max<int64_t>(n, 1) * Fo)) return st;
        HIP_TRY(ctx, launch_dz_colsum(dZ, lddz, use_y ? static_cast<const float*>(Y->data) : nullptr, use_y ? Y->ld : 0, vp->act,
                                      static_cast<float*>(ctx->ws_dz.p), n, Fo, part,
                                      grads->dbias ? static_cast<float*>(grads->dbias->data) : nullptr, 0, s));
        if (use_y) {
            dZ = static_cast<const float*>(ctx->ws_dz.p);
            lddz = Fo;
        }
    }

    // parameter gradients
    if (saga_status st = param_grad(ctx, static_cast<const float*>(A->data), A->ld, F, dZ, lddz, Fo, n, static_cast<float*>(grads->dW->data), grads->dW->ld)) return st;
    if (grads->dW_self)  // X is as wide as the messages except for POOL
        if (saga_status st = param_grad(ctx, static_cast<const float*>(X->data), X->ld, (int32_t)X->cols, dZ, lddz, Fo, n, static_cast<float*>(grads->dW_self->data), grads->dW_self->ld)) return st;
    if (ep->op == SAGA_EDGE_GATED) return gated_backward_rest(ctx, g, X, dZ, lddz, ep, vp, grads, agg == SAGA_AGG_MAX ? A : nullptr);
    if (ep->op == SAGA_EDGE_POOL || agg == SAGA_AGG_MAX) return max_pool_backward_rest(ctx, g, X, A, dZ, lddz, ep, agg, vp, grads);
    if (!grads->dX || n == 0) return SAGA_OK;

    // the edges grouped by source, and the edge data in that order
    if (saga_status st = ensure_transposed(ctx, g)) return st;
    const float* w_t = nullptr;
    if (saga_status st = transposed_weights(ctx, g, ep, &w_t)) return st;

    float* dX = static_cast<float*>(grads->dX->data);
    const int64_t lddx = grads->dX->ld;
    if (Fo <= F) {
        // propagate the narrower rows first: dX = (T dZ) W^T + dZ W_self^T, one product with two operands
        if (saga_status st = ctx->dev_alloc(&ctx->ws_grad, sizeof(float) * (size_t)n * Fo)) return st;
        float* G = static_cast<float*>(ctx->ws_grad.p);
        if (saga_status st = propagate_transposed(ctx, g, w_t, dZ, lddz, Fo, G, Fo, 0)) return st;
        return rows_times_wt(ctx, G, Fo, Fo, vp->W, vp->W_self ? dZ : nullptr, lddz, Fo, vp->W_self, n, F, dX, lddx);
    }
    // gradient of accum = dZ W^T, then propagate it; the vertex's own partial gradient goes into dX first
    if (saga_status st = ctx->dev_alloc(&ctx->ws_grad, sizeof(float) * (size_t)n * F)) return st;
    float* dA = static_cast<float*>(ctx->ws_grad.p);
    if (saga_status st = rows_times_wt(ctx, dZ, lddz, Fo, vp->W, nullptr, 0, 0, nullptr, n, F, dA, F)) return st;
    if (vp->W_self)
        if (saga_status st = rows_times_wt(ctx, dZ, lddz, Fo, vp->W_self, nullptr, 0, 0, nullptr, n, F, dX, lddx)) return st;
    return propagate_transposed(ctx, g, w_t, dA, F, F, dX, lddx, vp->W_self ? 1 : 0);
}

// bf16 layers (sum over COPY / MUL_WEIGHT messages): the rows that travel over the edges and through the dX product
// are bf16 with fp32 accumulation, like the forward pass; the parameter gradients are fp32 products of the fp32 Gather
// output (for dW_self: of X widened to fp32) with dZ, whose bf16 values are exact in fp32. With W_self the propagation
// always runs first and dX = [T dZ | dZ] [W ; W_self]^T is one product with two operand pairs.
saga_status resident_backward_bf16(saga_ctx* ctx, saga_graph* g, const saga_tensor* X, const saga_tensor* A, const saga_tensor* Y,
                                   const saga_tensor* dY, const saga_edge_params* ep, const saga_vertex_params* vp,
                                   const saga_layer_grads* grads)
{
    const int64_t n = g->n;
    const int32_t F = (int32_t)vp->W->rows, Fo = (int32_t)vp->W->cols;
    hipStream_t s = ctx->stream;
    saga_status st;
    const size_t nz = (size_t)std::max<int64_t>(n, 1) * Fo;
    if ((st = ctx->dev_alloc(&ctx->ws_dz, sizeof(float) * nz))) return st;
    if ((st = ctx->dev_alloc(&ctx->ws_dz16, sizeof(uint16_t) * nz))) return st;
    float* dZ32 = static_cast<float*>(ctx->ws_dz.p);
    uint16_t* dZ16 = static_cast<uint16_t*>(ctx->ws_dz16.p);
    const bool relu = vp->act == SAGA_ACT_RELU;
    HIP_TRY(ctx, launch_dz_bf16(static_cast<const uint16_t*>(dY->data), dY->ld, relu ? static_cast<const uint16_t*>(Y->data) : nullptr,
                                relu ? Y->ld : 0, dZ32, dZ16, n, Fo, s));
    if (grads->dbias) {
        if ((st = ctx->dev_alloc(&ctx->ws_splitk, sizeof(float) * (size_t)colsum_slabs(n) * Fo))) return st;
        HIP_TRY(ctx, launch_dz_colsum(dZ32, Fo, nullptr, 0, SAGA_ACT_NONE, nullptr, n, Fo, static_cast<float*>(ctx->ws_splitk.p),
                                      static_cast<float*>(grads->dbias->data), 0, s));
    }
    if ((st = param_grad(ctx, static_cast<const float*>(A->data), A->ld, F, dZ32, Fo, Fo, n, static_cast<float*>(grads->dW->data),
                         grads->dW->ld)))
        return st;
    const bool with_self = vp->W_self != nullptr;
    if (with_self) {  // dW_self = X^T dZ, with the rows of X widened to fp32 in the buffer the Gather output uses in forward calls
        if ((st = ctx->dev_alloc(&ctx->ws_accum, sizeof(float) * (size_t)std::max<int64_t>(n, 1) * F))) return st;
        float* X32 = static_cast<float*>(ctx->ws_accum.p);
        HIP_TRY(ctx, launch_dz_bf16(static_cast<const uint16_t*>(X->data), X->ld, nullptr, 0, X32, nullptr, n, F, s));
        if ((st = param_grad(ctx, X32, F, F, dZ32, Fo, Fo, n, static_cast<float*>(grads->dW_self->data), grads->dW_self->ld))) return st;
    }
    if (!grads->dX || n == 0) return SAGA_OK;
    if ((st = ensure_transposed(ctx, g))) return st;
    const float* w_t = nullptr;
    if ((st = transposed_weights(ctx, g, ep, &w_t))) return st;

    // rows x K (bf16) times W^T, W given as F x F_out: C[rows x F] bf16; own: the second operand pair (dZ, W_self)
    auto times_wt16 = [&](const uint16_t* rows16, int64_t ld, uint16_t* C, int64_t ldc, bool own) -> saga_status {
        int64_t n_pad, k_pad;
        bt_padded_shape(F, Fo, SAGA_BF16, &n_pad, &k_pad);
        const int64_t ldbt = own ? 2 * k_pad : k_pad;
        if (saga_status e = ctx->dev_alloc(&ctx->ws_bt, sizeof(uint16_t) * (size_t)(n_pad * ldbt))) return e;
        uint16_t* bt = static_cast<uint16_t*>(ctx->ws_bt.p);
        HIP_TRY(ctx, launch_zero_bytes(bt, sizeof(uint16_t) * (size_t)(n_pad * ldbt), s));
        HIP_TRY(ctx, launch_pack_bt_rows_bf16(static_cast<const uint16_t*>(vp->W->data), vp->W->ld, F, Fo, bt, ldbt, s));
        GemmArgs gm{};
        if (own) {
            HIP_TRY(ctx, launch_pack_bt_rows_bf16(static_cast<const uint16_t*>(vp->W_self->data), vp->W_self->ld, F, Fo, bt + k_pad, ldbt, s));
            gm.A2 = dZ16;
            gm.lda2 = Fo;
            gm.K2 = Fo;
        }
        gm.A = rows16;
        gm.lda = ld;
        gm.Bt = bt;
        gm.ldbt = ldbt;
        gm.C = C;
        gm.ldc = ldc;
        gm.M = n;
        gm.N = F;
        gm.K = Fo;
        gm.dtype = gm.out_dtype = SAGA_BF16;
        gm.act = SAGA_ACT_NONE;
        HIP_TRY(ctx, launch_gemm(gm, s));
        return SAGA_OK;
    };
    auto propagate16 = [&](const uint16_t* src, int64_t ld, int32_t width, uint16_t* out16, int64_t ld_out) -> saga_status {
        GatherArgs ga{};
        ga.edge_w = w_t;
        ga.src = src;
        ga.ld_src = ld;
        ga.F = width;
        ga.op = w_t ? SAGA_EDGE_MUL_WEIGHT : SAGA_EDGE_COPY;
        ga.out16 = out16;
        ga.ld_out16 = ld_out;
        // run_propagation sets dtype to fp32: give the bf16 view its own few lines. As in the forward pass, the well-filled
        // blocks of the adjacency matrix (here of its transpose: sources ranked by out-degree are the rows) go to the
        // matrix cores where the rows allow it, and the sparse kernel keeps the remainder.
        saga_graph* view = g->tr;
        bool hybrid = hybrid_applies(ctx, width, ld, src);
        if (hybrid) {
            if (saga_status e = ensure_hybrid(ctx, view, (int64_t)width * 2, width)) return e;
            hybrid = view->hyb.usable;
        }
        if (!hybrid)
            if (saga_status e = ensure_work_list(ctx, view, (int64_t)width * 2, width)) return e;
        const HybridDevice& h = view->hyb;
        ga.items = static_cast<const WorkItem*>(hybrid ? h.items.p : view->d_items.p);
        ga.n_items = hybrid ? h.n_items : view->n_items;
        ga.n_team = hybrid ? h.n_team : view->n_team;
        ga.row_idx = static_cast<const int32_t*>(hybrid ? h.rem_row_idx.p : view->d_row_idx.p);
        const int64_t n_slots = hybrid ? h.n_slots : view->n_slots, n_heavy = hybrid ? h.n_heavy : view->n_heavy;
        ga.dtype = SAGA_BF16;
        ga.agg = SAGA_AGG_SUM;
        ga.xcd_remap = ctx->opt_xcd_remap;
        ga.mma = ctx->opt_mma;
        if (n_slots > 0) {
            if (saga_status e = ctx->dev_alloc(&ctx->ws_partials, sizeof(float) * (size_t)n_slots * width)) return e;
            ga.partials = static_cast<float*>(ctx->ws_partials.p);
        }
        bool forked = false;
        if (hybrid)  // the weights in the edge order by source: the view's own copy of attached data, or this call's permuted ones
            if (saga_status e = hybrid_dense_launch(ctx, view, &ga, w_t != nullptr, w_t, w_t != nullptr && !ep->edge_weight, nullptr, &forked))
                return e;
        HIP_TRY(ctx, launch_gather(ga, s));
        if (forked) HIP_TRY(ctx, hipStreamWaitEvent(s, ctx->ev_join, 0));
        if (n_heavy > 0) {
            CombineArgs ca{};
            ca.heavy = static_cast<const HeavyVertex*>(hybrid ? h.heavy.p : view->d_heavy.p);
            ca.n_heavy = n_heavy;
            ca.partials = ga.partials;
            ca.F = width;
            ca.agg = SAGA_AGG_SUM;
            ca.out16 = out16;
            ca.ld_out16 = ld_out;
            HIP_TRY(ctx, launch_combine(ca, s));
        }
        return SAGA_OK;
    };

    uint16_t* dX = static_cast<uint16_t*>(grads->dX->data);
    const int64_t lddx = grads->dX->ld;
    const bool first = Fo <= F || with_self;  // propagate dZ, then the product
    const int32_t wmid = first ? Fo : F;
    if ((st = ctx->dev_alloc(&ctx->ws_grad, sizeof(uint16_t) * (size_t)n * wmid))) return st;
    uint16_t* mid = static_cast<uint16_t*>(ctx->ws_grad.p);
    if (first) {
        if ((st = propagate16(dZ16, Fo, Fo, mid, Fo))) return st;   // the narrower rows travel (with W_self: always dZ)
        return times_wt16(mid, Fo, dX, lddx, with_self);
    }
    if ((st = times_wt16(dZ16, Fo, mid, F, false))) return st;
    return propagate16(mid, F, F, dX, lddx);
}

// ---------------------------------------------------------------------------
// streamed layers (Section 3.1): tensors in host memory, host graph
// ---------------------------------------------------------------------------
// The edge order by source of a host graph, with its edge data: the chunk grid the backward propagation streams is
// built from it the way the forward one is built from the graph itself (chunks of edges clustered by source).
static saga_status ensure_transposed_host(saga_ctx* ctx, saga_graph* g)
{
    if (g->tr) return SAGA_OK;
    const int64_t n = g->n, nnz = g->nnz;
    saga_graph* t = new (std::nothrow) saga_graph();
    if (!t) return ctx->fail(SAGA_ERR_INTERNAL, "out of host memory");
    t->ctx = ctx;
    t->n = n;
    t->nnz = nnz;
    t->where = SAGA_MEM_HOST;
    g->tr = t;
    const bool weighted = !g->h_edge_data.empty();
    try {
        t->h_col_ptr.assign((size_t)n + 1, 0);
        t->h_row_idx.resize((size_t)nnz);
        if (weighted) t->h_edge_data.resize((size_t)nnz);
        int64_t* rp = t->h_col_ptr.data();
        const int32_t* src = g->h_row_idx.data();
        for (int64_t e = 0; e < nnz; ++e) ++rp[src[e] + 1];
        int64_t maxdeg = 0;
        for (int64_t u = 0; u < n; ++u) {
            maxdeg = std::max(maxdeg, rp[u + 1]);
            rp[u + 1] += rp[u];
        }
        t->max_degree = maxdeg;
        std::vector<int64_t> fill(rp, rp + n);
        const int64_t* cp = g->h_col_ptr.data();
        for (int64_t v = 0; v < n; ++v)
            for (int64_t e = cp[v]; e < cp[v + 1]; ++e) {
                const int64_t pos = fill[(size_t)src[e]]++;
                t->h_row_idx[(size_t)pos] = (int32_t)v;
                if (weighted) t->h_edge_data[(size_t)pos] = g->h_edge_data[(size_t)e];
            }
    } catch (...) {
        transposed_graph_destroy(ctx, g);
        return ctx->fail(SAGA_ERR_INTERNAL, "out of host memory");
    }
    return SAGA_OK;
}

// New edge data on a host graph whose edge order by source exists already: the same counting pass that built the order
// places every weight again (columns in order keep every group ascending in destination id), then the tiling of that
// order, if there is one, takes the weights over in place. A twin that was built without edge data gets them now; its
// tiling, made for unweighted chunks, is then replaced at the next call that needs weights.
saga_status transposed_host_refresh_weights(saga_ctx* ctx, saga_graph* g)
{
    saga_graph* t = g->tr;
    if (!t || t->where != SAGA_MEM_HOST || g->h_edge_data.empty()) return SAGA_OK;
    const int64_t n = g->n, nnz = g->nnz;
    try {
        t->h_edge_data.resize((size_t)nnz);
        std::vector<int64_t> fill(t->h_col_ptr.begin(), t->h_col_ptr.begin() + n);
        const int64_t* cp = g->h_col_ptr.data();
        const int32_t* src = g->h_row_idx.data();
        for (int64_t v = 0; v < n; ++v)
            for (int64_t e = cp[v]; e < cp[v + 1]; ++e) t->h_edge_data[(size_t)fill[(size_t)src[e]]++] = g->h_edge_data[(size_t)e];
    } catch (...) {
        transposed_graph_destroy(ctx, g);  // rebuilt, with the new data, by the next backward call
        return SAGA_OK;
    }
    chunk_grid_refresh_weights(t);
    return SAGA_OK;
}

// Parameter gradients of a streamed layer without the propagation: backward-ApplyVertex over tiles of rows copied in
// from host memory on the context's stream (dZ, the bias sums, dW += A^T dZ, tile after tile in a fixed order).
// h_dA (optional, pinned host, n x F compact): also receives the gradient of accum, dZ W^T, tile by tile.
static saga_status streamed_param_grads(saga_ctx* ctx, int64_t n, const saga_tensor* X, const saga_tensor* A, const saga_tensor* Y,
                                        const saga_tensor* dY, const saga_vertex_params* vp, const saga_layer_grads* grads,
                                        float* h_dA = nullptr)
{
    const int32_t F = (int32_t)vp->W->rows, Fo = (int32_t)vp->W->cols;
    const int32_t Fx = X ? (int32_t)X->cols : F;  // X is as wide as the messages except for POOL
    const bool use_y = vp->act != SAGA_ACT_NONE;  // the activation's derivative is taken from the layer's output
    hipStream_t s = ctx->stream;
    saga_status st;
    const int64_t t_auto = std::max<int64_t>(4096, ((int64_t)64 << 20) / (4 * (int64_t)std::max(F, Fo)));
    int64_t T = std::max<int64_t>(1, std::min<int64_t>(std::max<int64_t>(n, 1), ctx->opt_bwd_tile_rows > 0 ? ctx->opt_bwd_tile_rows : t_auto));
    if (ctx->budget > 0) {
        // the tiles, the split workspace of the parameter-gradient product (at most 1,024 partial F x F_out matrices, usually
        // far fewer) and the column-sum slabs have to fit beside whatever else the context holds
        const size_t per_row = sizeof(float) * ((size_t)F + 3 * (size_t)Fo + (grads->dW_self ? (size_t)Fx : 0) + (h_dA ? (size_t)F : 0));
        int64_t rps;
        int32_t nsp;
        gemm_tn_plan(T, F, Fo, &rps, &nsp);
        const size_t fixed = sizeof(float) * (size_t)nsp * F * Fo + sizeof(float) * (size_t)colsum_slabs(T) * Fo + (1 << 20);
        ctx->make_room(fixed + per_row * (size_t)T);
        const size_t left = ctx->budget > ctx->cur_bytes + fixed ? ctx->budget - ctx->cur_bytes - fixed : 0;
        T = std::max<int64_t>(64, std::min<int64_t>(T, (int64_t)(left / per_row)));
    }
    if ((st = ctx->dev_alloc(&ctx->ws_accum, sizeof(float) * (size_t)T * F))) return st;   // A tile
    if ((st = ctx->dev_alloc(&ctx->ws_grad, sizeof(float) * (size_t)T * Fo))) return st;   // dY tile
    if (use_y) {
        if ((st = ctx->dev_alloc(&ctx->ws_hoist, sizeof(float) * (size_t)T * Fo))) return st;  // Y tile
        if ((st = ctx->dev_alloc(&ctx->ws_dz, sizeof(float) * (size_t)T * Fo))) return st;     // dZ tile
    }
    if (grads->dbias)
        if ((st = ctx->dev_alloc(&ctx->ws_splitk, sizeof(float) * (size_t)colsum_slabs(T) * Fo))) return st;
    if (grads->dW_self)
        if ((st = ctx->dev_alloc(&ctx->ws_dh, sizeof(float) * (size_t)T * Fx))) return st;  // X tile (dW_self = X^T dZ)
    if (h_dA)
        if ((st = ctx->dev_alloc(&ctx->ws_tile, sizeof(float) * (size_t)T * F))) return st;  // tile of the gradient of accum
    float* tX = static_cast<float*>(ctx->ws_dh.p);
    float* tA = static_cast<float*>(ctx->ws_accum.p);
    float* tdY = static_cast<float*>(ctx->ws_grad.p);
    float* tY = static_cast<float*>(ctx->ws_hoist.p);
    float* tdZ = use_y ? static_cast<float*>(ctx->ws_dz.p) : tdY;
    int64_t h2d = 0, d2h = 0;
    auto rows_at = [](const saga_tensor* t, int64_t r) { return static_cast<const float*>(t->data) + r * t->ld; };
    for (int64_t r0 = 0; r0 < std::max<int64_t>(n, 1); r0 += T) {
        const int64_t rows = std::min(T, n - r0);
        const int acc = r0 > 0;
        if (rows > 0) {
            HIP_TRY(ctx, hipMemcpy2DAsync(tA, sizeof(float) * (size_t)F, rows_at(A, r0), sizeof(float) * (size_t)A->ld,
                                          sizeof(float) * (size_t)F, (size_t)rows, hipMemcpyHostToDevice, s));
            HIP_TRY(ctx, hipMemcpy2DAsync(tdY, sizeof(float) * (size_t)Fo, rows_at(dY, r0), sizeof(float) * (size_t)dY->ld,
                                          sizeof(float) * (size_t)Fo, (size_t)rows, hipMemcpyHostToDevice, s));
            h2d += rows * (int64_t)(F + Fo) * 4;
            if (use_y) {
                HIP_TRY(ctx, hipMemcpy2DAsync(tY, sizeof(float) * (size_t)Fo, rows_at(Y, r0), sizeof(float) * (size_t)Y->ld,
                                              sizeof(float) * (size_t)Fo, (size_t)rows, hipMemcpyHostToDevice, s));
                h2d += rows * (int64_t)Fo * 4;
            }
        }
        if (use_y || grads->dbias)
            HIP_TRY(ctx, launch_dz_colsum(tdY, Fo, use_y ? tY : nullptr, Fo, vp->act, tdZ, rows, Fo,
                                          grads->dbias ? static_cast<float*>(ctx->ws_splitk.p) : nullptr,
                                          grads->dbias ? static_cast<float*>(grads->dbias->data) : nullptr, acc, s));
        if ((st = param_grad(ctx, tA, F, F, tdZ, Fo, Fo, rows, static_cast<float*>(grads->dW->data), grads->dW->ld, acc))) return st;
        if (grads->dW_self) {
            if (rows > 0) {
                HIP_TRY(ctx, hipMemcpy2DAsync(tX, sizeof(float) * (size_t)Fx, rows_at(X, r0), sizeof(float) * (size_t)X->ld,
                                              sizeof(float) * (size_t)Fx, (size_t)rows, hipMemcpyHostToDevice, s));
                h2d += rows * (int64_t)Fx * 4;
            }
            if ((st = param_grad(ctx, tX, Fx, Fx, tdZ, Fo, Fo, rows, static_cast<float*>(grads->dW_self->data), grads->dW_self->ld, acc)))
                return st;
        }
        if (h_dA && rows > 0) {
            float* tDA = static_cast<float*>(ctx->ws_tile.p);
            if ((st = rows_times_wt(ctx, tdZ, Fo, Fo, vp->W, nullptr, 0, 0, nullptr, rows, F, tDA, F))) return st;
            HIP_TRY(ctx, hipMemcpyAsync(h_dA + r0 * F, tDA, sizeof(float) * (size_t)rows * F, hipMemcpyDeviceToHost, s));
            d2h += rows * (int64_t)F * 4;
        }
        // one stream: the next tile's copies queue behind this tile's kernels
    }
    HIP_TRY(ctx, hipStreamSynchronize(s));  // a streamed call returns when the host tensors are the caller's again
    ctx->acc.bytes_h2d += h2d;
    ctx->acc.bytes_d2h += d2h;
    return SAGA_OK;
}

// The second operand rows of a streamed backward pass's last product, for a layer with W_self: tile by tile,
// [pre | dZ] with dZ formed from the tile's rows of dY (and Y, through the activation's derivative; the Y tile passes
// through ctx->ws_dz, max_rows x Fo floats, which the caller allocates) and pre an optional block of pre_w columns
// copied from host rows. The vertex's own partial gradient is then dZ W_self^T inside that product.
static std::function<saga_status(int64_t, int64_t, float*, hipStream_t, int64_t*)>
own_rows_fill(saga_ctx* ctx, const saga_tensor* dY, const saga_tensor* Y, int32_t act, int32_t Fo, const float* pre_rows, int64_t ld_pre,
              int32_t pre_w, int64_t max_rows)
{
    return [=](int64_t row0, int64_t rows, float* dst, hipStream_t on, int64_t* h2d) -> saga_status {
        auto rows_of_t = [](const saga_tensor* t, int64_t r) { return static_cast<const float*>(t->data) + r * t->ld; };
        const int64_t ldd = (int64_t)pre_w + Fo;
        if (rows > max_rows) return ctx->fail(SAGA_ERR_INTERNAL, "own-row tile larger than planned");
        if (pre_w > 0) {
            HIP_TRY(ctx, hipMemcpy2DAsync(dst, sizeof(float) * (size_t)ldd, pre_rows + row0 * ld_pre, sizeof(float) * (size_t)ld_pre,
                                          sizeof(float) * (size_t)pre_w, (size_t)rows, hipMemcpyHostToDevice, on));
            *h2d += rows * (int64_t)pre_w * 4;
        }
        HIP_TRY(ctx, hipMemcpy2DAsync(dst + pre_w, sizeof(float) * (size_t)ldd, rows_of_t(dY, row0), sizeof(float) * (size_t)dY->ld,
                                      sizeof(float) * (size_t)Fo, (size_t)rows, hipMemcpyHostToDevice, on));
        *h2d += rows * (int64_t)Fo * 4;
        if (act != SAGA_ACT_NONE) {
            float* tY = static_cast<float*>(ctx->ws_dz.p);
            HIP_TRY(ctx, hipMemcpy2DAsync(tY, sizeof(float) * (size_t)Fo, rows_of_t(Y, row0), sizeof(float) * (size_t)Y->ld,
                                          sizeof(float) * (size_t)Fo, (size_t)rows, hipMemcpyHostToDevice, on));
            *h2d += rows * (int64_t)Fo * 4;
            HIP_TRY(ctx, launch_dz_colsum(dst + pre_w, ldd, tY, Fo, act, dst + pre_w, rows, Fo, nullptr, nullptr, 0, on, ldd));
        }
        return SAGA_OK;
    };
}

// Streamed backward pass of a layer with the max accumulator (COPY, MUL_WEIGHT or POOL messages) or with pooled messages
// under the sum accumulator; X, A, Y, dY and dX in host memory. Three passes:
//   1. tiles of rows: dZ, dW += A^T dZ, dbias (dW_self), and the gradient of accum dZ W^T out to pinned host memory;
//      pooled rows are formed again on the device, interval by interval, from the rows of X (VertexProducts);
//   2. the chunk schedule over the edges clustered by source. Max: rows [A | gradient of accum] of the destination side
//      travel, the row of the vertex itself (x_u, or its pooled row) sits beside the accumulator, and the edge function
//      is the max-gradient one of the resident pass; sum over pooled rows: the gradient of accum travels as it is;
//   3. per interval, while its sums dS are still on the device: pooled layers go through the sigmoid
//      (dPre = dS (.) sigmoid'(z), the slope formed from the interval's pre-activations), add dPre^T X and the column sums of dPre to dW_pool and db_pool, and the schedule's
//      ApplyVertex product is dX = dPre W_pool; otherwise dS is dX.
saga_status streamed_max_pool_backward(saga_ctx* ctx, saga_graph* g, const saga_tensor* X, const saga_tensor* A, const saga_tensor* Y,
                                       const saga_tensor* dY, const saga_edge_params* ep, int32_t agg, const saga_vertex_params* vp,
                                       const saga_layer_grads* grads)
{
    const int64_t n = g->n;
    const bool pool = ep->op == SAGA_EDGE_POOL;
    const int32_t Fm = (int32_t)vp->W->rows, F = (int32_t)X->cols;
    hipStream_t s = ctx->stream;
    saga_status st;
    const bool propagate = n > 0 && (pool || grads->dX);
    if (propagate) {
        const size_t need = sizeof(float) * (size_t)n * Fm;
        if (ctx->h_grad_bytes < need) {
            if (ctx->h_grad) (void)hipHostFree(ctx->h_grad);
            ctx->h_grad = nullptr;
            ctx->h_grad_bytes = 0;
            HIP_TRY(ctx, hipHostMalloc(reinterpret_cast<void**>(&ctx->h_grad), need, hipHostMallocDefault));
            ctx->h_grad_bytes = need;
        }
    }
    if ((st = streamed_param_grads(ctx, n, X, A, Y, dY, vp, grads, propagate ? ctx->h_grad : nullptr))) return st;
    if (n == 0) {
        if (pool) {
            if ((st = param_grad(ctx, nullptr, Fm, Fm, nullptr, F, F, 0, static_cast<float*>(grads->dW_pool->data), grads->dW_pool->ld))) return st;
            if (grads->db_pool) HIP_TRY(ctx, launch_fill_f32(static_cast<float*>(grads->db_pool->data), Fm, 0.f, s));
            HIP_TRY(ctx, hipStreamSynchronize(s));
        }
        return SAGA_OK;
    }
    if (!propagate) return SAGA_OK;
    for (DevBuf* b : {&ctx->ws_accum, &ctx->ws_grad, &ctx->ws_hoist, &ctx->ws_dz, &ctx->ws_dh, &ctx->ws_tile}) ctx->dev_free(b);
    VertexProducts prod;  // pooled rows are formed on the device from the rows of X, interval by interval
    prod.one_kernel = agg == SAGA_AGG_MAX;
    if (pool)
        if ((st = prod.init(ctx, X, ep))) return st;
    if ((st = ensure_transposed_host(ctx, g))) return st;
    const float* h_dA = ctx->h_grad;
    float* pooled_j = nullptr;  // where dst_fill left the pre-activations of the resident interval's pooled rows (its rows of X are in ws_tile)
    VertexFeed feed;
    StreamExtras ex;
    saga_tensor rows_t{};  // shape of the rows that travel
    rows_t.rows = n;
    rows_t.dtype = SAGA_F32;
    rows_t.mem = SAGA_MEM_HOST;
    saga_edge_params et{};
    et.op = pool ? SAGA_EDGE_COPY : ep->op;  // whether the chunks carry edge data
    if (agg == SAGA_AGG_MAX) {
        rows_t.cols = rows_t.ld = 2 * Fm;
        feed.bytes_per_row = 0;
        feed.fill = [&](int64_t row0, int64_t rows, float* dst, hipStream_t on, bool, int64_t* h2d) -> saga_status {
            // [the maximum gathered at the vertex | its gradient], side by side
            HIP_TRY(ctx, hipMemcpy2DAsync(dst, sizeof(float) * 2 * (size_t)Fm, static_cast<const float*>(A->data) + row0 * A->ld,
                                          sizeof(float) * (size_t)A->ld, sizeof(float) * (size_t)Fm, (size_t)rows, hipMemcpyHostToDevice, on));
            HIP_TRY(ctx, hipMemcpy2DAsync(dst + Fm, sizeof(float) * 2 * (size_t)Fm, h_dA + row0 * Fm, sizeof(float) * (size_t)Fm,
                                          sizeof(float) * (size_t)Fm, (size_t)rows, hipMemcpyHostToDevice, on));
            *h2d += rows * 2 * (int64_t)Fm * 4;
            return SAGA_OK;
        };
        ex.op = kGatherOpMaxGrad;
        ex.acc_width = Fm;
        if (pool) {  // the vertex's own pooled row beside its accumulator
            ex.dst_fill = [&](int64_t row0, int64_t rows, float* dst, hipStream_t on, int64_t* h2d) -> saga_status {
                pooled_j = dst;  // as pre-activations: the kernel forms the pooled row, the slope needs z itself
                return prod.rows(&ctx->ws_tile, row0, rows, 0, Fm, SAGA_ACT_NONE, dst, Fm, on, h2d);
            };
            ex.dst_sigmoid = true;
        } else {
            ex.dst_rows = static_cast<const float*>(X->data);
            ex.ld_dst = X->ld;
        }
    } else {
        rows_t.data = ctx->h_grad;  // sum over pooled rows: the gradient of accum travels unchanged
        rows_t.cols = rows_t.ld = Fm;
    }
    saga_vertex_params vt{};
    saga_tensor wp{}, wst_t{};
    vt.act = SAGA_ACT_NONE;
    const bool with_self = vp->W_self != nullptr;
    if (with_self) {
        // the vertex's own partial gradient dZ W_self^T joins dX as the second operand pair of the schedule's last
        // product (for a plain max Gather that product is otherwise the identity); its rows dZ are formed tile by tile
        const int32_t Fo = (int32_t)vp->W->cols;
        const bool use_y = vp->act != SAGA_ACT_NONE;
        const int64_t self_tile = std::min<int64_t>(n, std::max<int64_t>(4096, ((int64_t)64 << 20) / ((int64_t)F * 4)));
        if ((st = ctx->dev_alloc(&ctx->ws_wt, sizeof(float) * ((size_t)Fo * F + (pool ? 0 : (size_t)F * F))))) return st;
        float* wst = static_cast<float*>(ctx->ws_wt.p);
        HIP_TRY(ctx, launch_pack_bt_transpose(vp->W_self->data, vp->W_self->ld, F, Fo, SAGA_F32, wst, F, 0, s));
        wst_t.data = wst;
        wst_t.rows = Fo;
        wst_t.cols = wst_t.ld = F;
        wst_t.dtype = SAGA_F32;
        wst_t.mem = SAGA_MEM_DEVICE;
        vt.W_self = &wst_t;
        if (!pool) {
            HIP_TRY(ctx, launch_pack_bt_rows(nullptr, 0, 0, F, F, wst + (size_t)Fo * F, F, 0, s));  // identity
            wp = wst_t;
            wp.data = wst + (size_t)Fo * F;
            wp.rows = F;
            vt.W = &wp;
        }
        if (use_y)
            if ((st = ctx->dev_alloc(&ctx->ws_dz, sizeof(float) * (size_t)self_tile * Fo))) return st;
        ex.F_self = Fo;
        ex.self_fill = own_rows_fill(ctx, dY, Y, vp->act, Fo, nullptr, 0, 0, self_tile);
    }
    if (pool) {
        // dX = dPre W_pool: W_pool (F_pool x F) is already the "F_in x F_out" matrix of this product
        wp = *ep->W_pool;
        vt.W = &wp;
        ex.bytes_per_dst_row = sizeof(float) * ((size_t)Fm + F);
        {
            // the split workspace for the largest interval there can be, so that nothing is allocated inside the pipeline;
            // the column sums use it after the product's partial sums have been added up (same stream)
            int64_t rps;
            int32_t nsp;
            gemm_tn_plan(n, Fm, F, &rps, &nsp);
            const size_t need = std::max(sizeof(float) * (size_t)nsp * Fm * F, sizeof(float) * (size_t)colsum_slabs(n) * Fm);
            if ((st = ctx->dev_alloc(&ctx->ws_splitk, need))) return st;
        }
        bool any_done = false;
        ex.after_gather = [&, any_done](int64_t row0, int64_t rows, float* acc, hipStream_t on, int64_t* h2d) mutable -> saga_status {
            // the pre-activations of the interval's pooled rows and its rows of X: left by dst_fill (max), or formed here, on the compute stream
            // (sum: there are no constant rows, and the kernels that follow wait for them anyway)
            float* tS = pooled_j;
            if (agg != SAGA_AGG_MAX) {
                if (saga_status e = ctx->dev_alloc(&ctx->ws_hoist, sizeof(float) * (size_t)rows * Fm)) return e;  // intervals do not grow
                tS = static_cast<float*>(ctx->ws_hoist.p);
                if (saga_status e = prod.rows(&ctx->ws_tile, row0, rows, 0, Fm, SAGA_ACT_NONE, tS, Fm, on, h2d)) return e;
            }
            const float* tX = static_cast<const float*>(ctx->ws_tile.p);
            HIP_TRY(ctx, launch_sigmoid_grad(acc, tS, rows * (int64_t)Fm, on));
            if (saga_status e = param_grad(ctx, acc, Fm, Fm, tX, F, F, rows, static_cast<float*>(grads->dW_pool->data), grads->dW_pool->ld,
                                           any_done ? 1 : 0, on, false))
                return e;
            if (grads->db_pool)
                HIP_TRY(ctx, launch_dz_colsum(acc, Fm, nullptr, 0, SAGA_ACT_NONE, nullptr, rows, Fm,
                                              static_cast<float*>(ctx->ws_splitk.p), static_cast<float*>(grads->db_pool->data),
                                              any_done ? 1 : 0, on));
            any_done = true;
            return SAGA_OK;
        };
    }
    saga_tensor no_dx{};  // pooled layers without dX still need the pass for dW_pool: the schedule then writes nothing out
    return streamed_forward(ctx, g->tr, &rows_t, &et, SAGA_AGG_SUM, (pool || with_self) ? &vt : nullptr, grads->dX ? grads->dX : &no_dx,
                            agg == SAGA_AGG_MAX ? &feed : nullptr, &ex);
}

// Streamed backward pass of a gated layer (sum accumulator); X, A, Y, dY and dX in host memory. The per-vertex products
// [Ps | M | Pd] are formed on the device from the rows of X of the interval that needs them, as in the forward call;
// the gradient of accum and the per-vertex gradients [dPs | dM | dPd] pass through pinned host memory of the library's own:
//   1. tiles of rows: dZ, dW += A^T dZ, dbias, and the gradient of accum dZ W^T out to pinned memory;
//   2. the chunk schedule over the in-edges: rows [Ps | M] travel, [Pd | gradient of accum] of the resident interval sit
//      beside its accumulator, edge function "gate gradient": dPd_j. Per interval: dW_gd += dPd_j^T X_j, db += sums;
//      dPd_j goes out to pinned memory;
//   3. the chunk schedule over the edges clustered by source: rows [Pd | gradient of accum] travel, [Ps | M] of the
//      resident interval are the constants, edge function "both gate gradients": [dPs | dM]_J. Per interval:
//      dW_gs += dPs^T X_J, dW_m += dM^T X_J; the schedule's last product is
//      dX_J = [dPs | dM] [W_gs ; W_m] + dPd_J W_gd, the second pair fed from what pass 2 left in pinned memory.
saga_status streamed_gated_backward(saga_ctx* ctx, saga_graph* g, const saga_tensor* X, const saga_tensor* A, const saga_tensor* Y,
                                    const saga_tensor* dY, const saga_edge_params* ep, int32_t agg, const saga_vertex_params* vp,
                                    const saga_layer_grads* grads)
{
    // Under the max accumulator an edge passes gradient on only where its message is the maximum that was gathered at its
    // destination (A, the forward pass's Gather output, which the caller hands in): the rows of A ride along, as a third
    // constant row of the destination in the in-edge pass and as a third row per edge in the out-edge pass, and the edge
    // functions compare the recomputed message with them bit for bit, as on the resident path.
    const bool is_max = agg == SAGA_AGG_MAX;
    const int64_t n = g->n;
    const int32_t F = (int32_t)X->cols;
    hipStream_t s = ctx->stream;
    saga_status st;
    float* dWg = static_cast<float*>(grads->dW_gate->data);
    const int64_t lddwg = grads->dW_gate->ld;
    if (n > 0) {
        const size_t need = sizeof(float) * (size_t)n * 4 * F;  // gradient of accum (n x F), then [dPs | dM | dPd] (n x 3F)
        if (ctx->h_grad_bytes < need) {
            if (ctx->h_grad) (void)hipHostFree(ctx->h_grad);
            ctx->h_grad = nullptr;
            ctx->h_grad_bytes = 0;
            HIP_TRY(ctx, hipHostMalloc(reinterpret_cast<void**>(&ctx->h_grad), need, hipHostMallocDefault));
            ctx->h_grad_bytes = need;
        }
    }
    const bool with_self = vp->W_self != nullptr;
    const int32_t Fo = (int32_t)vp->W->cols;
    if ((st = streamed_param_grads(ctx, n, with_self ? X : nullptr, A, Y, dY, vp, grads, n > 0 ? ctx->h_grad : nullptr))) return st;
    if (n == 0) {  // sums over nothing
        if ((st = param_grad(ctx, nullptr, 3 * (int64_t)F, F, nullptr, F, F, 0, dWg, lddwg))) return st;
        if ((st = param_grad(ctx, nullptr, 3 * (int64_t)F, F, nullptr, F, F, 0, dWg + F, lddwg))) return st;
        if (grads->dW_msg)
            if ((st = param_grad(ctx, nullptr, 3 * (int64_t)F, F, nullptr, F, F, 0, static_cast<float*>(grads->dW_msg->data), grads->dW_msg->ld)))
                return st;
        if (grads->db_gate) HIP_TRY(ctx, launch_fill_f32(static_cast<float*>(grads->db_gate->data), F, 0.f, s));
        HIP_TRY(ctx, hipStreamSynchronize(s));
        return SAGA_OK;
    }
    for (DevBuf* b : {&ctx->ws_accum, &ctx->ws_grad, &ctx->ws_hoist, &ctx->ws_dz, &ctx->ws_dh, &ctx->ws_tile}) ctx->dev_free(b);
    VertexProducts prod;  // [Ps | M] and Pd of an interval are formed on the device from its rows of X, which stay in
                          // ws_tile (resident interval) for the parameter gradients added up per interval
    prod.one_kernel = is_max;
    if ((st = prod.init(ctx, X, ep))) return st;
    if ((st = ensure_transposed_host(ctx, g))) return st;
    const float* h_dA = ctx->h_grad;               // F per vertex
    float* h_dH = ctx->h_grad + (size_t)n * F;     // [dPs | dM | dPd], 3F per vertex
    const int64_t ldh = 3 * (int64_t)F;
    {
        // the split workspace for the largest interval there can be, so that nothing is allocated inside the pipeline;
        // the column sums use it after a product's partial sums have been added up (same stream)
        int64_t rps;
        int32_t nsp;
        gemm_tn_plan(n, F, F, &rps, &nsp);
        const size_t need = std::max(sizeof(float) * (size_t)nsp * F * F, sizeof(float) * (size_t)colsum_slabs(n) * F);
        if ((st = ctx->dev_alloc(&ctx->ws_splitk, need))) return st;
    }
    saga_edge_params et{};
    et.op = SAGA_EDGE_COPY;  // the chunks carry no edge data; the edge function is named in the extras

    // ---- pass 2: destination parts, over the in-edges ----
    {
        saga_tensor rows_t{};  // shape of the rows that travel, [Ps | M]: the feed forms them from the interval's rows of X
        rows_t.rows = n;
        rows_t.cols = rows_t.ld = 2 * F;
        rows_t.dtype = SAGA_F32;
        rows_t.mem = SAGA_MEM_HOST;
        saga_tensor out_t = rows_t;
        out_t.data = h_dH + 2 * F;
        out_t.cols = F;
        out_t.ld = ldh;
        VertexFeed feed;
        feed.bytes_per_row = sizeof(float) * (size_t)F;
        feed.fill = [&](int64_t row0, int64_t rows, float* dst, hipStream_t on, bool, int64_t* h2d) -> saga_status {
            return prod.rows(&ctx->ws_accum, row0, rows, 0, 2 * F, SAGA_ACT_NONE, dst, 2 * (int64_t)F, on, h2d);
        };
        StreamExtras ex;
        ex.op = is_max ? kGatherOpGateGradMax : kGatherOpGateGrad;
        ex.acc_width = F;
        const int64_t dw = (is_max ? 3 : 2) * (int64_t)F;  // [Pd | gradient of accum] and, under max, the maxima
        ex.dst_width = (int32_t)dw;
        ex.dst_fill = [&, dw](int64_t row0, int64_t rows, float* dst, hipStream_t on, int64_t* h2d) -> saga_status {
            // [Pd | gradient of accum ( | A )] of the resident interval; its rows of X stay in ws_tile for after_gather
            if (saga_status e = prod.rows(&ctx->ws_tile, row0, rows, 2 * F, F, SAGA_ACT_NONE, dst, dw, on, h2d)) return e;
            HIP_TRY(ctx, hipMemcpy2DAsync(dst + F, sizeof(float) * (size_t)dw, h_dA + row0 * F, sizeof(float) * (size_t)F,
                                          sizeof(float) * (size_t)F, (size_t)rows, hipMemcpyHostToDevice, on));
            *h2d += rows * (int64_t)F * 4;
            if (is_max) {
                HIP_TRY(ctx, hipMemcpy2DAsync(dst + 2 * F, sizeof(float) * (size_t)dw, static_cast<const float*>(A->data) + row0 * A->ld,
                                              sizeof(float) * (size_t)A->ld, sizeof(float) * (size_t)F, (size_t)rows, hipMemcpyHostToDevice, on));
                *h2d += rows * (int64_t)F * 4;
            }
            return SAGA_OK;
        };
        ex.bytes_per_dst_row = sizeof(float) * (size_t)F * (is_max ? 2 : 1);
        bool any_done = false;
        ex.after_gather = [&, any_done](int64_t, int64_t rows, float* acc, hipStream_t on, int64_t*) mutable -> saga_status {
            const float* tX = static_cast<const float*>(ctx->ws_tile.p);
            if (saga_status e = param_grad(ctx, acc, F, F, tX, F, F, rows, dWg + F, lddwg, any_done ? 1 : 0, on, false)) return e;
            if (grads->db_gate)
                HIP_TRY(ctx, launch_dz_colsum(acc, F, nullptr, 0, SAGA_ACT_NONE, nullptr, rows, F, static_cast<float*>(ctx->ws_splitk.p),
                                              static_cast<float*>(grads->db_gate->data), any_done ? 1 : 0, on));
            any_done = true;
            return SAGA_OK;
        };
        if ((st = streamed_forward(ctx, g, &rows_t, &et, SAGA_AGG_SUM, nullptr, &out_t, &feed, &ex))) return st;
    }

    // ---- pass 3: source parts and dX, over the edges clustered by source ----
    if ((st = ctx->dev_alloc(&ctx->ws_wt, sizeof(float) * (size_t)F * (2 * (size_t)F + (with_self ? (size_t)F + Fo : 0))))) return st;
    float* M1 = static_cast<float*>(ctx->ws_wt.p);  // [W_gs ; W_m] as a 2F x F matrix: row f of W_gs is W_gate[f][0..F)
    float* M2 = M1 + 2 * (size_t)F * F;             // with W_self: [W_gd ; W_self^T], (F + F_out) x F
    const float* Wg = static_cast<const float*>(ep->W_gate->data);
    HIP_TRY(ctx, launch_pack_bt_rows(Wg, ep->W_gate->ld, 0, F, F, M1, F, 0, s));
    HIP_TRY(ctx, launch_pack_bt_rows(ep->W_msg ? static_cast<const float*>(ep->W_msg->data) : nullptr, ep->W_msg ? ep->W_msg->ld : 0, 0, F, F,
                                     M1, F, F, s));
    const int64_t self_tile = std::min<int64_t>(n, std::max<int64_t>(4096, ((int64_t)64 << 20) / ((int64_t)F * 4)));
    if (with_self) {
        HIP_TRY(ctx, launch_pack_bt_rows(Wg, ep->W_gate->ld, F, F, F, M2, F, 0, s));
        HIP_TRY(ctx, launch_pack_bt_transpose(vp->W_self->data, vp->W_self->ld, F, Fo, SAGA_F32, M2 + (size_t)F * F, F, 0, s));
        if (vp->act != SAGA_ACT_NONE)
            if ((st = ctx->dev_alloc(&ctx->ws_dz, sizeof(float) * (size_t)self_tile * Fo))) return st;
    }
    HIP_TRY(ctx, hipStreamSynchronize(s));
    const int64_t tw = (is_max ? 3 : 2) * (int64_t)F;  // width of the rows that travel
    saga_tensor rows_t{};
    rows_t.rows = n;
    rows_t.cols = rows_t.ld = tw;
    rows_t.dtype = SAGA_F32;
    rows_t.mem = SAGA_MEM_HOST;
    VertexFeed feed;
    feed.bytes_per_row = sizeof(float) * (size_t)F * (is_max ? 2 : 1);
    feed.fill = [&, tw](int64_t row0, int64_t rows, float* dst, hipStream_t on, bool, int64_t* h2d) -> saga_status {
        // [the destination part of the gate's argument | the gradient of accum ( | the maxima )] of the vertices at the far end
        // of the out-edges
        if (saga_status e = prod.rows(&ctx->ws_accum, row0, rows, 2 * F, F, SAGA_ACT_NONE, dst, tw, on, h2d)) return e;
        HIP_TRY(ctx, hipMemcpy2DAsync(dst + F, sizeof(float) * (size_t)tw, h_dA + row0 * F, sizeof(float) * (size_t)F,
                                      sizeof(float) * (size_t)F, (size_t)rows, hipMemcpyHostToDevice, on));
        *h2d += rows * (int64_t)F * 4;
        if (is_max) {
            HIP_TRY(ctx, hipMemcpy2DAsync(dst + 2 * F, sizeof(float) * (size_t)tw, static_cast<const float*>(A->data) + row0 * A->ld,
                                          sizeof(float) * (size_t)A->ld, sizeof(float) * (size_t)F, (size_t)rows, hipMemcpyHostToDevice, on));
            *h2d += rows * (int64_t)F * 4;
        }
        return SAGA_OK;
    };
    StreamExtras ex;
    ex.op = is_max ? kGatherOpGateBothMax : kGatherOpGateBoth;
    ex.acc_width = F;
    ex.n_out = 2;
    ex.dst_width = 2 * F;
    ex.dst_fill = [&](int64_t row0, int64_t rows, float* dst, hipStream_t on, int64_t* h2d) -> saga_status {
        // [Ps | M] of the resident interval; its rows of X stay in ws_tile for after_gather
        return prod.rows(&ctx->ws_tile, row0, rows, 0, 2 * F, SAGA_ACT_NONE, dst, 2 * (int64_t)F, on, h2d);
    };
    if (with_self) {  // second operand rows [dPd | dZ]: the vertex's own partial gradient dZ W_self^T rides along
        ex.F_self = F + Fo;
        ex.self_fill = own_rows_fill(ctx, dY, Y, vp->act, Fo, h_dH + 2 * F, ldh, F, self_tile);
    } else {
        ex.self_rows = h_dH + 2 * F;  // dPd, the second operand of the last product
        ex.ld_self = ldh;
        ex.F_self = F;
    }
    ex.bytes_per_dst_row = sizeof(float) * (size_t)F;
    bool any_done = false;
    ex.after_gather = [&, any_done](int64_t, int64_t rows, float* acc, hipStream_t on, int64_t*) mutable -> saga_status {
        const float* tX = static_cast<const float*>(ctx->ws_tile.p);
        if (saga_status e = param_grad(ctx, acc, 2 * (int64_t)F, F, tX, F, F, rows, dWg, lddwg, any_done ? 1 : 0, on, false)) return e;
        if (grads->dW_msg)
            if (saga_status e = param_grad(ctx, acc + F, 2 * (int64_t)F, F, tX, F, F, rows, static_cast<float*>(grads->dW_msg->data),
                                           grads->dW_msg->ld, any_done ? 1 : 0, on, false))
                return e;
        any_done = true;
        return SAGA_OK;
    };
    saga_tensor m1_t{}, wgd_t{};
    m1_t.data = M1;
    m1_t.rows = 2 * F;
    m1_t.cols = F;
    m1_t.ld = F;
    m1_t.dtype = SAGA_F32;
    m1_t.mem = SAGA_MEM_DEVICE;
    wgd_t = *ep->W_gate;  // W_gd: the right half of W_gate, F x F with W_gate's row stride
    wgd_t.data = const_cast<float*>(Wg) + F;
    wgd_t.cols = F;
    if (with_self) {
        wgd_t.data = M2;
        wgd_t.rows = F + Fo;
        wgd_t.ld = F;
    }
    saga_vertex_params vt{};
    vt.W = &m1_t;
    vt.W_self = &wgd_t;
    vt.act = SAGA_ACT_NONE;
    saga_tensor no_dx{};
    return streamed_forward(ctx, g->tr, &rows_t, &et, SAGA_AGG_SUM, &vt, grads->dX ? grads->dX : &no_dx, &feed, &ex);
}

saga_status streamed_backward(saga_ctx* ctx, saga_graph* g, const saga_tensor* X, const saga_tensor* A, const saga_tensor* Y,
                              const saga_tensor* dY, const saga_edge_params* ep, const saga_vertex_params* vp, const saga_layer_grads* grads)
{
    const int64_t n = g->n;
    const int32_t F = (int32_t)vp->W->rows, Fo = (int32_t)vp->W->cols;
    const bool use_y = vp->act != SAGA_ACT_NONE;  // the activation's derivative is taken from the layer's output
    hipStream_t s = ctx->stream;
    saga_status st;

    if (!grads->dX || n == 0) return streamed_param_grads(ctx, n, X, A, Y, dY, vp, grads);
    const bool with_self = vp->W_self != nullptr;

    // ---- with dX: one pass. The propagation dX = (T dZ) W^T is the streamed forward schedule run on the edges grouped by
    // source, with dZ as the vertex data and W^T as the ApplyVertex matrix (no bias, no activation). dZ is not read
    // from anywhere: a source interval's rows of dY (and Y, A) are copied in, dZ is formed in place in the interval's
    // buffer, and the first time an interval comes by its share of dW and dbias is added, on the copy-in stream. ----
    if ((st = ctx->dev_alloc(&ctx->ws_wt, sizeof(float) * (size_t)F * Fo * (with_self ? 2 : 1)))) return st;
    HIP_TRY(ctx, launch_pack_bt_transpose(vp->W->data, vp->W->ld, F, Fo, SAGA_F32, ctx->ws_wt.p, F, 0, s));
    float* wst = static_cast<float*>(ctx->ws_wt.p) + (size_t)F * Fo;  // W_self^T, the second matrix of the backward "ApplyVertex"
    // tiles of the interval's own dZ for that second product: dY and Y of a tile of rows, turned into dZ
    const int64_t self_tile = std::min<int64_t>(n, std::max<int64_t>(4096, ((int64_t)64 << 20) / ((int64_t)F * 4)));
    if (with_self) {
        HIP_TRY(ctx, launch_pack_bt_transpose(vp->W_self->data, vp->W_self->ld, F, Fo, SAGA_F32, wst, F, 0, s));
        if (use_y)
            if ((st = ctx->dev_alloc(&ctx->ws_dz, sizeof(float) * (size_t)self_tile * Fo))) return st;
    }
    {
        // the split workspace for the largest interval there can be, so that nothing is allocated inside the pipeline
        int64_t rps;
        int32_t nsp;
        gemm_tn_plan(n, F, Fo, &rps, &nsp);
        const size_t need = std::max(sizeof(float) * (size_t)nsp * F * Fo, sizeof(float) * (size_t)colsum_slabs(n) * Fo);
        if ((st = ctx->dev_alloc(&ctx->ws_splitk, need))) return st;
    }
    for (DevBuf* b : {&ctx->ws_accum, &ctx->ws_hoist, &ctx->ws_dh}) ctx->dev_free(b);  // sized per interval below
    if ((st = ensure_transposed_host(ctx, g))) return st;
    bool any_done = false;
    VertexFeed feed;
    feed.bytes_per_row = sizeof(float) * ((size_t)F + (use_y ? (size_t)Fo : 0) + (with_self ? (size_t)F : 0));
    feed.fill = [&](int64_t row0, int64_t rows, float* dst, hipStream_t on, bool first_visit, int64_t* h2d) -> saga_status {
        auto rows_of_t = [](const saga_tensor* t, int64_t r) { return static_cast<const float*>(t->data) + r * t->ld; };
        HIP_TRY(ctx, hipMemcpy2DAsync(dst, sizeof(float) * (size_t)Fo, rows_of_t(dY, row0), sizeof(float) * (size_t)dY->ld,
                                      sizeof(float) * (size_t)Fo, (size_t)rows, hipMemcpyHostToDevice, on));
        *h2d += rows * (int64_t)Fo * 4;
        const bool sums = first_visit && grads->dbias;
        if (use_y) {
            if (saga_status e = ctx->dev_alloc(&ctx->ws_hoist, sizeof(float) * (size_t)rows * Fo)) return e;  // grows once: intervals do not grow
            float* tY = static_cast<float*>(ctx->ws_hoist.p);
            HIP_TRY(ctx, hipMemcpy2DAsync(tY, sizeof(float) * (size_t)Fo, rows_of_t(Y, row0), sizeof(float) * (size_t)Y->ld,
                                          sizeof(float) * (size_t)Fo, (size_t)rows, hipMemcpyHostToDevice, on));
            *h2d += rows * (int64_t)Fo * 4;
        }
        if (use_y || sums)   // in place: every element is read and written by one thread
            HIP_TRY(ctx, launch_dz_colsum(dst, Fo, use_y ? static_cast<const float*>(ctx->ws_hoist.p) : nullptr, Fo, vp->act, dst, rows, Fo,
                                          sums ? static_cast<float*>(ctx->ws_splitk.p) : nullptr,
                                          sums ? static_cast<float*>(grads->dbias->data) : nullptr, any_done ? 1 : 0, on));
        if (first_visit) {
            if (saga_status e = ctx->dev_alloc(&ctx->ws_accum, sizeof(float) * (size_t)rows * F)) return e;
            float* tA = static_cast<float*>(ctx->ws_accum.p);
            HIP_TRY(ctx, hipMemcpy2DAsync(tA, sizeof(float) * (size_t)F, rows_of_t(A, row0), sizeof(float) * (size_t)A->ld,
                                          sizeof(float) * (size_t)F, (size_t)rows, hipMemcpyHostToDevice, on));
            *h2d += rows * (int64_t)F * 4;
            if (saga_status e = param_grad(ctx, tA, F, F, dst, Fo, Fo, rows, static_cast<float*>(grads->dW->data), grads->dW->ld,
                                           any_done ? 1 : 0, on, false))
                return e;
            if (with_self) {  // dW_self += X_J^T dZ_J
                if (saga_status e = ctx->dev_alloc(&ctx->ws_dh, sizeof(float) * (size_t)rows * F)) return e;
                float* tX = static_cast<float*>(ctx->ws_dh.p);
                HIP_TRY(ctx, hipMemcpy2DAsync(tX, sizeof(float) * (size_t)F, rows_of_t(X, row0), sizeof(float) * (size_t)X->ld,
                                              sizeof(float) * (size_t)F, (size_t)rows, hipMemcpyHostToDevice, on));
                *h2d += rows * (int64_t)F * 4;
                if (saga_status e = param_grad(ctx, tX, F, F, dst, Fo, Fo, rows, static_cast<float*>(grads->dW_self->data),
                                               grads->dW_self->ld, any_done ? 1 : 0, on, false))
                    return e;
            }
            any_done = true;
        }
        return SAGA_OK;
    };
    HIP_TRY(ctx, hipStreamSynchronize(s));  // W^T is packed on the context's stream, the feed works on the copy-in stream
    saga_tensor dz_t{};
    dz_t.data = nullptr;  // shape only: the feed supplies the rows
    dz_t.rows = n;
    dz_t.cols = Fo;
    dz_t.ld = Fo;
    dz_t.dtype = SAGA_F32;
    dz_t.mem = SAGA_MEM_HOST;
    saga_tensor wt{};
    wt.data = ctx->ws_wt.p;
    wt.rows = Fo;
    wt.cols = F;
    wt.ld = F;
    wt.dtype = SAGA_F32;
    wt.mem = SAGA_MEM_DEVICE;
    saga_vertex_params vt{};
    vt.W = &wt;
    vt.act = SAGA_ACT_NONE;
    saga_edge_params et{};
    et.op = ep->op;
    if (!with_self) return streamed_forward(ctx, g->tr, &dz_t, &et, SAGA_AGG_SUM, &vt, grads->dX, &feed);

    // dX_J = (T dZ)_J W^T + dZ_J W_self^T: the vertex's own partial gradient is the second operand pair of the schedule's
    // ApplyVertex product, and the own rows dZ_J are formed tile by tile like the interval rows above
    saga_tensor wst_t = wt;
    wst_t.data = wst;
    vt.W_self = &wst_t;
    StreamExtras ex;
    ex.F_self = Fo;
    ex.self_fill = own_rows_fill(ctx, dY, Y, vp->act, Fo, nullptr, 0, 0, self_tile);
    return streamed_forward(ctx, g->tr, &dz_t, &et, SAGA_AGG_SUM, &vt, grads->dX, &feed, &ex);
}

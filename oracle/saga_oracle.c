/*
 * CPU oracle for one SAGA-NN layer (Scatter -> ApplyEdge -> Gather -> ApplyVertex).
 *
 * TEST INFRASTRUCTURE ONLY. This file is the slow, plain statement of what a
 * layer computes, used by tests/, by the smoke check and by the benchmark's
 * CPU-baseline leg. It shares no code with the HIP library and the library
 * never calls it.
 *
 * What it follows (NGra paper, arXiv 1810.08403):
 *   - stage semantics: Section 2.2 "Execution Semantics" (Scatter puts source
 *     and destination vertex data and edge data on every edge; ApplyEdge maps
 *     each edge to one tensor; Gather reduces those per destination with a
 *     commutative, associative accumulator; ApplyVertex maps the result);
 *   - accumulators sum and max: Section 2.2, last paragraph;
 *   - GCN layer: Figure 10 (ApplyEdge = src x edge.data, Gather = sum,
 *     ApplyVertex = ReLU(W (x) accum));
 *   - CommNet's pass-through ApplyEdge and its two-term ApplyVertex
 *     ReLU(W_H (x) vertex + W_C (x) accum): Figure 9;
 *   - max-pooling GCN: ApplyEdge sigma(W_pool (x) src + b), Gather max: Figure 11
 *     (sigma is not specified there; the logistic sigmoid is used);
 *   - gated layer: Example 2.1 and Figure 2 (gate = sigmoid of a linear map of
 *     source and destination data, message = gate (.) source data), widened
 *     with an optional bias and an optional message matrix;
 *   - hoisting of vertex-only products out of ApplyEdge: Section 3.2;
 *   - the backward stages (backward-ApplyVertex, -Gather, -ApplyEdge, -Scatter,
 *     Section 2.2) as the chain rule of the forward definitions: linear layers
 *     (whole graph and sampled), the gated layer (whole graph, and sampled
 *     rows of the input gradient), the max accumulator with
 *     COPY / MUL_WEIGHT / max-pooling messages (whole graph, and sampled rows
 *     of the input gradient; further down in this file).
 *
 * Every function is pinned by tests/test_oracle_pins.py against something
 * other than itself (dense matrix forms, finite differences of the forward
 * functions, automatic differentiation of dense formulations, hand-made
 * cases); none is "parity unpinned".
 *
 * Conventions. An edge goes from source u to destination v. The graph is
 * destination-major CSC: in-edges of v are row_idx[col_ptr[v] .. col_ptr[v+1]).
 * X is n x F row-major fp32. The gate matrix W_gate is F x 2F row-major; its
 * columns 0..F-1 multiply the source row and F..2F-1 the destination row.
 * W_msg is F x F row-major (output channel major); NULL means identity.
 * W (ApplyVertex) is F x F_out row-major so that Y = A W.
 * All sums are accumulated in fp64 and returned as fp64; nothing is rounded on
 * the way except where the definition itself is an fp32 operation:
 * for MUL_WEIGHT the per-edge message is the single IEEE fp32 product
 * w_e * x (so that max-Gather is reproducible bit for bit).
 * Gather over an empty in-edge set yields 0 for both accumulators.
 *
 * Besides each value the oracle returns the scale against which a
 * floating-point error of that value is measured (A_abs, Y_abs): the same
 * expression with every term of every sum replaced by its absolute value.
 * A gated message g * t (g = sigmoid(z), t = sum_k Wm[f,k] x_u[k]) is itself
 * built from sums, so its scale is g * (T + |t| (1 - g) Z), where T and Z are
 * the absolute-term sums of t and of the gate's pre-activation z, and
 * g (1 - g) is the sigmoid's derivative: a first-order forward error bound
 * per unit of relative rounding error.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { EDGE_COPY = 0, EDGE_MUL_WEIGHT = 1, EDGE_GATED = 2 };
enum { AGG_SUM = 0, AGG_MAX = 1 };
enum { ACT_NONE = 0, ACT_RELU = 1 };

int saga_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

static double sigmoid(double z) { return 1.0 / (1.0 + exp(-z)); }

/*
 * Per-vertex products of Section 3.2: Ps = X Wgs^T, Pd = X Wgd^T, M = X Wm^T
 * (M = X when W_msg is NULL). Outputs are n x F fp64.
 */
int saga_oracle_hoist(int64_t n, const float* X, int64_t F, const float* W_gate, const float* W_msg,
                      double* Ps, double* Pd, double* M, double* Ps_abs, double* Pd_abs, double* M_abs)
{
    if (!X || !W_gate || !Ps || !Pd || !M || n < 0 || F <= 0) return 1;
    if ((Ps_abs || Pd_abs || M_abs) && !(Ps_abs && Pd_abs && M_abs)) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t v = 0; v < n; ++v) {
        const float* x = X + v * F;
        for (int64_t f = 0; f < F; ++f) {
            const float* wg = W_gate + f * 2 * F;
            double s = 0.0, d = 0.0, sa = 0.0, da = 0.0;
            for (int64_t k = 0; k < F; ++k) {
                s += (double)wg[k] * (double)x[k];
                d += (double)wg[F + k] * (double)x[k];
                sa += fabs((double)wg[k] * (double)x[k]);
                da += fabs((double)wg[F + k] * (double)x[k]);
            }
            Ps[v * F + f] = s;
            Pd[v * F + f] = d;
            double t = (double)x[f], ta = fabs((double)x[f]);
            if (W_msg) {
                const float* wm = W_msg + f * F;
                t = 0.0;
                ta = 0.0;
                for (int64_t k = 0; k < F; ++k) {
                    t += (double)wm[k] * (double)x[k];
                    ta += fabs((double)wm[k] * (double)x[k]);
                }
            }
            M[v * F + f] = t;
            if (Ps_abs) {
                Ps_abs[v * F + f] = sa;
                Pd_abs[v * F + f] = da;
                M_abs[v * F + f] = ta;
            }
        }
    }
    return 0;
}

/*
 * Max-pooling ApplyEdge of Figure 11 (MP-GCN), hoisted: it depends on the
 * source only, so H[u] = sigmoid(W_pool x_u + b) is one product per vertex
 * (Section 3.2). W_pool is Fp x F row-major (row = output channel), b is Fp
 * (nullable). H and its error scale H_abs are n x Fp fp64.
 */
int saga_oracle_hoist_pool(int64_t n, const float* X, int64_t F, const float* W_pool, const float* b_pool, int64_t Fp,
                           double* H, double* H_abs)
{
    if (!X || !W_pool || !H || n < 0 || F <= 0 || Fp <= 0) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t v = 0; v < n; ++v) {
        const float* x = X + v * F;
        for (int64_t c = 0; c < Fp; ++c) {
            const float* wp = W_pool + c * F;
            double z = b_pool ? (double)b_pool[c] : 0.0, za = fabs(z);
            for (int64_t k = 0; k < F; ++k) {
                z += (double)wp[k] * (double)x[k];
                za += fabs((double)wp[k] * (double)x[k]);
            }
            const double g = sigmoid(z);
            H[v * Fp + c] = g;
            if (H_abs) H_abs[v * Fp + c] = g * (1.0 + (1.0 - g) * za);
        }
    }
    return 0;
}

/*
 * Arguments of one layer. Message width Fm = F_pool for EDGE_POOL, else F.
 *
 *   edge_op    EDGE_COPY / EDGE_MUL_WEIGHT (edge_w[nnz]) / EDGE_GATED / EDGE_POOL
 *   W_gate, b_gate, W_msg   gated parameters (b_gate, W_msg nullable)
 *   W_pool, b_pool, F_pool  max-pooling parameters (Figure 11; b_pool nullable)
 *   Ps, Pd, M (+ _abs)      when Ps is non-NULL the gated message is formed from these hoisted
 *                           per-vertex products instead of per-edge products
 *   H, H_abs   when H is non-NULL the pooled message is read from this hoisted array
 *   agg        AGG_SUM / AGG_MAX
 *   W, bias    ApplyVertex parameters, W is Fm x F_out; W NULL skips ApplyVertex
 *   W_self     F x F_out, nullable: adds vertex (x) W_self, CommNet's ApplyVertex (Figure 9)
 *   vlist, nv  destination vertices to compute (vlist NULL: all, nv must equal n)
 *   A, A_abs   nv x Fm  Gather output and its error scale (nullable)
 *   Y, Y_abs   nv x F_out ApplyVertex output and its scale (Y required iff W)
 */
typedef struct saga_oracle_args {
    int64_t n;
    const int64_t* col_ptr;
    const int32_t* row_idx;
    const float* X;
    int64_t F;
    int32_t edge_op, agg;
    const float* edge_w;
    const float *W_gate, *b_gate, *W_msg;
    const float *W_pool, *b_pool;
    int64_t F_pool;
    const double *Ps, *Pd, *M, *Ps_abs, *Pd_abs, *M_abs;
    const double *H, *H_abs;
    const float *W, *bias, *W_self;
    int64_t F_out;
    int32_t act, pad;
    const int64_t* vlist;
    int64_t nv;
    double *A, *A_abs, *Y, *Y_abs;
} saga_oracle_args;

enum { EDGE_POOL = 3 };
enum { ACT_SIGMOID = 2 };

int saga_oracle_layer(const saga_oracle_args* p)
{
    if (!p || !p->col_ptr || !p->X || p->F <= 0 || p->n < 0 || p->nv < 0) return 1;
    const int64_t n = p->n, F = p->F, nv = p->nv, F_out = p->F_out;
    const int edge_op = p->edge_op, agg = p->agg, act = p->act;
    if (!p->vlist && nv != n) return 1;
    if (edge_op < 0 || edge_op > 3 || agg < 0 || agg > 1) return 1;
    if (edge_op == EDGE_MUL_WEIGHT && !p->edge_w) return 1;
    if (edge_op == EDGE_GATED && !p->W_gate && !p->Ps) return 1;
    if (edge_op == EDGE_POOL && ((!p->W_pool && !p->H) || p->F_pool <= 0)) return 1;
    if (p->W && (!p->Y || F_out <= 0)) return 1;
    if (p->W_self && !p->W) return 1;
    if (p->Ps && (!p->Pd || !p->M || !p->Ps_abs || !p->Pd_abs || !p->M_abs)) return 1;
    if (p->H && !p->H_abs) return 1;
    const int64_t Fm = edge_op == EDGE_POOL ? p->F_pool : F;
    const int64_t* col_ptr = p->col_ptr;
    const int32_t* row_idx = p->row_idx;
    const float* X = p->X;
    const float *W_gate = p->W_gate, *b_gate = p->b_gate, *W_msg = p->W_msg;
    int bad = 0;

#pragma omp parallel
    {
        double* acc = (double*)malloc(sizeof(double) * (size_t)Fm * 4);
        double* aab = acc + Fm;
        double* msg = acc + 2 * Fm;
        double* mab = acc + 3 * Fm; /* error scale of msg */
#pragma omp for schedule(dynamic, 16)
        for (int64_t i = 0; i < nv; ++i) {
            const int64_t v = p->vlist ? p->vlist[i] : i;
            if (v < 0 || v >= n) {
#pragma omp atomic write
                bad = 1;
                continue;
            }
            const int64_t e0 = col_ptr[v], e1 = col_ptr[v + 1];
            for (int64_t f = 0; f < Fm; ++f) { acc[f] = 0.0; aab[f] = 0.0; }
            const float* xv = X + v * F;

            for (int64_t e = e0; e < e1; ++e) {
                const int64_t u = row_idx[e];
                const float* xu = X + u * F;
                /* ---- Scatter + ApplyEdge: message msg[f] of edge u -> v ---- */
                if (edge_op == EDGE_COPY) {
                    for (int64_t f = 0; f < F; ++f) { msg[f] = (double)xu[f]; mab[f] = fabs(msg[f]); }
                } else if (edge_op == EDGE_MUL_WEIGHT) {
                    const float w = p->edge_w[e];
                    for (int64_t f = 0; f < F; ++f) {
                        const float pr = w * xu[f]; /* one fp32 multiply */
                        msg[f] = (double)pr;
                        mab[f] = fabs(msg[f]);
                    }
                } else if (edge_op == EDGE_POOL) {
                    if (p->H) {
                        for (int64_t c = 0; c < Fm; ++c) { msg[c] = p->H[u * Fm + c]; mab[c] = p->H_abs[u * Fm + c]; }
                    } else {
                        for (int64_t c = 0; c < Fm; ++c) {
                            const float* wp = p->W_pool + c * F;
                            double z = p->b_pool ? (double)p->b_pool[c] : 0.0, za = fabs(z);
                            for (int64_t k = 0; k < F; ++k) {
                                z += (double)wp[k] * (double)xu[k];
                                za += fabs((double)wp[k] * (double)xu[k]);
                            }
                            const double g = sigmoid(z);
                            msg[c] = g;
                            mab[c] = g * (1.0 + (1.0 - g) * za);
                        }
                    }
                } else if (p->Ps) {
                    for (int64_t f = 0; f < F; ++f) {
                        const double b = b_gate ? (double)b_gate[f] : 0.0;
                        const double z = p->Ps[u * F + f] + p->Pd[v * F + f] + b;
                        const double za = p->Ps_abs[u * F + f] + p->Pd_abs[v * F + f] + fabs(b);
                        const double g = sigmoid(z), t = p->M[u * F + f];
                        msg[f] = g * t;
                        mab[f] = g * (p->M_abs[u * F + f] + fabs(t) * (1.0 - g) * za);
                    }
                } else {
                    for (int64_t f = 0; f < F; ++f) {
                        const float* wg = W_gate + f * 2 * F;
                        double z = b_gate ? (double)b_gate[f] : 0.0;
                        double za = fabs(z);
                        for (int64_t k = 0; k < F; ++k) {
                            z += (double)wg[k] * (double)xu[k];
                            za += fabs((double)wg[k] * (double)xu[k]);
                        }
                        for (int64_t k = 0; k < F; ++k) {
                            z += (double)wg[F + k] * (double)xv[k];
                            za += fabs((double)wg[F + k] * (double)xv[k]);
                        }
                        double t = (double)xu[f], ta = fabs((double)xu[f]);
                        if (W_msg) {
                            const float* wm = W_msg + f * F;
                            t = 0.0;
                            ta = 0.0;
                            for (int64_t k = 0; k < F; ++k) {
                                t += (double)wm[k] * (double)xu[k];
                                ta += fabs((double)wm[k] * (double)xu[k]);
                            }
                        }
                        const double g = sigmoid(z);
                        msg[f] = g * t;
                        mab[f] = g * (ta + fabs(t) * (1.0 - g) * za);
                    }
                }
                /* ---- Gather ---- */
                if (agg == AGG_SUM) {
                    for (int64_t f = 0; f < Fm; ++f) { acc[f] += msg[f]; aab[f] += mab[f]; }
                } else if (e == e0) {
                    for (int64_t f = 0; f < Fm; ++f) { acc[f] = msg[f]; aab[f] = mab[f]; }
                } else {
                    /* the maximum moves by no more than the largest error among its candidates */
                    for (int64_t f = 0; f < Fm; ++f) {
                        if (msg[f] > acc[f]) acc[f] = msg[f];
                        if (mab[f] > aab[f]) aab[f] = mab[f];
                    }
                }
            }
            if (p->A) memcpy(p->A + i * Fm, acc, sizeof(double) * (size_t)Fm);
            if (p->A_abs) memcpy(p->A_abs + i * Fm, aab, sizeof(double) * (size_t)Fm);

            /* ---- ApplyVertex: Y = act(bias + A W [+ x_v W_self]) ---- */
            if (p->W) {
                for (int64_t o = 0; o < F_out; ++o) {
                    double y = p->bias ? (double)p->bias[o] : 0.0;
                    double ya = fabs(y);
                    for (int64_t f = 0; f < Fm; ++f) {
                        const double w = (double)p->W[f * F_out + o];
                        y += acc[f] * w;
                        ya += aab[f] * fabs(w);
                    }
                    if (p->W_self) {
                        for (int64_t k = 0; k < F; ++k) {
                            const double t = (double)xv[k] * (double)p->W_self[k * F_out + o];
                            y += t;
                            ya += fabs(t);
                        }
                    }
                    if (act == ACT_RELU && y < 0.0) y = 0.0;
                    if (act == ACT_SIGMOID) { const double g = sigmoid(y); ya = g * (1.0 + (1.0 - g) * ya); y = g; }
                    p->Y[i * F_out + o] = y;
                    if (p->Y_abs) p->Y_abs[i * F_out + o] = ya;
                }
            }
        }
        free(acc);
    }
    return bad;
}

/*
 * Backward pass of one layer with the sum accumulator and a linear ApplyEdge
 * (EDGE_COPY or EDGE_MUL_WEIGHT), following the reverse stage order of
 * Section 2.2: backward-ApplyVertex (parameter gradients, gradient of accum and
 * the vertex's own partial gradient), backward-Gather (sum: every in-edge of v
 * receives the gradient of accum[v]), backward-ApplyEdge (times the edge
 * weight), backward-Scatter (every vertex adds up the partial gradients that
 * arrive over its out-edges and its own).
 *
 *   Z = A W + X W_self + bias,  Y = act(Z),  act in {none, ReLU, sigmoid}
 *   dZ = dY (.) act'(Z)                 (ReLU: 1 where Z > 0; sigmoid: Y (1 - Y))
 *   dW = A^T dZ,  dW_self = X^T dZ,  dbias = sum_v dZ[v]
 *   dA = dZ W^T
 *   dX[u] = sum_{e: u -> v} w_e dA[v]  +  dZ[u] W_self^T
 *
 * A (n x F, fp64) is the Gather output of the forward oracle; everything is
 * accumulated in fp64. Outputs may be NULL except where marked. The *_abs
 * outputs hold the same sums with every term replaced by its absolute value;
 * where dZ enters a term, its own error scale (act_backward) takes the place
 * of |dZ|, which is the same thing for none and ReLU.
 */

/*
 * dZ = dY * act'(z) for one element, and the scale of dZ's first-order error for a
 * caller that forms the derivative from the layer's stored fp32 output, as the backward
 * stage of Section 2.2 does (it is handed the vertex data, not the pre-activation):
 * none, ReLU: |dZ| (nothing is rounded before the products that use it);
 * sigmoid: with s = sigmoid(z), d = s (1 - s):  |dY| (d + |1 - 2s| (d za + s)), i.e. the
 * rounding of the stored s and of z (absolute-term sum za) carried through d' = 1 - 2s,
 * plus the rounding of the product itself.
 */
static void act_backward(int act, double z, double za, double g, double* dz, double* dz_abs)
{
    if (act == ACT_RELU) {
        *dz = z > 0.0 ? g : 0.0;
        *dz_abs = fabs(*dz);
    } else if (act == ACT_SIGMOID) {
        const double s = sigmoid(z), d = s * (1.0 - s), c = fabs(1.0 - 2.0 * s);
        *dz = g * d;
        *dz_abs = fabs(g) * (d + c * (d * za + s));
    } else {
        *dz = g;
        *dz_abs = fabs(g);
    }
}

typedef struct saga_oracle_bwd_args {
    int64_t n;
    const int64_t* col_ptr;
    const int32_t* row_idx;
    const float* X;      /* n x F, needed for dW_self only */
    int64_t F;
    int32_t edge_op, act;
    const float* edge_w;
    const double* A;     /* n x F */
    const float *W, *bias, *W_self;
    int64_t F_out;
    const float* dY;     /* n x F_out */
    double *dX, *dX_abs; /* n x F */
    double *dW, *dW_abs; /* F x F_out */
    double *dW_self;     /* F x F_out */
    double *dbias;       /* F_out */
    double *dA;          /* n x F, nullable: gradient of the Gather output */
    double *dW_self_abs; /* F x F_out, nullable */
    double *dbias_abs;   /* F_out, nullable */
} saga_oracle_bwd_args;

int saga_oracle_layer_backward(const saga_oracle_bwd_args* p)
{
    if (!p || !p->col_ptr || !p->A || !p->W || !p->dY || p->F <= 0 || p->F_out <= 0 || p->n < 0) return 1;
    if (p->edge_op != EDGE_COPY && p->edge_op != EDGE_MUL_WEIGHT) return 1;
    if (p->edge_op == EDGE_MUL_WEIGHT && !p->edge_w) return 1;
    if (p->act != ACT_NONE && p->act != ACT_RELU && p->act != ACT_SIGMOID) return 1;
    if ((p->W_self || p->dW_self) && !p->X) return 1;
    const int64_t n = p->n, F = p->F, Fo = p->F_out;
    double* dZ = (double*)malloc(sizeof(double) * 2 * (size_t)(n > 0 ? n : 1) * (size_t)Fo);
    double* dA = (double*)calloc((size_t)(n > 0 ? n : 1) * (size_t)F, sizeof(double));
    double* dAa = (double*)calloc((size_t)(n > 0 ? n : 1) * (size_t)F, sizeof(double));
    if (!dZ || !dA || !dAa) { free(dZ); free(dA); free(dAa); return 2; }
    double* dZa = dZ + (size_t)(n > 0 ? n : 1) * (size_t)Fo;

    /* backward-ApplyVertex, per vertex: recompute Z for the activation's derivative */
#pragma omp parallel for schedule(static)
    for (int64_t v = 0; v < n; ++v) {
        for (int64_t o = 0; o < Fo; ++o) {
            double z = p->bias ? (double)p->bias[o] : 0.0, za = fabs(z);
            for (int64_t f = 0; f < F; ++f) {
                const double t = p->A[v * F + f] * (double)p->W[f * Fo + o];
                z += t;
                za += fabs(t);
            }
            if (p->W_self)
                for (int64_t k = 0; k < F; ++k) {
                    const double t = (double)p->X[v * F + k] * (double)p->W_self[k * Fo + o];
                    z += t;
                    za += fabs(t);
                }
            act_backward(p->act, z, za, (double)p->dY[v * Fo + o], &dZ[v * Fo + o], &dZa[v * Fo + o]);
        }
        for (int64_t f = 0; f < F; ++f) {
            double s = 0.0, sa = 0.0;
            for (int64_t o = 0; o < Fo; ++o) {
                s += dZ[v * Fo + o] * (double)p->W[f * Fo + o];
                sa += dZa[v * Fo + o] * fabs((double)p->W[f * Fo + o]);
            }
            dA[v * F + f] = s;
            dAa[v * F + f] = sa;
        }
    }
    /* parameter gradients: one (f, o) entry per iteration, a sum over all vertices */
#pragma omp parallel for schedule(static)
    for (int64_t fo = 0; fo < F * Fo; ++fo) {
        const int64_t f = fo / Fo, o = fo % Fo;
        double s = 0.0, sa = 0.0, ss = 0.0, ssa = 0.0;
        for (int64_t v = 0; v < n; ++v) {
            s += p->A[v * F + f] * dZ[v * Fo + o];
            sa += fabs(p->A[v * F + f]) * dZa[v * Fo + o];
            if (p->dW_self) {
                ss += (double)p->X[v * F + f] * dZ[v * Fo + o];
                ssa += fabs((double)p->X[v * F + f]) * dZa[v * Fo + o];
            }
        }
        if (p->dW) p->dW[fo] = s;
        if (p->dW_abs) p->dW_abs[fo] = sa;
        if (p->dW_self) p->dW_self[fo] = ss;
        if (p->dW_self && p->dW_self_abs) p->dW_self_abs[fo] = ssa;
    }
    if (p->dbias)
        for (int64_t o = 0; o < Fo; ++o) {
            double s = 0.0, sa = 0.0;
            for (int64_t v = 0; v < n; ++v) {
                s += dZ[v * Fo + o];
                sa += dZa[v * Fo + o];
            }
            p->dbias[o] = s;
            if (p->dbias_abs) p->dbias_abs[o] = sa;
        }
    if (p->dA) memcpy(p->dA, dA, sizeof(double) * (size_t)n * (size_t)F);

    /* backward-Gather, backward-ApplyEdge, backward-Scatter: feature slices in parallel,
     * the edge list walked in order inside each slice (no two threads touch one entry) */
    if (p->dX) {
#pragma omp parallel for schedule(static)
        for (int64_t f = 0; f < F; ++f) {
            for (int64_t u = 0; u < n; ++u) {
                double s = 0.0, sa = 0.0;
                if (p->W_self)
                    for (int64_t o = 0; o < Fo; ++o) {
                        s += dZ[u * Fo + o] * (double)p->W_self[f * Fo + o];
                        sa += dZa[u * Fo + o] * fabs((double)p->W_self[f * Fo + o]);
                    }
                p->dX[u * F + f] = s;
                if (p->dX_abs) p->dX_abs[u * F + f] = sa;
            }
            for (int64_t v = 0; v < n; ++v)
                for (int64_t e = p->col_ptr[v]; e < p->col_ptr[v + 1]; ++e) {
                    const int64_t u = p->row_idx[e];
                    const double w = p->edge_op == EDGE_MUL_WEIGHT ? (double)p->edge_w[e] : 1.0;
                    p->dX[u * F + f] += w * dA[v * F + f];
                    if (p->dX_abs) p->dX_abs[u * F + f] += fabs(w) * dAa[v * F + f];
                }
        }
    }
    free(dZ);
    free(dA);
    free(dAa);
    return 0;
}

/*
 * The same backward definitions evaluated only where asked, for graphs too large to do
 * whole: rows of dX for the source vertices in ulist (n_u of them, distinct), and the
 * entries dW[w_f[i]][w_o[i]] for i < n_w. dbias is cheap and always whole (p->dbias, if
 * given). Every pre-activation the results depend on is recomputed from A (and X, W_self)
 * exactly as in the whole-graph form. Outputs: dX_rows, dX_rows_abs (n_u x F), dW_vals,
 * dW_abs_vals (n_w).
 */
static double bwd_dz(const saga_oracle_bwd_args* p, int64_t v, int64_t o, double* dz_abs)
{
    const double g = (double)p->dY[v * p->F_out + o];
    double z = 0.0, za = 0.0, dz;
    if (p->act != ACT_NONE) {
        z = p->bias ? (double)p->bias[o] : 0.0;
        za = fabs(z);
        for (int64_t f = 0; f < p->F; ++f) {
            const double t = p->A[v * p->F + f] * (double)p->W[f * p->F_out + o];
            z += t;
            za += fabs(t);
        }
        if (p->W_self)
            for (int64_t k = 0; k < p->F; ++k) {
                const double t = (double)p->X[v * p->F + k] * (double)p->W_self[k * p->F_out + o];
                z += t;
                za += fabs(t);
            }
    }
    act_backward(p->act, z, za, g, &dz, dz_abs);
    return dz;
}

int saga_oracle_backward_sample(const saga_oracle_bwd_args* p, int64_t n_u, const int64_t* ulist, double* dX_rows,
                                double* dX_rows_abs, int64_t n_w, const int64_t* w_f, const int64_t* w_o, double* dW_vals,
                                double* dW_abs_vals)
{
    if (!p || !p->col_ptr || !p->A || !p->W || !p->dY || p->F <= 0 || p->F_out <= 0 || p->n < 0) return 1;
    if (p->edge_op != EDGE_COPY && p->edge_op != EDGE_MUL_WEIGHT) return 1;
    if (p->edge_op == EDGE_MUL_WEIGHT && !p->edge_w) return 1;
    if (p->act != ACT_NONE && p->act != ACT_RELU && p->act != ACT_SIGMOID) return 1;
    if (p->W_self && !p->X) return 1;
    const int64_t n = p->n, F = p->F, Fo = p->F_out;

    if (p->dbias) {
#pragma omp parallel for schedule(static)
        for (int64_t o = 0; o < Fo; ++o) {
            double s = 0.0, sa = 0.0, da;
            for (int64_t v = 0; v < n; ++v) {
                s += bwd_dz(p, v, o, &da);
                sa += da;
            }
            p->dbias[o] = s;
            if (p->dbias_abs) p->dbias_abs[o] = sa;
        }
    }
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < n_w; ++i) {
        const int64_t f = w_f[i], o = w_o[i];
        double s = 0.0, sa = 0.0, da;
        for (int64_t v = 0; v < n; ++v) {
            s += p->A[v * F + f] * bwd_dz(p, v, o, &da);
            sa += fabs(p->A[v * F + f]) * da;
        }
        dW_vals[i] = s;
        dW_abs_vals[i] = sa;
    }

    if (n_u > 0) {
        /* which sample, if any, a source id belongs to */
        int64_t* slot = (int64_t*)malloc(sizeof(int64_t) * (size_t)(n > 0 ? n : 1));
        if (!slot) return 2;
        for (int64_t u = 0; u < n; ++u) slot[u] = -1;
        for (int64_t i = 0; i < n_u; ++i) {
            if (ulist[i] < 0 || ulist[i] >= n || slot[ulist[i]] >= 0) { free(slot); return 1; }
            slot[ulist[i]] = i;
        }
        /* the vertex's own partial gradient */
#pragma omp parallel for schedule(dynamic, 1)
        for (int64_t i = 0; i < n_u; ++i) {
            const int64_t u = ulist[i];
            for (int64_t f = 0; f < F; ++f) {
                double s = 0.0, sa = 0.0;
                if (p->W_self)
                    for (int64_t o = 0; o < Fo; ++o) {
                        double da;
                        s += bwd_dz(p, u, o, &da) * (double)p->W_self[f * Fo + o];
                        sa += da * fabs((double)p->W_self[f * Fo + o]);
                    }
                dX_rows[i * F + f] = s;
                dX_rows_abs[i * F + f] = sa;
            }
        }
        /* every edge whose source is sampled adds w_e * (dZ[v] W^T) to that sample's row;
         * destinations in parallel, each with a private copy of the sample rows, added up
         * in thread order afterwards */
        int nt = 1;
#ifdef _OPENMP
        nt = omp_get_max_threads();
#endif
        double* priv = (double*)calloc((size_t)nt * 2 * (size_t)n_u * (size_t)F, sizeof(double));
        if (!priv) { free(slot); return 2; }
#pragma omp parallel
        {
            int tid = 0;
#ifdef _OPENMP
            tid = omp_get_thread_num();
#endif
            double* mine = priv + (size_t)tid * 2 * (size_t)n_u * (size_t)F;
            double* mine_abs = mine + (size_t)n_u * (size_t)F;
            double* dz = (double*)malloc(sizeof(double) * (size_t)(2 * Fo + 2 * F));
            double* dza = dz + Fo;
            double* da = dza + Fo;     /* gradient of accum[v], and the same with absolute terms */
            double* da_abs = da + F;
#pragma omp for schedule(dynamic, 64)
            for (int64_t v = 0; v < n; ++v) {
                int have = 0;
                for (int64_t e = p->col_ptr[v]; e < p->col_ptr[v + 1]; ++e) {
                    const int64_t i = slot[p->row_idx[e]];
                    if (i < 0) continue;
                    if (!have) {
                        for (int64_t o = 0; o < Fo; ++o) dz[o] = bwd_dz(p, v, o, &dza[o]);
                        for (int64_t f = 0; f < F; ++f) {
                            double s = 0.0, sa = 0.0;
                            for (int64_t o = 0; o < Fo; ++o) {
                                s += dz[o] * (double)p->W[f * Fo + o];
                                sa += dza[o] * fabs((double)p->W[f * Fo + o]);
                            }
                            da[f] = s;
                            da_abs[f] = sa;
                        }
                        have = 1;
                    }
                    const double w = p->edge_op == EDGE_MUL_WEIGHT ? (double)p->edge_w[e] : 1.0;
                    for (int64_t f = 0; f < F; ++f) {
                        mine[i * F + f] += w * da[f];
                        mine_abs[i * F + f] += fabs(w) * da_abs[f];
                    }
                }
            }
            free(dz);
        }
        for (int t = 0; t < nt; ++t) {
            const double* mine = priv + (size_t)t * 2 * (size_t)n_u * (size_t)F;
            for (int64_t k = 0; k < n_u * F; ++k) {
                dX_rows[k] += mine[k];
                dX_rows_abs[k] += mine[(size_t)n_u * (size_t)F + k];
            }
        }
        free(priv);
        free(slot);
    }
    return 0;
}

/*
 * Backward pass of a gated layer (Example 2.1 / Figure 2 with the optional bias b and message
 * matrix W_m), sum accumulator, following the backward stages of Section 2.2:
 *
 *   forward   s_e = W_gs x_u + W_gd x_v + b,  g_e = sigmoid(s_e),  t_u = W_m x_u,
 *             m_e = g_e (.) t_u,  A[v] = sum of m_e over in-edges,  Y = act(A W [+ X W_self] + bias)
 *   backward-ApplyVertex   dZ = dY (.) act'(Z), dW = A^T dZ, dbias = sum_v dZ, dA = dZ W^T
 *                          [dW_self = X^T dZ, and dZ[u] W_self^T joins dX[u]]
 *   backward-Gather        every in-edge e of v receives dm_e = dA[v]
 *   backward-ApplyEdge     dt_e = g_e (.) dm_e,  ds_e = dm_e (.) t_u (.) g_e (.) (1 - g_e);
 *                          the source receives (ds_e through W_gs, dt_e through W_m), the destination ds_e
 *                          through W_gd; parameters: dW_gs += ds_e x_u^T, dW_gd += ds_e x_v^T, db += ds_e,
 *                          dW_m += dt_e x_u^T
 *   backward-Scatter       dX[u] = sum over out-edges (W_gs^T ds_e + W_m^T dt_e) + sum over in-edges W_gd^T ds_e
 *
 * The per-vertex products (Section 3.2) are formed once in fp64; the per-edge sums are first
 * collected per vertex (dPs[u], dM[u] over out-edges, dPd[v] over in-edges), which is the same
 * sum regrouped. W_gate is F x 2F (row = output channel, columns [0,F) source, [F,2F)
 * destination); W_msg F x F (row = output channel) or NULL for the identity, in which case
 * dW_msg is the gradient with respect to an explicit identity matrix.
 * Every *_abs output is the first-order error scale of its value: all sums with absolute
 * terms, and for each use of g the rounding of its argument propagated through g' = g (1 - g).
 *
 * Max accumulator (agg = AGG_MAX; A[v][f] = max of m_e[f] over in-edges, 0 without in-edges): the
 * Gather output is recomputed here from the hoisted products (p->A is not read) so that
 * backward-Gather can ask, per edge and feature, whether the message equals the maximum; an edge
 * whose message does receives dm_e[f] = dA[v][f] whole (ties: every maximal edge, as for the other
 * max layers), every other edge receives nothing for that feature. Everything else is unchanged.
 * The recomputed Gather output is returned in A_max (n x F, nullable).
 */
typedef struct saga_oracle_gbwd_args {
    int64_t n;
    const int64_t* col_ptr;
    const int32_t* row_idx;
    const float* X;
    int64_t F;
    const float *W_gate, *b_gate, *W_msg;
    const double* A;
    const float *W, *bias;
    int64_t F_out;
    int32_t act, agg;    /* agg: AGG_SUM, or AGG_MAX (see below) */
    const float* dY;
    double *dX, *dX_abs, *dW, *dW_abs, *dbias;
    double *dW_gate, *dW_gate_abs, *db_gate, *db_gate_abs, *dW_msg, *dW_msg_abs;
    const float* W_self;                        /* F x F_out, nullable: Z = A W + X W_self + bias */
    double *dW_self, *dW_self_abs, *dbias_abs;  /* nullable (dW_self with W_self only) */
    double *A_max;                              /* n x F out, nullable (AGG_MAX only) */
} saga_oracle_gbwd_args;

int saga_oracle_gated_backward(const saga_oracle_gbwd_args* p)
{
    if (!p || !p->col_ptr || !p->X || !p->W_gate || !p->W || !p->dY || p->F <= 0 || p->F_out <= 0 || p->n < 0) return 1;
    if (p->agg != AGG_SUM && p->agg != AGG_MAX) return 1;
    if (p->agg == AGG_SUM && !p->A) return 1;
    if (p->act != ACT_NONE && p->act != ACT_RELU && p->act != ACT_SIGMOID) return 1;
    if (!p->dX || !p->dX_abs || !p->dW || !p->dW_abs || !p->dbias || !p->dW_gate || !p->dW_gate_abs || !p->db_gate ||
        !p->db_gate_abs || !p->dW_msg || !p->dW_msg_abs)
        return 1;
    if (p->dW_self && !p->W_self) return 1;
    const int64_t n = p->n, F = p->F, Fo = p->F_out;
    const int is_max = p->agg == AGG_MAX;
    const size_t nf = (size_t)(n > 0 ? n : 1) * (size_t)F, nz = (size_t)(n > 0 ? n : 1) * (size_t)Fo;
    double* buf = (double*)calloc(15 * nf + 2 * nz, sizeof(double));
    if (!buf) return 2;
    double *Ps = buf, *Pd = Ps + nf, *M = Pd + nf, *Psa = M + nf, *Pda = Psa + nf, *Ma = Pda + nf;
    double *dA = Ma + nf, *dAa = dA + nf, *dPs = dAa + nf, *dPd = dPs + nf, *dM = dPd + nf;
    double *dPsa = dM + nf, *dPda = dPsa + nf, *dMa = dPda + nf, *Amax = dMa + nf, *dZ = Amax + nf, *dZa = dZ + nz;
    if (saga_oracle_hoist(n, p->X, F, p->W_gate, p->W_msg, Ps, Pd, M, Psa, Pda, Ma)) { free(buf); return 1; }
    const double* Ain = p->A;
    if (is_max) {
        /* Gather with the max accumulator, the message formed exactly as in backward-Gather below */
#pragma omp parallel for schedule(dynamic, 16)
        for (int64_t v = 0; v < n; ++v)
            for (int64_t f = 0; f < F; ++f) {
                const double b = p->b_gate ? (double)p->b_gate[f] : 0.0;
                double best = 0.0;
                for (int64_t e = p->col_ptr[v]; e < p->col_ptr[v + 1]; ++e) {
                    const int64_t u = p->row_idx[e];
                    const double m = sigmoid(Ps[u * F + f] + Pd[v * F + f] + b) * M[u * F + f];
                    if (e == p->col_ptr[v] || m > best) best = m;
                }
                Amax[v * F + f] = best;
            }
        Ain = Amax;
        if (p->A_max) memcpy(p->A_max, Amax, sizeof(double) * (size_t)n * (size_t)F);
    }

    /* backward-ApplyVertex */
#pragma omp parallel for schedule(static)
    for (int64_t v = 0; v < n; ++v) {
        for (int64_t o = 0; o < Fo; ++o) {
            double z = p->bias ? (double)p->bias[o] : 0.0, za = fabs(z);
            for (int64_t f = 0; f < F; ++f) {
                const double t = Ain[v * F + f] * (double)p->W[f * Fo + o];
                z += t;
                za += fabs(t);
            }
            if (p->W_self)
                for (int64_t k = 0; k < F; ++k) {
                    const double t = (double)p->X[v * F + k] * (double)p->W_self[k * Fo + o];
                    z += t;
                    za += fabs(t);
                }
            act_backward(p->act, z, za, (double)p->dY[v * Fo + o], &dZ[v * Fo + o], &dZa[v * Fo + o]);
        }
        for (int64_t f = 0; f < F; ++f) {
            double s = 0.0, sa = 0.0;
            for (int64_t o = 0; o < Fo; ++o) {
                s += dZ[v * Fo + o] * (double)p->W[f * Fo + o];
                sa += dZa[v * Fo + o] * fabs((double)p->W[f * Fo + o]);
            }
            dA[v * F + f] = s;
            dAa[v * F + f] = sa;
        }
    }
    /* dW (and dW_self): one row of W per thread, every entry a sum over the vertices in order */
#pragma omp parallel
    {
        double* row = (double*)malloc(sizeof(double) * 4 * (size_t)Fo);
#pragma omp for schedule(static)
        for (int64_t f = 0; f < F; ++f) {
            for (int64_t o = 0; o < 4 * Fo; ++o) row[o] = 0.0;
            for (int64_t v = 0; v < n; ++v) {
                const double a = Ain[v * F + f], x = (double)p->X[v * F + f];
                for (int64_t o = 0; o < Fo; ++o) {
                    row[o] += a * dZ[v * Fo + o];
                    row[Fo + o] += fabs(a) * dZa[v * Fo + o];
                    row[2 * Fo + o] += x * dZ[v * Fo + o];
                    row[3 * Fo + o] += fabs(x) * dZa[v * Fo + o];
                }
            }
            for (int64_t o = 0; o < Fo; ++o) {
                p->dW[f * Fo + o] = row[o];
                p->dW_abs[f * Fo + o] = row[Fo + o];
                if (p->dW_self) p->dW_self[f * Fo + o] = row[2 * Fo + o];
                if (p->dW_self && p->dW_self_abs) p->dW_self_abs[f * Fo + o] = row[3 * Fo + o];
            }
        }
        free(row);
    }
    for (int64_t o = 0; o < Fo; ++o) {
        double s = 0.0, sa = 0.0;
        for (int64_t v = 0; v < n; ++v) {
            s += dZ[v * Fo + o];
            sa += dZa[v * Fo + o];
        }
        p->dbias[o] = s;
        if (p->dbias_abs) p->dbias_abs[o] = sa;
    }

    /* backward-Gather and backward-ApplyEdge: a block of features per thread, the edges in order */
    const int64_t FB = 8, nfb = (F + FB - 1) / FB;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t fb = 0; fb < nfb; ++fb) {
        const int64_t f0 = fb * FB, f1 = f0 + FB < F ? f0 + FB : F;
        for (int64_t v = 0; v < n; ++v)
            for (int64_t e = p->col_ptr[v]; e < p->col_ptr[v + 1]; ++e) {
                const int64_t u = p->row_idx[e];
                for (int64_t f = f0; f < f1; ++f) {
                    const double b = p->b_gate ? (double)p->b_gate[f] : 0.0;
                    const double s = Ps[u * F + f] + Pd[v * F + f] + b;
                    const double Za = Psa[u * F + f] + Pda[v * F + f] + fabs(b);
                    const double g = sigmoid(s), t = M[u * F + f], Ta = Ma[u * F + f];
                    if (is_max && g * t != Amax[v * F + f]) continue; /* this edge did not supply the maximum of feature f */
                    const double da = dA[v * F + f], daa = dAa[v * F + f];
                    dM[u * F + f] += g * da;
                    dMa[u * F + f] += g * (daa + fabs(da) * (1.0 - g) * Za);
                    const double ds = da * t * g * (1.0 - g);
                    const double dsa = g * (1.0 - g) * (daa * fabs(t) + fabs(da) * Ta + fabs(da * t) * fabs(1.0 - 2.0 * g) * Za);
                    dPs[u * F + f] += ds;
                    dPd[v * F + f] += ds;
                    dPsa[u * F + f] += dsa;
                    dPda[v * F + f] += dsa;
                }
            }
    }

    /* backward-Scatter: the three per-vertex gradients through their matrices */
#pragma omp parallel for schedule(static)
    for (int64_t u = 0; u < n; ++u)
        for (int64_t k = 0; k < F; ++k) {
            double s = 0.0, sa = 0.0;
            for (int64_t f = 0; f < F; ++f) {
                const double wgs = (double)p->W_gate[f * 2 * F + k], wgd = (double)p->W_gate[f * 2 * F + F + k];
                const double wm = p->W_msg ? (double)p->W_msg[f * F + k] : (f == k ? 1.0 : 0.0);
                s += dPs[u * F + f] * wgs + dM[u * F + f] * wm + dPd[u * F + f] * wgd;
                sa += dPsa[u * F + f] * fabs(wgs) + dMa[u * F + f] * fabs(wm) + dPda[u * F + f] * fabs(wgd);
            }
            if (p->W_self) /* the vertex's own partial gradient */
                for (int64_t o = 0; o < Fo; ++o) {
                    s += dZ[u * Fo + o] * (double)p->W_self[k * Fo + o];
                    sa += dZa[u * Fo + o] * fabs((double)p->W_self[k * Fo + o]);
                }
            p->dX[u * F + k] = s;
            p->dX_abs[u * F + k] = sa;
        }
    /* parameter gradients of ApplyEdge: one output channel per thread, every entry a sum over the vertices in order */
#pragma omp parallel
    {
        double* row = (double*)malloc(sizeof(double) * 6 * (size_t)F);
#pragma omp for schedule(static)
        for (int64_t f = 0; f < F; ++f) {
            for (int64_t k = 0; k < 6 * F; ++k) row[k] = 0.0;
            double *gs = row, *gsa = row + F, *gd = row + 2 * F, *gda = row + 3 * F, *gm = row + 4 * F, *gma = row + 5 * F;
            for (int64_t v = 0; v < n; ++v) {
                const double a = dPs[v * F + f], aa = dPsa[v * F + f], d = dPd[v * F + f], da = dPda[v * F + f];
                const double mm = dM[v * F + f], ma = dMa[v * F + f];
                for (int64_t k = 0; k < F; ++k) {
                    const double x = (double)p->X[v * F + k];
                    gs[k] += a * x;
                    gsa[k] += aa * fabs(x);
                    gd[k] += d * x;
                    gda[k] += da * fabs(x);
                    gm[k] += mm * x;
                    gma[k] += ma * fabs(x);
                }
            }
            for (int64_t k = 0; k < F; ++k) {
                p->dW_gate[f * 2 * F + k] = gs[k];
                p->dW_gate_abs[f * 2 * F + k] = gsa[k];
                p->dW_gate[f * 2 * F + F + k] = gd[k];
                p->dW_gate_abs[f * 2 * F + F + k] = gda[k];
                p->dW_msg[f * F + k] = gm[k];
                p->dW_msg_abs[f * F + k] = gma[k];
            }
        }
        free(row);
    }
    for (int64_t f = 0; f < F; ++f) {
        double s = 0.0, sa = 0.0;
        for (int64_t v = 0; v < n; ++v) {
            s += dPd[v * F + f];
            sa += dPda[v * F + f];
        }
        p->db_gate[f] = s;
        p->db_gate_abs[f] = sa;
    }
    free(buf);
    return 0;
}

/*
 * The gated backward definitions evaluated only for the rows dX[ulist] (n_u distinct vertices), for graphs
 * too large to do whole. A sampled vertex u needs dPs[u], dM[u] (sums over its out-edges) and dPd[u] (a sum
 * over its in-edges), hence the per-vertex products of u and of its neighbours only; those are formed here
 * exactly as in the whole-graph form. Sum accumulator, no activation and no W_self: p->dY is taken as dZ (p->act must be
 * ACT_NONE, p->A and the parameter-gradient outputs are not used). Outputs n_u x F.
 */
int saga_oracle_gated_backward_sample(const saga_oracle_gbwd_args* p, int64_t n_u, const int64_t* ulist, double* dX_rows,
                                      double* dX_rows_abs)
{
    if (!p || !p->col_ptr || !p->X || !p->W_gate || !p->W || !p->dY || p->F <= 0 || p->F_out <= 0 || p->n < 0) return 1;
    if (p->act != ACT_NONE || p->agg != AGG_SUM || p->W_self || n_u < 0 || (n_u > 0 && (!ulist || !dX_rows || !dX_rows_abs))) return 1;
    const int64_t n = p->n, F = p->F, Fo = p->F_out, nnz = p->col_ptr[n];
    if (n_u == 0) return 0;
    /* the edges grouped by source */
    int64_t* optr = (int64_t*)calloc((size_t)n + 2, sizeof(int64_t));
    int32_t* odst = (int32_t*)malloc(sizeof(int32_t) * (size_t)(nnz > 0 ? nnz : 1));
    int64_t* as_src = (int64_t*)malloc(sizeof(int64_t) * (size_t)(n > 0 ? n : 1));  /* compact row of a vertex whose Ps, M are needed */
    int64_t* as_dst = (int64_t*)malloc(sizeof(int64_t) * (size_t)(n > 0 ? n : 1));  /* ... whose Pd, dA are needed */
    if (!optr || !odst || !as_src || !as_dst) { free(optr); free(odst); free(as_src); free(as_dst); return 2; }
    for (int64_t e = 0; e < nnz; ++e) optr[p->row_idx[e] + 2]++;
    for (int64_t u = 0; u < n; ++u) optr[u + 2] += optr[u + 1];
    for (int64_t v = 0; v < n; ++v)
        for (int64_t e = p->col_ptr[v]; e < p->col_ptr[v + 1]; ++e) odst[optr[p->row_idx[e] + 1]++] = (int32_t)v;
    /* now optr[u] .. optr[u + 1] are u's out-edges */
    for (int64_t v = 0; v < n; ++v) as_src[v] = as_dst[v] = -1;
    int64_t ns = 0, nd = 0;
    for (int64_t i = 0; i < n_u; ++i) {
        const int64_t u = ulist[i];
        if (u < 0 || u >= n) { free(optr); free(odst); free(as_src); free(as_dst); return 1; }
        if (as_src[u] < 0) as_src[u] = ns++;
        if (as_dst[u] < 0) as_dst[u] = nd++;
        for (int64_t e = p->col_ptr[u]; e < p->col_ptr[u + 1]; ++e)
            if (as_src[p->row_idx[e]] < 0) as_src[p->row_idx[e]] = ns++;
        for (int64_t e = optr[u]; e < optr[u + 1]; ++e)
            if (as_dst[odst[e]] < 0) as_dst[odst[e]] = nd++;
    }
    double* buf = (double*)calloc(4 * (size_t)ns * (size_t)F + 4 * (size_t)nd * (size_t)F, sizeof(double));
    if (!buf) { free(optr); free(odst); free(as_src); free(as_dst); return 2; }
    double *Ps = buf, *Psa = Ps + ns * F, *M = Psa + ns * F, *Ma = M + ns * F;
    double *Pd = Ma + ns * F, *Pda = Pd + nd * F, *dA = Pda + nd * F, *dAa = dA + nd * F;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t v = 0; v < n; ++v) {
        const float* x = p->X + v * F;
        if (as_src[v] >= 0) {
            const int64_t r = as_src[v];
            for (int64_t f = 0; f < F; ++f) {
                const float* wg = p->W_gate + f * 2 * F;
                double s = 0.0, sa = 0.0, t = (double)x[f], ta = fabs((double)x[f]);
                for (int64_t k = 0; k < F; ++k) {
                    s += (double)wg[k] * (double)x[k];
                    sa += fabs((double)wg[k] * (double)x[k]);
                }
                if (p->W_msg) {
                    const float* wm = p->W_msg + f * F;
                    t = 0.0;
                    ta = 0.0;
                    for (int64_t k = 0; k < F; ++k) {
                        t += (double)wm[k] * (double)x[k];
                        ta += fabs((double)wm[k] * (double)x[k]);
                    }
                }
                Ps[r * F + f] = s;
                Psa[r * F + f] = sa;
                M[r * F + f] = t;
                Ma[r * F + f] = ta;
            }
        }
        if (as_dst[v] >= 0) {
            const int64_t r = as_dst[v];
            for (int64_t f = 0; f < F; ++f) {
                const float* wg = p->W_gate + f * 2 * F + F;
                double d = 0.0, da = 0.0, g = 0.0, ga = 0.0;
                for (int64_t k = 0; k < F; ++k) {
                    d += (double)wg[k] * (double)x[k];
                    da += fabs((double)wg[k] * (double)x[k]);
                }
                for (int64_t o = 0; o < Fo; ++o) {
                    const double t = (double)p->dY[v * Fo + o] * (double)p->W[f * Fo + o];
                    g += t;
                    ga += fabs(t);
                }
                Pd[r * F + f] = d;
                Pda[r * F + f] = da;
                dA[r * F + f] = g;
                dAa[r * F + f] = ga;
            }
        }
    }
    /* per sampled vertex: the three sums of backward-ApplyEdge, then backward-Scatter's products */
#pragma omp parallel
    {
        double* acc = (double*)malloc(sizeof(double) * 6 * (size_t)F);
        double *dPs = acc, *dPsa = acc + F, *dM = acc + 2 * F, *dMa = acc + 3 * F, *dPd = acc + 4 * F, *dPda = acc + 5 * F;
#pragma omp for schedule(dynamic, 1)
        for (int64_t i = 0; i < n_u; ++i) {
            const int64_t u = ulist[i], us = as_src[u], ud = as_dst[u];
            for (int64_t k = 0; k < 6 * F; ++k) acc[k] = 0.0;
            for (int64_t e = optr[u]; e < optr[u + 1]; ++e) {          /* u as the source of u -> v */
                const int64_t vd = as_dst[odst[e]];
                for (int64_t f = 0; f < F; ++f) {
                    const double b = p->b_gate ? (double)p->b_gate[f] : 0.0;
                    const double z = Ps[us * F + f] + Pd[vd * F + f] + b, Za = Psa[us * F + f] + Pda[vd * F + f] + fabs(b);
                    const double g = sigmoid(z), t = M[us * F + f], Ta = Ma[us * F + f];
                    const double da = dA[vd * F + f], daa = dAa[vd * F + f];
                    dM[f] += g * da;
                    dMa[f] += g * (daa + fabs(da) * (1.0 - g) * Za);
                    dPs[f] += da * t * g * (1.0 - g);
                    dPsa[f] += g * (1.0 - g) * (daa * fabs(t) + fabs(da) * Ta + fabs(da * t) * fabs(1.0 - 2.0 * g) * Za);
                }
            }
            for (int64_t e = p->col_ptr[u]; e < p->col_ptr[u + 1]; ++e) {  /* u as the destination of w -> u */
                const int64_t ws = as_src[p->row_idx[e]];
                for (int64_t f = 0; f < F; ++f) {
                    const double b = p->b_gate ? (double)p->b_gate[f] : 0.0;
                    const double z = Ps[ws * F + f] + Pd[ud * F + f] + b, Za = Psa[ws * F + f] + Pda[ud * F + f] + fabs(b);
                    const double g = sigmoid(z), t = M[ws * F + f], Ta = Ma[ws * F + f];
                    const double da = dA[ud * F + f], daa = dAa[ud * F + f];
                    dPd[f] += da * t * g * (1.0 - g);
                    dPda[f] += g * (1.0 - g) * (daa * fabs(t) + fabs(da) * Ta + fabs(da * t) * fabs(1.0 - 2.0 * g) * Za);
                }
            }
            for (int64_t k = 0; k < F; ++k) {
                double s = 0.0, sa = 0.0;
                for (int64_t f = 0; f < F; ++f) {
                    const double wgs = (double)p->W_gate[f * 2 * F + k], wgd = (double)p->W_gate[f * 2 * F + F + k];
                    const double wm = p->W_msg ? (double)p->W_msg[f * F + k] : (f == k ? 1.0 : 0.0);
                    s += dPs[f] * wgs + dM[f] * wm + dPd[f] * wgd;
                    sa += dPsa[f] * fabs(wgs) + dMa[f] * fabs(wm) + dPda[f] * fabs(wgd);
                }
                dX_rows[i * F + k] = s;
                dX_rows_abs[i * F + k] = sa;
            }
        }
        free(acc);
    }
    free(buf);
    free(optr);
    free(odst);
    free(as_src);
    free(as_dst);
    return 0;
}

/* the vertex's own partial gradient: dX[u] += dZ[u] W_self^T (and its scale) */
static void self_gradient(int64_t n, int64_t F, int64_t Fo, const double* dZ, const double* dZa, const float* W_self, double* dX,
                          double* dX_abs)
{
#pragma omp parallel for schedule(static)
    for (int64_t u = 0; u < n; ++u)
        for (int64_t k = 0; k < F; ++k) {
            double s = 0.0, sa = 0.0;
            for (int64_t o = 0; o < Fo; ++o) {
                s += dZ[u * Fo + o] * (double)W_self[k * Fo + o];
                sa += dZa[u * Fo + o] * fabs((double)W_self[k * Fo + o]);
            }
            dX[u * F + k] += s;
            dX_abs[u * F + k] += sa;
        }
}

/*
 * Backward pass of a layer with the max accumulator (the max-pooling GCN of Figure 11, and max
 * over COPY / MUL_WEIGHT messages), through the backward stages of Section 2.2.
 *
 *   forward   m_e = x_u (COPY), w_e x_u (MUL_WEIGHT, one fp32 multiply), sigmoid(W_p x_u + b_p) (POOL);
 *             A[v][f] = max over in-edges of m_e[f] (0 without in-edges);  Y = act(A W [+ X W_self] + bias)
 *   backward-ApplyVertex   dZ, dW = A^T dZ, dbias, dA = dZ W^T [dW_self = X^T dZ, dZ[u] W_self^T joins dX[u]]
 *                          as for the sum layers
 *   backward-Gather        the gradient of A[v][f] goes to every in-edge whose message equals the
 *                          maximum (the paper does not say what happens on ties; here every
 *                          maximal edge receives the whole gradient, nothing is divided)
 *   backward-ApplyEdge     times w_e (MUL_WEIGHT); POOL: through the sigmoid, per vertex because the
 *                          message depends on the source only: dPre[u] = dS[u] (.) h_u (.) (1 - h_u)
 *   backward-Scatter       dS[u] = sum over out-edges of what they received; COPY / MUL_WEIGHT: dX = dS;
 *                          POOL: dX = dPre W_p, dW_pool = dPre^T X, db_pool = sum_u dPre[u]
 *
 * A is recomputed here from the same definitions as the forward oracle (max decisions in the
 * precision of the messages: fp32 products for MUL_WEIGHT, fp64 sigmoids for POOL).
 * *_abs: error scales (sums of absolute terms; for POOL the rounding of the sigmoid's argument
 * carried through h' and h'').
 */
typedef struct saga_oracle_mbwd_args {
    int64_t n;
    const int64_t* col_ptr;
    const int32_t* row_idx;
    const float* X;
    int64_t F;
    int32_t edge_op, act;
    const float* edge_w;
    const float *W_pool, *b_pool;
    int64_t F_pool;
    const float *W, *bias;
    int64_t F_out;
    const float* dY;
    double *A;                       /* n x Fm out (nullable): the recomputed Gather output */
    double *dX, *dX_abs;             /* n x F */
    double *dW, *dW_abs, *dbias;     /* Fm x F_out, F_out */
    double *dW_pool, *dW_pool_abs;   /* F_pool x F (POOL) */
    double *db_pool, *db_pool_abs;   /* F_pool (POOL) */
    const float* W_self;                        /* F x F_out, nullable: Z = A W + X W_self + bias */
    double *dW_self, *dW_self_abs, *dbias_abs;  /* nullable (dW_self with W_self only) */
} saga_oracle_mbwd_args;

int saga_oracle_max_backward(const saga_oracle_mbwd_args* p)
{
    if (!p || !p->col_ptr || !p->X || !p->W || !p->dY || p->F <= 0 || p->F_out <= 0 || p->n < 0) return 1;
    const int op = p->edge_op;
    if (op != EDGE_COPY && op != EDGE_MUL_WEIGHT && op != EDGE_POOL) return 1;
    if (op == EDGE_MUL_WEIGHT && !p->edge_w) return 1;
    if (op == EDGE_POOL && (!p->W_pool || p->F_pool <= 0 || !p->dW_pool || !p->dW_pool_abs || !p->db_pool || !p->db_pool_abs)) return 1;
    if (p->act != ACT_NONE && p->act != ACT_RELU && p->act != ACT_SIGMOID) return 1;
    if (!p->dX || !p->dX_abs || !p->dW || !p->dW_abs || !p->dbias) return 1;
    if (p->dW_self && !p->W_self) return 1;
    const int64_t n = p->n, F = p->F, Fo = p->F_out, Fm = op == EDGE_POOL ? p->F_pool : F;
    const size_t nm = (size_t)(n > 0 ? n : 1) * (size_t)Fm, nz = (size_t)(n > 0 ? n : 1) * (size_t)Fo;
    double* buf = (double*)calloc(8 * nm + 2 * nz, sizeof(double));
    if (!buf) return 2;
    double *S = buf, *Sz = S + nm, *A = Sz + nm, *dA = A + nm, *dAa = dA + nm, *dS = dAa + nm, *dSa = dS + nm, *spare = dSa + nm;
    double *dZ = spare + nm, *dZa = dZ + nz;

    /* the per-vertex part of the message: x_u, or h_u = sigmoid(W_p x_u + b_p) with the absolute-term sum of its argument */
#pragma omp parallel for schedule(static)
    for (int64_t u = 0; u < n; ++u)
        for (int64_t c = 0; c < Fm; ++c) {
            if (op == EDGE_POOL) {
                double z = p->b_pool ? (double)p->b_pool[c] : 0.0, za = fabs(z);
                for (int64_t k = 0; k < F; ++k) {
                    const double t = (double)p->W_pool[c * F + k] * (double)p->X[u * F + k];
                    z += t;
                    za += fabs(t);
                }
                S[u * Fm + c] = sigmoid(z);
                Sz[u * Fm + c] = za;
            } else {
                S[u * Fm + c] = (double)p->X[u * F + c];
            }
        }
    /* Gather */
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t v = 0; v < n; ++v)
        for (int64_t c = 0; c < Fm; ++c) {
            double best = 0.0;
            for (int64_t e = p->col_ptr[v]; e < p->col_ptr[v + 1]; ++e) {
                const int64_t u = p->row_idx[e];
                double m = S[u * Fm + c];
                if (op == EDGE_MUL_WEIGHT) { const float pr = p->edge_w[e] * p->X[u * F + c]; m = (double)pr; }
                if (e == p->col_ptr[v] || m > best) best = m;
            }
            A[v * Fm + c] = best;
        }
    if (p->A) memcpy(p->A, A, sizeof(double) * (size_t)n * (size_t)Fm);

    /* backward-ApplyVertex */
#pragma omp parallel for schedule(static)
    for (int64_t v = 0; v < n; ++v) {
        for (int64_t o = 0; o < Fo; ++o) {
            double z = p->bias ? (double)p->bias[o] : 0.0, za = fabs(z);
            for (int64_t c = 0; c < Fm; ++c) {
                const double t = A[v * Fm + c] * (double)p->W[c * Fo + o];
                z += t;
                za += fabs(t);
            }
            if (p->W_self)
                for (int64_t k = 0; k < F; ++k) {
                    const double t = (double)p->X[v * F + k] * (double)p->W_self[k * Fo + o];
                    z += t;
                    za += fabs(t);
                }
            act_backward(p->act, z, za, (double)p->dY[v * Fo + o], &dZ[v * Fo + o], &dZa[v * Fo + o]);
        }
        for (int64_t c = 0; c < Fm; ++c) {
            double s = 0.0, sa = 0.0;
            for (int64_t o = 0; o < Fo; ++o) {
                s += dZ[v * Fo + o] * (double)p->W[c * Fo + o];
                sa += dZa[v * Fo + o] * fabs((double)p->W[c * Fo + o]);
            }
            dA[v * Fm + c] = s;
            dAa[v * Fm + c] = sa;
        }
    }
#pragma omp parallel for schedule(static)
    for (int64_t co = 0; co < Fm * Fo; ++co) {
        const int64_t c = co / Fo, o = co % Fo;
        double s = 0.0, sa = 0.0;
        for (int64_t v = 0; v < n; ++v) {
            s += A[v * Fm + c] * dZ[v * Fo + o];
            sa += fabs(A[v * Fm + c]) * dZa[v * Fo + o];
        }
        p->dW[co] = s;
        p->dW_abs[co] = sa;
    }
    if (p->dW_self) {
#pragma omp parallel for schedule(static)
        for (int64_t ko = 0; ko < F * Fo; ++ko) {
            const int64_t k = ko / Fo, o = ko % Fo;
            double s = 0.0, sa = 0.0;
            for (int64_t v = 0; v < n; ++v) {
                s += (double)p->X[v * F + k] * dZ[v * Fo + o];
                sa += fabs((double)p->X[v * F + k]) * dZa[v * Fo + o];
            }
            p->dW_self[ko] = s;
            if (p->dW_self_abs) p->dW_self_abs[ko] = sa;
        }
    }
    for (int64_t o = 0; o < Fo; ++o) {
        double s = 0.0, sa = 0.0;
        for (int64_t v = 0; v < n; ++v) {
            s += dZ[v * Fo + o];
            sa += dZa[v * Fo + o];
        }
        p->dbias[o] = s;
        if (p->dbias_abs) p->dbias_abs[o] = sa;
    }

    /* backward-Gather, backward-ApplyEdge's edge factor and backward-Scatter: a block of features per thread, edges in order */
    const int64_t FB = 8, nfb = (Fm + FB - 1) / FB;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t fb = 0; fb < nfb; ++fb) {
        const int64_t c0 = fb * FB, c1 = c0 + FB < Fm ? c0 + FB : Fm;
        for (int64_t v = 0; v < n; ++v)
            for (int64_t e = p->col_ptr[v]; e < p->col_ptr[v + 1]; ++e) {
                const int64_t u = p->row_idx[e];
                for (int64_t c = c0; c < c1; ++c) {
                    double m = S[u * Fm + c], w = 1.0;
                    if (op == EDGE_MUL_WEIGHT) { const float pr = p->edge_w[e] * p->X[u * F + c]; m = (double)pr; w = (double)p->edge_w[e]; }
                    if (m == A[v * Fm + c]) {
                        dS[u * Fm + c] += w * dA[v * Fm + c];
                        dSa[u * Fm + c] += fabs(w) * dAa[v * Fm + c];
                    }
                }
            }
    }

    if (op != EDGE_POOL) {
        memcpy(p->dX, dS, sizeof(double) * (size_t)n * (size_t)F);
        memcpy(p->dX_abs, dSa, sizeof(double) * (size_t)n * (size_t)F);
        if (p->W_self) self_gradient(n, F, Fo, dZ, dZa, p->W_self, p->dX, p->dX_abs);
        free(buf);
        return 0;
    }
    /* POOL: through the sigmoid (dPre overwrites dS), then the per-vertex product */
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < n * Fm; ++i) {
        const double h = S[i], d1 = h * (1.0 - h);
        dSa[i] = dSa[i] * d1 + fabs(dS[i]) * d1 * fabs(1.0 - 2.0 * h) * Sz[i];
        dS[i] = dS[i] * d1;
    }
#pragma omp parallel for schedule(static)
    for (int64_t u = 0; u < n; ++u)
        for (int64_t k = 0; k < F; ++k) {
            double s = 0.0, sa = 0.0;
            for (int64_t c = 0; c < Fm; ++c) {
                s += dS[u * Fm + c] * (double)p->W_pool[c * F + k];
                sa += dSa[u * Fm + c] * fabs((double)p->W_pool[c * F + k]);
            }
            p->dX[u * F + k] = s;
            p->dX_abs[u * F + k] = sa;
        }
    if (p->W_self) self_gradient(n, F, Fo, dZ, dZa, p->W_self, p->dX, p->dX_abs);
#pragma omp parallel for schedule(static)
    for (int64_t c = 0; c < Fm; ++c) {
        double bs = 0.0, bsa = 0.0;
        for (int64_t k = 0; k < F; ++k) p->dW_pool[c * F + k] = p->dW_pool_abs[c * F + k] = 0.0;
        for (int64_t u = 0; u < n; ++u) {
            const double d = dS[u * Fm + c], da = dSa[u * Fm + c];
            bs += d;
            bsa += da;
            for (int64_t k = 0; k < F; ++k) {
                p->dW_pool[c * F + k] += d * (double)p->X[u * F + k];
                p->dW_pool_abs[c * F + k] += da * fabs((double)p->X[u * F + k]);
            }
        }
        p->db_pool[c] = bs;
        p->db_pool_abs[c] = bsa;
    }
    free(buf);
    return 0;
}

/*
 * saga_oracle_max_backward's definitions evaluated only for the rows dX[ulist] (n_u distinct source
 * vertices), for graphs too large to do whole. A row dX[u] needs: the messages of u's out-edges; for
 * every destination v of such an edge the maximum A[v] over all of v's in-edges (the whole column is
 * walked), the pre-activation of v and from it dZ[v] and dA[v] = dZ[v] W^T; for POOL the pooled row of
 * every source (one product per vertex, all of them) and the sigmoid's slope at u; with W_self the
 * vertex's own partial gradient dZ[u] W_self^T, which needs A[u] as well. Every quantity is formed by the
 * same expressions, in the same order inside a row, as in the whole-graph function; nothing is shared
 * with it but act_backward and sigmoid. Outputs dX_rows, dX_rows_abs: n_u x F.
 */
int saga_oracle_max_backward_sample(const saga_oracle_mbwd_args* p, int64_t n_u, const int64_t* ulist, double* dX_rows,
                                    double* dX_rows_abs)
{
    if (!p || !p->col_ptr || !p->X || !p->W || !p->dY || p->F <= 0 || p->F_out <= 0 || p->n < 0) return 1;
    if (n_u < 0 || (n_u > 0 && (!ulist || !dX_rows || !dX_rows_abs))) return 1;
    const int op = p->edge_op;
    if (op != EDGE_COPY && op != EDGE_MUL_WEIGHT && op != EDGE_POOL) return 1;
    if (op == EDGE_MUL_WEIGHT && !p->edge_w) return 1;
    if (op == EDGE_POOL && (!p->W_pool || p->F_pool <= 0)) return 1;
    if (p->act != ACT_NONE && p->act != ACT_RELU && p->act != ACT_SIGMOID) return 1;
    const int64_t n = p->n, F = p->F, Fo = p->F_out, Fm = op == EDGE_POOL ? p->F_pool : F;
    if (n_u == 0) return 0;

    /* which sample a vertex is, and which destinations the rows depend on */
    int64_t* sample_of = (int64_t*)malloc(sizeof(int64_t) * (size_t)(n > 0 ? n : 1));
    int64_t* slot_of = (int64_t*)malloc(sizeof(int64_t) * (size_t)(n > 0 ? n : 1));
    if (!sample_of || !slot_of) { free(sample_of); free(slot_of); return 2; }
    for (int64_t v = 0; v < n; ++v) sample_of[v] = slot_of[v] = -1;
    for (int64_t i = 0; i < n_u; ++i) {
        if (ulist[i] < 0 || ulist[i] >= n || sample_of[ulist[i]] >= 0) { free(sample_of); free(slot_of); return 1; }
        sample_of[ulist[i]] = i;
    }
    int64_t n_t = 0; /* destinations whose A, dZ and dA are needed */
    for (int64_t v = 0; v < n; ++v) {
        int need = p->W_self && sample_of[v] >= 0;
        for (int64_t e = p->col_ptr[v]; e < p->col_ptr[v + 1] && !need; ++e) need = sample_of[p->row_idx[e]] >= 0;
        if (need) slot_of[v] = n_t++;
    }
    int64_t* tlist = (int64_t*)malloc(sizeof(int64_t) * (size_t)(n_t > 0 ? n_t : 1));
    const size_t tm = (size_t)(n_t > 0 ? n_t : 1) * (size_t)Fm, tz = (size_t)(n_t > 0 ? n_t : 1) * (size_t)Fo;
    const size_t um = (size_t)n_u * (size_t)Fm;
    double* T = (double*)calloc(3 * tm + 2 * tz + 2 * um, sizeof(double));
    double *H = NULL, *Hz = NULL;
    if (op == EDGE_POOL) {
        H = (double*)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1) * (size_t)Fm);
        Hz = (double*)malloc(sizeof(double) * um);
    }
    if (!tlist || !T || (op == EDGE_POOL && (!H || !Hz))) {
        free(sample_of); free(slot_of); free(tlist); free(T); free(H); free(Hz);
        return 2;
    }
    double *A = T, *dA = A + tm, *dAa = dA + tm, *dZ = dAa + tm, *dZa = dZ + tz, *dS = dZa + tz, *dSa = dS + um;
    for (int64_t v = 0; v < n; ++v)
        if (slot_of[v] >= 0) tlist[slot_of[v]] = v;

    /* POOL: the pooled row of every vertex (any of them may supply a maximum); the absolute-term sum of the
     * sigmoid's argument only where the slope is taken, at the sampled vertices */
    if (op == EDGE_POOL) {
#pragma omp parallel for schedule(static)
        for (int64_t u = 0; u < n; ++u)
            for (int64_t c = 0; c < Fm; ++c) {
                double z = p->b_pool ? (double)p->b_pool[c] : 0.0, za = fabs(z);
                for (int64_t k = 0; k < F; ++k) {
                    const double t = (double)p->W_pool[c * F + k] * (double)p->X[u * F + k];
                    z += t;
                    za += fabs(t);
                }
                H[u * Fm + c] = sigmoid(z);
                if (sample_of[u] >= 0) Hz[sample_of[u] * Fm + c] = za;
            }
    }

    /* Gather and backward-ApplyVertex at the destinations that matter */
#pragma omp parallel for schedule(dynamic, 4)
    for (int64_t t = 0; t < n_t; ++t) {
        const int64_t v = tlist[t];
        /* the running maximum of every feature sits in A's row (zero-filled: the value without in-edges) */
        for (int64_t e = p->col_ptr[v]; e < p->col_ptr[v + 1]; ++e) {
            const int64_t u = p->row_idx[e];
            for (int64_t c = 0; c < Fm; ++c) {
                double m;
                if (op == EDGE_POOL) m = H[u * Fm + c];
                else if (op == EDGE_MUL_WEIGHT) { const float pr = p->edge_w[e] * p->X[u * F + c]; m = (double)pr; }
                else m = (double)p->X[u * F + c];
                if (e == p->col_ptr[v] || m > A[t * Fm + c]) A[t * Fm + c] = m;
            }
        }
        for (int64_t o = 0; o < Fo; ++o) {
            double z = p->bias ? (double)p->bias[o] : 0.0, za = fabs(z);
            for (int64_t c = 0; c < Fm; ++c) {
                const double tt = A[t * Fm + c] * (double)p->W[c * Fo + o];
                z += tt;
                za += fabs(tt);
            }
            if (p->W_self)
                for (int64_t k = 0; k < F; ++k) {
                    const double tt = (double)p->X[v * F + k] * (double)p->W_self[k * Fo + o];
                    z += tt;
                    za += fabs(tt);
                }
            act_backward(p->act, z, za, (double)p->dY[v * Fo + o], &dZ[t * Fo + o], &dZa[t * Fo + o]);
        }
        for (int64_t c = 0; c < Fm; ++c) {
            double s = 0.0, sa = 0.0;
            for (int64_t o = 0; o < Fo; ++o) {
                s += dZ[t * Fo + o] * (double)p->W[c * Fo + o];
                sa += dZa[t * Fo + o] * fabs((double)p->W[c * Fo + o]);
            }
            dA[t * Fm + c] = s;
            dAa[t * Fm + c] = sa;
        }
    }

    /* backward-Gather, the edge factor and backward-Scatter for the sampled sources: one feature per
     * iteration, destinations and their edges in stored order */
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t c = 0; c < Fm; ++c)
        for (int64_t t = 0; t < n_t; ++t) {
            const int64_t v = tlist[t];
            for (int64_t e = p->col_ptr[v]; e < p->col_ptr[v + 1]; ++e) {
                const int64_t u = p->row_idx[e], i = sample_of[u];
                if (i < 0) continue;
                double m, w = 1.0;
                if (op == EDGE_POOL) m = H[u * Fm + c];
                else if (op == EDGE_MUL_WEIGHT) { const float pr = p->edge_w[e] * p->X[u * F + c]; m = (double)pr; w = (double)p->edge_w[e]; }
                else m = (double)p->X[u * F + c];
                if (m == A[t * Fm + c]) {
                    dS[i * Fm + c] += w * dA[t * Fm + c];
                    dSa[i * Fm + c] += fabs(w) * dAa[t * Fm + c];
                }
            }
        }

    for (int64_t i = 0; i < n_u; ++i) {
        const int64_t u = ulist[i];
        if (op == EDGE_POOL) {
            /* through the sigmoid, then the per-vertex product */
            for (int64_t c = 0; c < Fm; ++c) {
                const double h = H[u * Fm + c], d1 = h * (1.0 - h);
                dSa[i * Fm + c] = dSa[i * Fm + c] * d1 + fabs(dS[i * Fm + c]) * d1 * fabs(1.0 - 2.0 * h) * Hz[i * Fm + c];
                dS[i * Fm + c] = dS[i * Fm + c] * d1;
            }
            for (int64_t k = 0; k < F; ++k) {
                double s = 0.0, sa = 0.0;
                for (int64_t c = 0; c < Fm; ++c) {
                    s += dS[i * Fm + c] * (double)p->W_pool[c * F + k];
                    sa += dSa[i * Fm + c] * fabs((double)p->W_pool[c * F + k]);
                }
                dX_rows[i * F + k] = s;
                dX_rows_abs[i * F + k] = sa;
            }
        } else {
            for (int64_t k = 0; k < F; ++k) {
                dX_rows[i * F + k] = dS[i * F + k];
                dX_rows_abs[i * F + k] = dSa[i * F + k];
            }
        }
        if (p->W_self) {
            const int64_t t = slot_of[u];
            for (int64_t k = 0; k < F; ++k) {
                double s = 0.0, sa = 0.0;
                for (int64_t o = 0; o < Fo; ++o) {
                    s += dZ[t * Fo + o] * (double)p->W_self[k * Fo + o];
                    sa += dZa[t * Fo + o] * fabs((double)p->W_self[k * Fo + o]);
                }
                dX_rows[i * F + k] += s;
                dX_rows_abs[i * F + k] += sa;
            }
        }
    }
    free(sample_of); free(slot_of); free(tlist); free(T); free(H); free(Hz);
    return 0;
}

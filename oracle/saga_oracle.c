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
 *   - CommNet's pass-through ApplyEdge: Figure 9;
 *   - gated layer: Example 2.1 and Figure 2 (gate = sigmoid of a linear map of
 *     source and destination data, message = gate (.) source data), widened
 *     with an optional bias and an optional message matrix;
 *   - hoisting of vertex-only products out of ApplyEdge: Section 3.2.
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
 * One layer for the destination vertices in vlist (all vertices when vlist is
 * NULL, then nv must equal n).
 *
 *   edge_op    EDGE_COPY / EDGE_MUL_WEIGHT (edge_w[nnz]) / EDGE_GATED
 *   W_gate, b_gate, W_msg   gated parameters (b_gate, W_msg nullable)
 *   Ps, Pd, M  when Ps is non-NULL the gated message is formed from these
 *              hoisted per-vertex products instead of per-edge products;
 *              Ps_abs, Pd_abs, M_abs are their absolute-term sums
 *   agg        AGG_SUM / AGG_MAX
 *   W, bias    ApplyVertex parameters; W NULL skips ApplyVertex
 *   A, A_abs   nv x F   Gather output and its absolute-term sum (nullable)
 *   Y, Y_abs   nv x F_out ApplyVertex output and its scale (nullable iff W NULL)
 * Returns 0, or nonzero on a bad argument.
 */
int saga_oracle_layer(int64_t n, const int64_t* col_ptr, const int32_t* row_idx,
                      const float* X, int64_t F,
                      int edge_op, const float* edge_w,
                      const float* W_gate, const float* b_gate, const float* W_msg,
                      const double* Ps, const double* Pd, const double* M,
                      const double* Ps_abs, const double* Pd_abs, const double* M_abs,
                      int agg,
                      const float* W, const float* bias, int64_t F_out, int act,
                      const int64_t* vlist, int64_t nv,
                      double* A, double* A_abs, double* Y, double* Y_abs)
{
    if (!col_ptr || !X || F <= 0 || n < 0 || nv < 0) return 1;
    if (!vlist && nv != n) return 1;
    if (edge_op == EDGE_MUL_WEIGHT && !edge_w) return 1;
    if (edge_op == EDGE_GATED && !W_gate && !Ps) return 1;
    if (edge_op < 0 || edge_op > 2 || agg < 0 || agg > 1) return 1;
    if (W && (!Y || F_out <= 0)) return 1;
    if (Ps && (!Pd || !M || !Ps_abs || !Pd_abs || !M_abs)) return 1;
    int bad = 0;

#pragma omp parallel
    {
        double* acc = (double*)malloc(sizeof(double) * (size_t)F * 4);
        double* aab = acc + F;
        double* msg = acc + 2 * F;
        double* mab = acc + 3 * F; /* error scale of msg */
#pragma omp for schedule(dynamic, 16)
        for (int64_t i = 0; i < nv; ++i) {
            const int64_t v = vlist ? vlist[i] : i;
            if (v < 0 || v >= n) {
#pragma omp atomic write
                bad = 1;
                continue;
            }
            const int64_t e0 = col_ptr[v], e1 = col_ptr[v + 1];
            for (int64_t f = 0; f < F; ++f) { acc[f] = 0.0; aab[f] = 0.0; }
            const float* xv = X + v * F;

            for (int64_t e = e0; e < e1; ++e) {
                const int64_t u = row_idx[e];
                const float* xu = X + u * F;
                /* ---- Scatter + ApplyEdge: message msg[f] of edge u -> v ---- */
                if (edge_op == EDGE_COPY) {
                    for (int64_t f = 0; f < F; ++f) { msg[f] = (double)xu[f]; mab[f] = fabs(msg[f]); }
                } else if (edge_op == EDGE_MUL_WEIGHT) {
                    const float w = edge_w[e];
                    for (int64_t f = 0; f < F; ++f) {
                        const float p = w * xu[f]; /* one fp32 multiply */
                        msg[f] = (double)p;
                        mab[f] = fabs(msg[f]);
                    }
                } else if (Ps) {
                    for (int64_t f = 0; f < F; ++f) {
                        const double b = b_gate ? (double)b_gate[f] : 0.0;
                        const double z = Ps[u * F + f] + Pd[v * F + f] + b;
                        const double za = Ps_abs[u * F + f] + Pd_abs[v * F + f] + fabs(b);
                        const double g = sigmoid(z), t = M[u * F + f];
                        msg[f] = g * t;
                        mab[f] = g * (M_abs[u * F + f] + fabs(t) * (1.0 - g) * za);
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
                    for (int64_t f = 0; f < F; ++f) { acc[f] += msg[f]; aab[f] += mab[f]; }
                } else if (e == e0) {
                    for (int64_t f = 0; f < F; ++f) { acc[f] = msg[f]; aab[f] = mab[f]; }
                } else {
                    for (int64_t f = 0; f < F; ++f) if (msg[f] > acc[f]) { acc[f] = msg[f]; aab[f] = mab[f]; }
                }
            }
            if (A) memcpy(A + i * F, acc, sizeof(double) * (size_t)F);
            if (A_abs) memcpy(A_abs + i * F, aab, sizeof(double) * (size_t)F);

            /* ---- ApplyVertex: Y = act(bias + A W) ---- */
            if (W) {
                for (int64_t o = 0; o < F_out; ++o) {
                    double y = bias ? (double)bias[o] : 0.0;
                    double ya = fabs(y);
                    for (int64_t f = 0; f < F; ++f) {
                        const double w = (double)W[f * F_out + o];
                        y += acc[f] * w;
                        ya += aab[f] * fabs(w);
                    }
                    if (act == ACT_RELU && y < 0.0) y = 0.0;
                    Y[i * F_out + o] = y;
                    if (Y_abs) Y_abs[i * F_out + o] = ya;
                }
            }
        }
        free(acc);
    }
    return bad;
}

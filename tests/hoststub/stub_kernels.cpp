// CPU stand-ins for every kernel launcher the host code of libsaga calls (declared in saga_internal.h).
// Test infrastructure: each launcher enqueues a closure on the given stream that computes what the kernel
// computes, with plain loops, touching every byte the kernel would touch (whole padded weight panels, the
// split workspaces), so that AddressSanitizer checks the sizes the host code allocated and the pointers it
// formed. They share no code with the HIP kernels and none with the oracle; the numbers only have to be
// good enough to tell a correct schedule from one that read stale or foreign data.
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "saga_internal.h"

namespace {

[[noreturn]] void die(const char* what)
{
    fprintf(stderr, "hoststub kernel: %s\n", what);
    fflush(stderr);
    abort();
}

float bf16_to_f32(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, 4);
    return f;
}
uint16_t f32_to_bf16(float f)
{
    uint32_t x;
    memcpy(&x, &f, 4);
    if ((x & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((x >> 16) | 0x40u);
    x += 0x7fffu + ((x >> 16) & 1u);
    return (uint16_t)(x >> 16);
}
float load_elem(const void* base, int64_t idx, int32_t dtype)
{
    return dtype == SAGA_F32 ? static_cast<const float*>(base)[idx] : bf16_to_f32(static_cast<const uint16_t*>(base)[idx]);
}
float sigmoid(float z) { return (float)(1.0 / (1.0 + std::exp(-(double)z))); }
float apply_act(float y, int act)
{
    if (act == SAGA_ACT_RELU) return y > 0.f ? y : 0.f;
    if (act == SAGA_ACT_SIGMOID) return sigmoid(y);
    return y;
}
const float kNegInf = -__builtin_huge_valf();

void store_finished(const GatherArgs& a, float* out, int64_t ld_out, int64_t v, int f, float val, int agg, bool empty, bool with16)
{
    if (a.accumulate) {
        const float prev = out[v * ld_out + f];
        val = agg == SAGA_AGG_SUM ? prev + val : (val > prev ? val : prev);
    } else if (agg == SAGA_AGG_MAX && empty) {
        val = 0.f;
    }
    if (a.bias || a.act != SAGA_ACT_NONE) val = apply_act(val + (a.bias ? a.bias[f] : 0.f), a.act);
    if (out) out[v * ld_out + f] = val;
    if (with16 && a.out16) a.out16[v * a.ld_out16 + f] = f32_to_bf16(val);
}

void gather_cpu(const GatherArgs a)
{
    const bool under_max = a.op == kGatherOpGateGradMax || a.op == kGatherOpGateBothMax;  // only maximal edges count
    const bool grad = a.op == kGatherOpGateGrad || a.op == kGatherOpGateBoth || under_max;
    const bool maxgrad = a.op == kGatherOpMaxGrad;
    const bool gated = a.op == SAGA_EDGE_GATED || grad || maxgrad;
    const bool both = a.op == kGatherOpGateBoth || a.op == kGatherOpGateBothMax;
    const int agg = (grad || maxgrad) ? SAGA_AGG_SUM : a.agg;
    const float* w = (!gated || maxgrad) ? a.edge_w : nullptr;
    for (int64_t i = 0; i < a.n_items; ++i) {
        const WorkItem it = a.items[i];
        if (it.e0 > it.e1 || it.v < 0) die("malformed work item");
        for (int f = 0; f < a.F; ++f) {
            double acc = agg == SAGA_AGG_SUM ? 0.0 : (double)kNegInf, acc2 = 0.0;
            float c1 = 0.f, c2 = 0.f;
            if (gated) {
                c1 = a.dst[(int64_t)it.v * a.ld_dst + f];
                if (maxgrad && a.dst_sigmoid) c1 = sigmoid(c1);
            }
            if (grad) c2 = a.dst2[(int64_t)it.v * a.ld_dst2 + f];
            const float c3 = a.op == kGatherOpGateGradMax ? a.dst3[(int64_t)it.v * a.ld_dst3 + f] : 0.f;
            for (int32_t e = it.e0; e < it.e1; ++e) {
                const int64_t u = a.row_idx[e];
                if (u < 0) die("negative source id reached the propagation kernel");
                const float we = w ? w[e] : 1.f;
                const float x = load_elem(a.src, u * a.ld_src + f, a.dtype);
                const float m = gated ? static_cast<const float*>(a.src2)[u * a.ld_src2 + f] : 0.f;
                if (a.op == SAGA_EDGE_GATED) {
                    const double msg = (double)sigmoid(x + c1) * m;
                    acc = agg == SAGA_AGG_SUM ? acc + msg : (msg > acc ? msg : acc);
                } else if (grad) {
                    if (under_max) {  // the forward stand-in's message, formed again and compared with the kept maximum
                        // over the in-edges the message matrix's row travels (m) and the maximum is the item's third constant
                        // row; over the out-edges that row is the item's own (c2) and the maximum travels as a third row
                        const bool in_edges = a.op == kGatherOpGateGradMax;
                        const float kept = in_edges ? c3 : static_cast<const float*>(a.src3)[u * a.ld_src3 + f];
                        if ((float)((double)sigmoid(x + c1) * (in_edges ? m : c2)) != kept) continue;
                    }
                    const double g = 1.0 / (1.0 + std::exp(-((double)x + c1)));
                    acc += g * (1.0 - g) * ((double)c2 * m);
                    if (both) acc2 += g * m;
                } else if (maxgrad) {
                    if (we * c1 == x) acc += we * m;
                } else {
                    const float msg = we * x;  // one fp32 product, as on the GPU: the max Gather is compared bit for bit
                    acc = agg == SAGA_AGG_SUM ? acc + (double)msg : (msg > acc ? (double)msg : acc);
                }
            }
            if (it.slot >= 0) {
                a.partials[(int64_t)it.slot * a.F + f] = (float)acc;
                if (both) a.partials2[(int64_t)it.slot * a.F + f] = (float)acc2;
            } else {
                store_finished(a, a.out, a.ld_out, it.v, f, (float)acc, agg, it.e0 == it.e1, true);
                if (both) store_finished(a, a.out2, a.ld_out2, it.v, f, (float)acc2, SAGA_AGG_SUM, false, false);
            }
        }
    }
}

void combine_cpu(const CombineArgs a)
{
    for (int64_t h = 0; h < a.n_heavy; ++h) {
        const HeavyVertex hv = a.heavy[h];
        if (hv.nslots < 1) die("cut column without partial rows");
        for (int f = 0; f < a.F; ++f) {
            float r = a.partials[(int64_t)hv.slot0 * a.F + f];
            for (int s = 1; s < hv.nslots; ++s) {
                const float x = a.partials[(int64_t)(hv.slot0 + s) * a.F + f];
                r = a.agg == SAGA_AGG_SUM ? r + x : (x > r ? x : r);
            }
            if (a.accumulate) {
                const float prev = a.out[(int64_t)hv.v * a.ld_out + f];
                r = a.agg == SAGA_AGG_SUM ? prev + r : (r > prev ? r : prev);
            }
            if (a.bias || a.act != SAGA_ACT_NONE) r = apply_act(r + (a.bias ? a.bias[f] : 0.f), a.act);
            if (a.out) a.out[(int64_t)hv.v * a.ld_out + f] = r;
            if (a.out16) a.out16[(int64_t)hv.v * a.ld_out16 + f] = f32_to_bf16(r);
        }
    }
}

// the output-tile width the MFMA product picks for N columns (it reads whole tiles of rows of the packed weights)
int gemm_bn(int32_t N, int32_t dtype)
{
    if (N > 64) return 128;
    if (dtype != SAGA_F32) return 64;
    return N > 32 ? 64 : 32;
}

void gemm_cpu(const GemmArgs a)
{
    int64_t np, kp, kp2 = 0;
    bt_padded_shape(a.N, a.K, a.dtype, &np, &kp);
    if (a.A2) bt_padded_shape(a.N, a.K2, a.dtype, &np, &kp2);
    if (a.ldbt < kp + kp2) die("packed weights narrower than the padded K the product reads");
    // every packed row a tile reads must be there and finite in the padded columns (the kernel multiplies them by zeros)
    const int bn = gemm_bn(a.N, a.dtype);
    const int64_t rows_read = ((int64_t)a.N + bn - 1) / bn * bn;
    for (int64_t n = 0; n < rows_read; ++n)
        for (int64_t k = 0; k < kp + kp2; ++k) {
            const float b = load_elem(a.Bt, n * a.ldbt + k, a.dtype);
            const bool inside = n < a.N && (k < a.K || (k >= kp && k < kp + a.K2));
            if (n < a.N && !inside && !(b == b && std::fabs(b) < 3e38f)) die("padding of the packed weights is not finite");
        }
    if (a.row_ids) {  // the list is padded to whole tiles of 64 rows with its last entry, ascending before that
        if (a.A2 || a.dtype != SAGA_F32) die("a row list on a product that does not take one");
        const int64_t padded = (a.M + 63) / 64 * 64;
        for (int64_t i = 0; i < padded; ++i) {
            if (a.row_ids[i] < 0) die("negative row in a row list");
            if (i > 0 && (i < a.M ? a.row_ids[i] <= a.row_ids[i - 1] : a.row_ids[i] != a.row_ids[a.M - 1])) die("row list out of order or badly padded");
        }
    }
    for (int64_t i = 0; i < a.M; ++i) {
        const int64_t m = a.row_ids ? a.row_ids[i] : i;
        for (int32_t n = 0; n < a.N; ++n) {
            double s = 0.0;
            for (int32_t k = 0; k < a.K; ++k) s += (double)load_elem(a.A, m * a.lda + k, a.dtype) * load_elem(a.Bt, (int64_t)n * a.ldbt + k, a.dtype);
            if (a.A2)
                for (int32_t k = 0; k < a.K2; ++k)
                    s += (double)load_elem(a.A2, m * a.lda2 + k, a.dtype) * load_elem(a.Bt, (int64_t)n * a.ldbt + kp + k, a.dtype);
            float y = apply_act((float)s + (a.bias ? a.bias[n] : 0.f), a.act);
            if (a.out_dtype == SAGA_F32)
                static_cast<float*>(a.C)[m * a.ldc + n] = y;
            else
                static_cast<uint16_t*>(a.C)[m * a.ldc + n] = f32_to_bf16(y);
        }
    }
}

}  // namespace

hipError_t launch_gather(const GatherArgs& a, hipStream_t s)
{
    if (a.n_items <= 0) return hipSuccess;
    if ((a.bias || a.act != SAGA_ACT_NONE) && a.accumulate) return hipErrorInvalidValue;
    if (a.ld_src < 0 || a.ld_src >= (1LL << 30) || a.ld_src2 < 0 || a.ld_src2 >= (1LL << 30)) return hipErrorInvalidValue;
    const bool both_any = a.op == kGatherOpGateBoth || a.op == kGatherOpGateBothMax;
    const bool grad = a.op == kGatherOpGateGrad || a.op == kGatherOpGateGradMax || both_any;
    const bool gated = a.op == SAGA_EDGE_GATED || grad || a.op == kGatherOpMaxGrad;
    if (gated) {
        if (!a.src2 || !a.dst || (grad && (!a.dst2 || a.agg != SAGA_AGG_SUM))) return hipErrorInvalidValue;
        if (a.op == kGatherOpMaxGrad && a.agg != SAGA_AGG_SUM) return hipErrorInvalidValue;
        if (both_any && (!a.out || !a.out2 || a.out16 || (a.partials && !a.partials2))) return hipErrorInvalidValue;
        if (a.op == kGatherOpGateGradMax && !a.dst3) return hipErrorInvalidValue;
        if (a.op == kGatherOpGateBothMax && !a.src3) return hipErrorInvalidValue;
        if (a.dtype != SAGA_F32) return hipErrorInvalidValue;
    }
    const GatherArgs copy = a;
    stub_enqueue(s, [copy] { gather_cpu(copy); });
    return hipSuccess;
}

hipError_t launch_combine(const CombineArgs& a, hipStream_t s)
{
    if (a.n_heavy <= 0) return hipSuccess;
    const CombineArgs copy = a;
    stub_enqueue(s, [copy] { combine_cpu(copy); });
    return hipSuccess;
}

// The dense blocks: the 64 x 32 operand of every block is rebuilt from its compact edge list exactly as the kernel does
// (same cell order, same two-part bf16 weights), then multiplied out with plain loops.
hipError_t launch_dense_blocks(const DenseArgs& a, hipStream_t s)
{
    if (a.n_chunks <= 0) return hipSuccess;
    if (a.F <= 0 || a.F % 128 != 0 || a.ld % 8 != 0) return hipErrorInvalidValue;
    const DenseArgs d = a;
    stub_enqueue(s, [d] {
        std::vector<float> A((size_t)kDenseM * kDenseK);
        std::vector<double> acc((size_t)kDenseM * d.F);
        for (int64_t c = 0; c < d.n_chunks; ++c) {
            const DenseChunk ch = d.chunks[c];
            std::fill(acc.begin(), acc.end(), 0.0);
            for (int b = ch.b0; b < ch.b1; ++b) {
                std::fill(A.begin(), A.end(), 0.f);
                // undo the lane order: cell = ((sub-tile * 64 + lane) * 8 + k % 8), lane = (k / 8) * 16 + m % 16
                auto cell_to_mk = [](int pos, int* m, int* k) {
                    const int j = pos & 7, lane = (pos >> 3) & 63, mt = pos >> 9;
                    *m = mt * 16 + (lane & 15);
                    *k = (lane >> 4) * 8 + j;
                };
                if (d.blk_tile[b] >= 0) {
                    if (d.blk_e0[b] != d.blk_e0[b + 1]) die("a block kept as a finished operand has an edge list too");
                    const uint16_t* t = d.de_tiles + (int64_t)d.blk_tile[b] * kDenseTileElems;
                    for (int pos = 0; pos < kDenseM * kDenseK; ++pos) {
                        int m, k;
                        cell_to_mk(pos, &m, &k);
                        A[(size_t)m * kDenseK + k] = bf16_to_f32(t[pos]) + (d.use_low ? bf16_to_f32(t[pos + kDenseM * kDenseK]) : 0.f);
                    }
                } else {
                    if (d.blk_e0[b + 1] - d.blk_e0[b] > kDenseListMax || d.blk_e0[b + 1] <= d.blk_e0[b]) die("edge list of a block out of range");
                    for (int e = d.blk_e0[b]; e < d.blk_e0[b + 1]; ++e) {
                        const int pos = d.de_pos[e];
                        if (pos < 0 || pos >= kDenseM * kDenseK) die("dense edge outside its block");
                        int m, k;
                        cell_to_mk(pos, &m, &k);
                        if (A[(size_t)m * kDenseK + k] != 0.f) die("two dense edges in one cell");
                        const uint32_t w = d.de_w[e];
                        A[(size_t)m * kDenseK + k] = bf16_to_f32((uint16_t)(w & 0xffffu)) + (d.use_low ? bf16_to_f32((uint16_t)(w >> 16)) : 0.f);
                    }
                }
                const int32_t* ids = d.src_tile_ids + (int64_t)d.blk_src_tile[b] * kDenseK;
                for (int m = 0; m < kDenseM; ++m)
                    for (int k = 0; k < kDenseK; ++k) {
                        const float wmk = A[(size_t)m * kDenseK + k];
                        if (wmk == 0.f) continue;
                        for (int f = 0; f < d.F; ++f) acc[(size_t)m * d.F + f] += (double)wmk * bf16_to_f32(d.X[(int64_t)ids[k] * d.ld + f]);
                    }
                for (int k = 0; k < kDenseK; ++k) (void)d.X[(int64_t)ids[k] * d.ld];  // every row of the block is read, weighted or not
            }
            for (int m = 0; m < kDenseM; ++m) {
                const int slot0 = d.tile_row_slot0[(int64_t)ch.tile * kDenseM + m];
                if (slot0 < 0) continue;
                for (int f = 0; f < d.F; ++f) d.partials[(int64_t)(slot0 + ch.cidx) * d.F + f] = (float)acc[(size_t)m * d.F + f];
            }
        }
    });
    return hipSuccess;
}

hipError_t launch_pack_hybrid_weights(const PackArgs& in, hipStream_t s)
{
    PackArgs a = in;
    if (!a.w) a.n_rem = 0;
    if (a.n_list + a.n_tile + a.n_rem <= 0) return hipSuccess;
    stub_enqueue(s, [a] {
        auto split = [&](float x, uint16_t* hi, uint16_t* lo) {
            *hi = f32_to_bf16(x);
            *lo = f32_to_bf16(x - bf16_to_f32(*hi));
        };
        for (int64_t i = 0; i < a.n_list; ++i) {
            uint16_t hi, lo;
            split(a.w ? a.w[a.de_edge[i]] : 1.0f, &hi, &lo);
            a.de_w[i] = (uint32_t)hi | ((uint32_t)lo << 16);
        }
        for (int64_t i = 0; i < a.n_tile; ++i) {
            uint16_t hi, lo;
            split(a.w ? a.w[a.dt_edge[i]] : 1.0f, &hi, &lo);
            a.de_tiles[a.dt_addr[i]] = hi;
            a.de_tiles[a.dt_addr[i] + kDenseM * kDenseK] = lo;
        }
        for (int64_t i = 0; i < a.n_rem; ++i) a.rem_w[i] = a.w[a.rem_edge[i]];
    });
    return hipSuccess;
}

hipError_t launch_fill_f32(float* p, int64_t count, float value, hipStream_t s)
{
    if (count <= 0) return hipSuccess;
    stub_enqueue(s, [=] {
        for (int64_t i = 0; i < count; ++i) p[i] = value;
    });
    return hipSuccess;
}
hipError_t launch_neg_inf_to_zero(float* p, int64_t count, hipStream_t s)
{
    if (count <= 0) return hipSuccess;
    stub_enqueue(s, [=] {
        for (int64_t i = 0; i < count; ++i)
            if (p[i] == kNegInf) p[i] = 0.f;
    });
    return hipSuccess;
}
hipError_t launch_f32_to_bf16(const float* in, uint16_t* out, int64_t count, hipStream_t s)
{
    if (count <= 0) return hipSuccess;
    stub_enqueue(s, [=] {
        for (int64_t i = 0; i < count; ++i) out[i] = f32_to_bf16(in[i]);
    });
    return hipSuccess;
}
hipError_t launch_validate_columns(const int64_t* col_ptr, int64_t n_cols, const int32_t* row_idx, int64_t n_src, int32_t* flag, hipStream_t s)
{
    if (n_cols <= 0) return hipSuccess;
    stub_enqueue(s, [=] {
        for (int64_t v = 0; v < n_cols; ++v)
            for (int64_t e = col_ptr[v]; e < col_ptr[v + 1]; ++e) {
                const int32_t u = row_idx[e];
                if (u < 0 || u >= n_src || (e > col_ptr[v] && row_idx[e - 1] >= u)) *flag = 1;
            }
    });
    return hipSuccess;
}

void bt_padded_shape(int32_t N, int32_t K, int32_t dtype, int64_t* n_pad, int64_t* k_pad)
{
    const int kt = dtype == SAGA_F32 ? 16 : 64;
    *n_pad = ((int64_t)N + 127) / 128 * 128;
    *k_pad = ((int64_t)K + kt - 1) / kt * kt;
}

static int64_t g_row_list_launches = 0;
extern "C" int64_t stub_row_list_launches() { return g_row_list_launches; }

// the real product kernel that takes row lists wants K = 128 and at least 16,384 rows; the stand-in takes lists from 64 rows
// on, so that small graphs reach the host code that builds and hands over the lists
bool gemm_takes_row_list(const GemmArgs& a)
{
    return a.row_ids && a.dtype == SAGA_F32 && a.out_dtype == SAGA_F32 && !a.tiled_only && !a.A2 && a.K == 128 && a.M >= 64;
}

hipError_t launch_gemm(const GemmArgs& a, hipStream_t s)
{
    if (a.M <= 0 || a.N <= 0) return hipSuccess;
    if (a.row_ids && !gemm_takes_row_list(a)) return hipErrorInvalidValue;
    if (a.row_ids) ++g_row_list_launches;
    if (a.K <= 0 || (a.A2 && a.K2 <= 0)) return hipErrorInvalidValue;
    if (a.dtype == SAGA_F32 && a.out_dtype != SAGA_F32) return hipErrorInvalidValue;
    const GemmArgs copy = a;
    stub_enqueue(s, [copy] { gemm_cpu(copy); });
    return hipSuccess;
}

hipError_t launch_pack_bt_transpose(const void* W, int64_t ldw, int32_t K, int32_t N, int32_t dtype, void* Bt, int64_t ldbt, int64_t col0,
                                    hipStream_t s)
{
    if ((int64_t)N * K <= 0) return hipSuccess;
    stub_enqueue(s, [=] {
        for (int64_t k = 0; k < K; ++k)
            for (int64_t n = 0; n < N; ++n) {
                if (dtype == SAGA_F32)
                    static_cast<float*>(Bt)[n * ldbt + col0 + k] = static_cast<const float*>(W)[k * ldw + n];
                else
                    static_cast<uint16_t*>(Bt)[n * ldbt + col0 + k] = static_cast<const uint16_t*>(W)[k * ldw + n];
            }
    });
    return hipSuccess;
}
hipError_t launch_pack_bt_rows(const float* Wsrc, int64_t ldw, int64_t col0, int32_t R, int32_t K, float* Bt, int64_t ldbt, int64_t row0,
                               hipStream_t s)
{
    if ((int64_t)R * K <= 0) return hipSuccess;
    stub_enqueue(s, [=] {
        for (int64_t r = 0; r < R; ++r)
            for (int64_t k = 0; k < K; ++k) Bt[(row0 + r) * ldbt + k] = Wsrc ? Wsrc[r * ldw + col0 + k] : (r == k ? 1.f : 0.f);
    });
    return hipSuccess;
}
hipError_t launch_pack_bt_rows_bf16(const uint16_t* Wsrc, int64_t ldw, int32_t R, int32_t K, uint16_t* Bt, int64_t ldbt, hipStream_t s)
{
    if ((int64_t)R * K <= 0) return hipSuccess;
    stub_enqueue(s, [=] {
        for (int64_t r = 0; r < R; ++r)
            for (int64_t k = 0; k < K; ++k) Bt[r * ldbt + k] = Wsrc[r * ldw + k];
    });
    return hipSuccess;
}
hipError_t launch_stage_scatter_apply(const void* X, int64_t ldx, int32_t dtype, const int32_t* src, const float* edge_w, float* S, int32_t* iota,
                                      int32_t F, int64_t n_edges, hipStream_t s)
{
    if (n_edges <= 0 || F <= 0) return hipSuccess;
    stub_enqueue(s, [=] {
        for (int64_t e = 0; e < n_edges; ++e) {
            for (int f = 0; f < F; ++f) S[e * F + f] = (edge_w ? edge_w[e] : 1.f) * load_elem(X, (int64_t)src[e] * ldx + f, dtype);
            iota[e] = (int32_t)e;
        }
    });
    return hipSuccess;
}
hipError_t launch_zero_bytes(void* p, size_t bytes, hipStream_t s)
{
    if (bytes == 0) return hipSuccess;
    if (bytes % 4 != 0 || (reinterpret_cast<uintptr_t>(p) & 3u)) return hipErrorInvalidValue;
    stub_enqueue(s, [=] { memset(p, 0, bytes); });
    return hipSuccess;
}
hipError_t launch_copy_bytes(void* dst, const void* src, size_t bytes, hipStream_t s)
{
    if (bytes == 0) return hipSuccess;
    if (bytes % 16 != 0 || (reinterpret_cast<uintptr_t>(dst) & 15u) || (reinterpret_cast<uintptr_t>(src) & 15u)) return hipErrorInvalidValue;
    stub_enqueue(s, [=] { memcpy(dst, src, bytes); });
    return hipSuccess;
}

void gemm_tn_plan(int64_t n, int32_t FP, int32_t FQ, int64_t* rows_per_split, int32_t* n_split)
{
    // any division of the rows into ranges that are multiples of 16 serves the host code; the sizes of the
    // workspaces it allocates from these numbers are what is being checked
    const int BN = FQ > 64 ? 128 : (FQ > 32 ? 64 : 32);
    const int BM = FQ > 64 ? 128 : (FQ > 32 ? 128 : 256);
    const int64_t tiles = (int64_t)((FP + BM - 1) / BM) * ((FQ + BN - 1) / BN);
    int64_t want = std::max<int64_t>(1, 2048 / std::max<int64_t>(tiles, 1));
    want = std::min<int64_t>(want, std::max<int64_t>(1, n / 256));
    want = std::min<int64_t>(want, 1024);
    int64_t rows = (std::max<int64_t>(n, 1) + want - 1) / want;
    rows = (rows + 15) / 16 * 16;
    *rows_per_split = rows;
    *n_split = (int32_t)std::max<int64_t>(1, (n + rows - 1) / rows);
}

hipError_t launch_gemm_tn(const GemmTnArgs& a, float* C, int64_t ldc, int accumulate, hipStream_t s)
{
    if (a.FP <= 0 || a.FQ <= 0) return hipSuccess;
    if (a.n_split < 1 || a.rows_per_split < 1 || a.rows_per_split % 16 != 0 || !a.part) return hipErrorInvalidValue;
    if ((int64_t)a.n_split * a.rows_per_split < a.n) return hipErrorInvalidValue;
    const GemmTnArgs copy = a;
    stub_enqueue(s, [copy, C, ldc, accumulate] {
        const GemmTnArgs& t = copy;
        const int64_t count = (int64_t)t.FP * t.FQ;
        for (int32_t k = 0; k < t.n_split; ++k) {
            const int64_t r0 = (int64_t)k * t.rows_per_split, r1 = std::min<int64_t>(t.n, r0 + t.rows_per_split);
            for (int32_t p = 0; p < t.FP; ++p)
                for (int32_t q = 0; q < t.FQ; ++q) {
                    double sum = 0.0;
                    for (int64_t r = r0; r < r1; ++r) sum += (double)t.P[r * t.ldp + p] * t.Q[r * t.ldq + q];
                    t.part[(int64_t)k * count + (int64_t)p * t.FQ + q] = (float)sum;
                }
        }
        for (int64_t i = 0; i < count; ++i) {
            float sum = 0.f;
            for (int32_t k = 0; k < t.n_split; ++k) sum += t.part[(int64_t)k * count + i];
            float* c = C + (i / t.FQ) * ldc + (i % t.FQ);
            *c = accumulate ? *c + sum : sum;
        }
    });
    return hipSuccess;
}

int64_t colsum_slabs(int64_t rows) { return std::max<int64_t>(1, std::min<int64_t>(1024, (rows + 127) / 128)); }

hipError_t launch_dz_colsum(const float* dY, int64_t lddy, const float* Y, int64_t ldy, int32_t act, float* dZ, int64_t rows, int32_t F,
                            float* part, float* dbias, int accumulate, hipStream_t s, int64_t lddz)
{
    if (F <= 0) return hipSuccess;
    if (lddz <= 0) lddz = F;
    if (act == SAGA_ACT_NONE) Y = nullptr;
    if (act != SAGA_ACT_NONE && !Y) return hipErrorInvalidValue;
    if (!Y && !part) return hipSuccess;
    stub_enqueue(s, [=] {
        const int64_t slabs = colsum_slabs(rows);
        const int64_t R = (std::max<int64_t>(rows, 1) + slabs - 1) / slabs;
        for (int64_t b = 0; b < slabs; ++b) {
            const int64_t r0 = b * R, r1 = std::min(rows, r0 + R);
            for (int32_t c = 0; c < F; ++c) {
                float sum = 0.f;
                for (int64_t r = r0; r < r1; ++r) {
                    float g = dY[r * lddy + c];
                    if (Y) {
                        const float y = Y[r * ldy + c];
                        g = act == SAGA_ACT_RELU ? (y > 0.f ? g : 0.f) : g * (y * (1.f - y));
                        dZ[r * lddz + c] = g;
                    }
                    sum += g;
                }
                if (part) part[b * F + c] = sum;
            }
        }
        if (part)
            for (int32_t c = 0; c < F; ++c) {
                float sum = 0.f;
                for (int64_t b = 0; b < slabs; ++b) sum += part[b * F + c];
                dbias[c] = accumulate ? dbias[c] + sum : sum;
            }
    });
    return hipSuccess;
}

hipError_t launch_dz_bf16(const uint16_t* dY, int64_t lddy, const uint16_t* Y, int64_t ldy, float* dZ32, uint16_t* dZ16, int64_t rows, int32_t F,
                          hipStream_t s)
{
    if (rows * F <= 0) return hipSuccess;
    stub_enqueue(s, [=] {
        for (int64_t r = 0; r < rows; ++r)
            for (int32_t c = 0; c < F; ++c) {
                uint16_t g = dY[r * lddy + c];
                if (Y && !(bf16_to_f32(Y[r * ldy + c]) > 0.f)) g = 0;
                if (dZ16) dZ16[r * F + c] = g;
                dZ32[r * F + c] = bf16_to_f32(g);
            }
    });
    return hipSuccess;
}

hipError_t launch_permute_f32(const float* in, const int32_t* perm, float* out, int64_t count, hipStream_t s)
{
    if (count <= 0) return hipSuccess;
    stub_enqueue(s, [=] {
        for (int64_t i = 0; i < count; ++i) out[i] = in[perm[i]];
    });
    return hipSuccess;
}

hipError_t launch_sigmoid_grad(float* d, const float* z, int64_t count, hipStream_t s)
{
    if (count <= 0) return hipSuccess;
    stub_enqueue(s, [=] {
        for (int64_t i = 0; i < count; ++i) {
            const double g = 1.0 / (1.0 + std::exp(-(double)z[i]));
            d[i] *= (float)(g * (1.0 - g));
        }
    });
    return hipSuccess;
}

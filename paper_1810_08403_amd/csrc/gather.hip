// Fused Scatter -> ApplyEdge -> Gather kernels for gfx950 (the fused-gather
// operator of Section 3.2, built on the kernel principle of Section 3.3:
// parallelise along the feature row of each vertex, one in-edge group per
// execution unit, accumulate in registers, write one row).
//
// What differs from the paper's P100 kernels:
//   * the execution unit is one 64-lane wavefront per work item, not a thread
//     block, and a lane moves 16 bytes per load, so a 1 KiB row is one
//     wave-wide load; narrower rows put several edges side by side in one
//     wavefront (64 / lanes-per-row edges per load) and finish with a
//     cross-lane reduction;
//   * per-edge tuples are never written: Scatter exists only as the loads;
//   * source ids reach the lanes through wave-uniform loads or one coalesced
//     64-id load plus lane permutes, not through shared memory;
//   * several independent row loads are kept in flight per lane to cover HBM
//     latency;
//   * heavy columns are cut into items of bounded length whose partial rows
//     are combined in a fixed order, so sums are reproducible.
//
// Kernels: k_gather_wide (rows of >= 64 fragments of 16 bytes), k_gather_narrow
// (fewer: several edges side by side in a wavefront), both templates over the
// per-edge function; k_gather_wide_mma / k_gather_narrow_mma (optional: bf16
// sums whose multiply-accumulate runs on the matrix unit); k_combine (partial
// rows of cut columns); k_stage_scatter / k_stage_apply_edge (the stages one by
// one through a per-edge tensor, the baseline the fused operator is measured
// against); small fill / copy / validation kernels.
#include <cmath>
#include <type_traits>

#include "device_math.h"
#include "saga_internal.h"

namespace {

constexpr int kWavesPerBlock = 4;
constexpr int kInFlight = 8;  // independent 16-byte loads per lane

__device__ __forceinline__ float neg_inf() { return -__builtin_huge_valf(); }

template <int AGG>
__device__ __forceinline__ float identity()
{
    return AGG == SAGA_AGG_SUM ? 0.0f : neg_inf();
}

// Gather's accumulate step. For max the message is formed first by a single
// multiply (no contraction is possible: there is no addition to fuse with), then one
// maximum instruction takes it in: fmaxf is the larger of two finite values whatever
// their order, bit for bit what `m > acc ? m : acc` gives (a compare and a select, which
// made the bf16 max layer of 512-wide rows ALU-bound) except for the sign of a zero maximum.
template <int AGG>
__device__ __forceinline__ float accumulate(float acc, float w, float x)
{
    if (AGG == SAGA_AGG_SUM) return fmaf(w, x, acc);
    return __builtin_fmaxf(w * x, acc);
}
template <int AGG>
__device__ __forceinline__ float combine(float a, float b)
{
    if (AGG == SAGA_AGG_SUM) return a + b;
    return __builtin_fmaxf(b, a);
}

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f)
{
    uint32_t x = __float_as_uint(f);
    if ((x & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((x >> 16) | 0x40u);  // NaN stays NaN
    x += 0x7fffu + ((x >> 16) & 1u);
    return (uint16_t)(x >> 16);
}

// ApplyVertex's bias and activation on a finished row element (transform-first layers)
__device__ __forceinline__ float finish_vertex(float y, float bias, int act)
{
    y += bias;
    if (act == SAGA_ACT_RELU) y = y > 0.f ? y : 0.f;
    if (act == SAGA_ACT_SIGMOID) y = sigmoid_f32(y);
    return y;
}

// A 16-byte store that is not going to be read again by this kernel (partial rows, finished rows): marked
// non-temporal so that it does not displace the band of source rows the wavefronts around it are sharing in the L2.
typedef float f32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void store_stream4(float* p, float a, float b, float c, float d)
{
    const f32x4_t v = {a, b, c, d};
    __builtin_nontemporal_store(v, reinterpret_cast<f32x4_t*>(p));
}

// ---- 16-byte (or one-element) row fragments --------------------------------
template <typename T, int VEC>
struct Frag;

template <>
struct Frag<float, 4> {
    uint4 r;
    __device__ __forceinline__ void load(const float* p) { r = *reinterpret_cast<const uint4*>(p); }
    __device__ __forceinline__ void zero() { r = make_uint4(0, 0, 0, 0); }
    __device__ __forceinline__ float get(int j) const
    {
        return __uint_as_float(j == 0 ? r.x : j == 1 ? r.y : j == 2 ? r.z : r.w);
    }
};
template <>
struct Frag<float, 1> {
    float r;
    __device__ __forceinline__ void load(const float* p) { r = *p; }
    __device__ __forceinline__ void zero() { r = 0.f; }
    __device__ __forceinline__ float get(int) const { return r; }
};
template <>
struct Frag<uint16_t, 8> {
    uint4 r;
    __device__ __forceinline__ void load(const uint16_t* p) { r = *reinterpret_cast<const uint4*>(p); }
    __device__ __forceinline__ void zero() { r = make_uint4(0, 0, 0, 0); }
    __device__ __forceinline__ float get(int j) const
    {
        const uint32_t d = (j >> 1) == 0 ? r.x : (j >> 1) == 1 ? r.y : (j >> 1) == 2 ? r.z : r.w;
        return __uint_as_float((j & 1) ? (d & 0xffff0000u) : (d << 16));
    }
};
template <>
struct Frag<uint16_t, 1> {
    uint16_t r;
    __device__ __forceinline__ void load(const uint16_t* p) { r = *p; }
    __device__ __forceinline__ void zero() { r = 0; }
    __device__ __forceinline__ float get(int) const { return __uint_as_float((uint32_t)r << 16); }
};

// Workgroups are dealt to the 8 XCDs round-robin. Within every run of
// 8 * kXcdRun workgroups, hand each XCD kXcdRun consecutive entries of the
// work list instead of every eighth one, so that the wavefronts resident on
// one XCD (about 1024) read neighbouring entries through one L2, while all
// XCDs still advance through the list at the same pace.
constexpr int kXcdRun = 256;
__device__ __forceinline__ int64_t logical_block(int remap)
{
    const int64_t b = blockIdx.x;
    if (!remap) return b;
    const int64_t group = b / (8 * kXcdRun);
    if (group >= (int64_t)gridDim.x / (8 * kXcdRun)) return b;  // ragged last run: as dealt
    const int64_t r = b - group * (8 * kXcdRun);
    return group * (8 * kXcdRun) + (r & 7) * kXcdRun + (r >> 3);
}

template <int VEC>
__device__ __forceinline__ void store_row(const GatherArgs& a, int v, int slot, int col0, const float (&val)[VEC],
                                          int agg, bool empty_column);

// The second row of the two-output edge function: same rules, its own destinations, fp32 only.
template <int VEC>
__device__ __forceinline__ void store_row2(const GatherArgs& a, int v, int slot, int col0, const float (&val)[VEC])
{
    GatherArgs b = a;
    b.out = a.out2;
    b.ld_out = a.ld_out2;
    b.partials = a.partials2;
    b.out16 = nullptr;
    store_row<VEC>(b, v, slot, col0, val, SAGA_AGG_SUM, false);
}

template <int VEC>
__device__ __forceinline__ void store_row(const GatherArgs& a, int v, int slot, int col0, const float (&val)[VEC],
                                          int agg, bool empty_column)
{
    // col0: first feature of this lane's fragment
    if (slot >= 0) {
        float* p = a.partials + (int64_t)slot * a.F + col0;
        if constexpr (VEC % 4 == 0) {
#pragma unroll
            for (int j = 0; j < VEC; j += 4)
                store_stream4(p + j, val[j], val[j + 1], val[j + 2], val[j + 3]);
        } else {
#pragma unroll
            for (int j = 0; j < VEC; ++j) p[j] = val[j];
        }
        return;
    }
    float outv[VEC];
#pragma unroll
    for (int j = 0; j < VEC; ++j) outv[j] = val[j];
    if (a.accumulate) {
        const float* p = a.out + (int64_t)v * a.ld_out + col0;
#pragma unroll
        for (int j = 0; j < VEC; ++j) outv[j] = agg == SAGA_AGG_SUM ? p[j] + outv[j] : (outv[j] > p[j] ? outv[j] : p[j]);
    } else if (agg == SAGA_AGG_MAX && empty_column) {
#pragma unroll
        for (int j = 0; j < VEC; ++j) outv[j] = 0.f;
    }
    if (a.bias || a.act != SAGA_ACT_NONE) {
#pragma unroll
        for (int j = 0; j < VEC; ++j) outv[j] = finish_vertex(outv[j], a.bias ? a.bias[col0 + j] : 0.f, a.act);
    }
    if (a.out) {
        float* p = a.out + (int64_t)v * a.ld_out + col0;
        if constexpr (VEC % 4 == 0) {
#pragma unroll
            for (int j = 0; j < VEC; j += 4)
                store_stream4(p + j, outv[j], outv[j + 1], outv[j + 2], outv[j + 3]);
        } else {
#pragma unroll
            for (int j = 0; j < VEC; ++j) p[j] = outv[j];
        }
    }
    if (a.out16) {
        uint16_t* p = a.out16 + (int64_t)v * a.ld_out16 + col0;
        if constexpr (VEC == 8) {
            uint4 pk;
            pk.x = f32_to_bf16_rne(outv[0]) | ((uint32_t)f32_to_bf16_rne(outv[1]) << 16);
            pk.y = f32_to_bf16_rne(outv[2]) | ((uint32_t)f32_to_bf16_rne(outv[3]) << 16);
            pk.z = f32_to_bf16_rne(outv[4]) | ((uint32_t)f32_to_bf16_rne(outv[5]) << 16);
            pk.w = f32_to_bf16_rne(outv[6]) | ((uint32_t)f32_to_bf16_rne(outv[7]) << 16);
            store_stream4(reinterpret_cast<float*>(p), __uint_as_float(pk.x), __uint_as_float(pk.y), __uint_as_float(pk.z), __uint_as_float(pk.w));
        } else {
#pragma unroll
            for (int j = 0; j < VEC; ++j) p[j] = f32_to_bf16_rne(outv[j]);
        }
    }
}

// A wavefront's share of the work list. Blocks [0, n_team) take one team item each: the four
// wavefronts of the block split its edges and reduce their rows through LDS (fixed order), so a
// long column costs one partial row per team item, not one per wavefront. Later blocks take
// four solo items, one per wavefront.
struct ItemView {
    int v, e0, e1, slot;  // e0..e1: this wavefront's edges
    bool team;
    bool empty_item;      // the whole item has no edges (only a solo item can)
};
__device__ __forceinline__ bool fetch_item(const GatherArgs& a, ItemView* it)
{
    const int wave = threadIdx.x >> 6;
    const int64_t blk = logical_block(a.xcd_remap);
    const bool team = blk < a.n_team;
    const int64_t id = team ? blk : a.n_team + (blk - a.n_team) * kWavesPerBlock + wave;
    if (id >= a.n_items) return false;  // only in the last solo block, where no barrier follows
    const int4 raw = *reinterpret_cast<const int4*>(a.items + id);
    it->v = __builtin_amdgcn_readfirstlane(raw.x);
    int e0 = __builtin_amdgcn_readfirstlane(raw.y);
    int e1 = __builtin_amdgcn_readfirstlane(raw.z);
    it->slot = __builtin_amdgcn_readfirstlane(raw.w);
    it->team = team;
    it->empty_item = e0 == e1;
    if (team) {
        // equal shares, rounded up to the unroll width of the edge loop
        const int per = (((e1 - e0 + kWavesPerBlock - 1) / kWavesPerBlock) + 7) & ~7;
        const int w = __builtin_amdgcn_readfirstlane(wave);
        e0 = min(e1, e0 + w * per);
        e1 = min(e1, e0 + per);
    }
    it->e0 = e0;
    it->e1 = e1;
    return true;
}

// Team reduction: wavefronts 1..3 park their row fragments in LDS (team_park), the block
// synchronises once, and wavefront 0 adds them in wavefront order (team_collect) and stores.
template <int NV>
__device__ __forceinline__ void team_park(float* red, int per_wave, int slot_in_wave, bool active, const float (&val)[NV])
{
    const int wave = threadIdx.x >> 6;
    if (wave > 0 && active) {
#pragma unroll
        for (int j = 0; j < NV; ++j) red[(wave - 1) * per_wave + slot_in_wave * NV + j] = val[j];
    }
}
template <int AGG, int NV>
__device__ __forceinline__ void team_collect(const float* red, int per_wave, int slot_in_wave, float (&val)[NV])
{
#pragma unroll
    for (int w = 0; w < kWavesPerBlock - 1; ++w)
#pragma unroll
        for (int j = 0; j < NV; ++j) val[j] = combine<AGG>(val[j], red[w * per_wave + slot_in_wave * NV + j]);
}

// ---------------------------------------------------------------------------
// rows of >= 64 fragments: every lane owns RC fragments of the row, one edge
// per wave-wide load, U edges in flight. The gated forms read two fragments per edge.
// ---------------------------------------------------------------------------
// Source ids and edge weights are read through the constant address space with
// wave-uniform addresses, so they arrive in scalar registers (read-only scalar
// loads) and the row base address is formed on the scalar unit.
typedef const int32_t __attribute__((address_space(4))) * const_i32_ptr;
typedef const float __attribute__((address_space(4))) * const_f32_ptr;

template <int U, bool TAIL, bool WEIGHTED>
__device__ __forceinline__ void fetch_ids_w(const_i32_ptr ridx, const_f32_ptr ew, int e, int e1, int (&u)[U], float (&w)[U])
{
#pragma unroll
    for (int k = 0; k < U; ++k) {
        // past the end of the item, re-read its last edge (always a valid address) and ignore it
        const int ee = TAIL ? min(e + k, e1 - 1) : e + k;
        u[k] = ridx[ee];
        w[k] = WEIGHTED ? ew[ee] : 1.0f;
    }
}
template <int U, bool TAIL>
__device__ __forceinline__ void fetch_ids(const_i32_ptr ridx, const_f32_ptr ew, int e, int e1, int (&u)[U], float (&w)[U])
{
    if (ew)
        fetch_ids_w<U, TAIL, true>(ridx, ew, e, e1, u, w);
    else
        fetch_ids_w<U, TAIL, false>(ridx, ew, e, e1, u, w);
}

// The per-edge function (template parameter EF). The gated forms read two rows per edge, x from
// `src` and m from `src2`, and per-item constant rows c1 (from `dst`) and, for the gradient form, c2
// (from `dst2`):
//   kEfLinear    acc (+)= w_e * x
//   kEfGate      acc (+)= sigmoid(x + c1) * m                      (forward message, and the message-part gradient)
//   kEfGateGrad  acc  += g (1 - g) * (c2 * m),  g = sigmoid(x + c1)  (gradient with respect to the gate's argument)
//   kEfGateBoth  both of the above at once from the same loads: acc += g (1 - g) * (c2 * m), acc2 += g * m
//   kEfMaxGrad   acc += w_e * m where w_e * c1 == x, else nothing   (gradient of a max Gather: x is the maximum that
//                was gathered at the other end of the edge, c1 this vertex's own row, so the test says "this vertex
//                supplied the maximum"; the product is the same single fp32 multiply that formed the message). With
//                `dst_sigmoid` the constant row is stored as pre-activations z and c1 = sigmoid(z) is formed once per
//                item, by the function the pooled rows were made with, so that the backward pass keeps z for the slope
//   kEfGateGradMax / kEfGateBothMax  the two gradient forms for a gated layer under the max accumulator: the edge
//                contributes only where its message equals the maximum that was gathered at the edge's destination,
//                sigmoid(x + c1) * m == c3 with c3 a third constant row (in-edge pass: the item is the destination), or
//                sigmoid(x + c1) * c2 == t with t a third row per edge (out-edge pass: the message's m is this item's
//                constant row c2, the destination's maximum travels with the edge). The message is formed by the very
//                expression of kEfGate (sigmoid_f32 of one fp32 sum, one multiply), so the comparison is bit for bit.
constexpr int kEfLinear = 0, kEfGate = 1, kEfGateGrad = 2, kEfGateBoth = 3, kEfMaxGrad = 4, kEfGateGradMax = 5, kEfGateBothMax = 6;
constexpr bool ef_is_grad(int ef) { return ef == kEfGateGrad || ef == kEfGateBoth || ef == kEfGateGradMax || ef == kEfGateBothMax; }
constexpr bool ef_is_both(int ef) { return ef == kEfGateBoth || ef == kEfGateBothMax; }
constexpr bool ef_third_row(int ef) { return ef == kEfGateBothMax; }    // a third row per edge
constexpr bool ef_third_const(int ef) { return ef == kEfGateGradMax; }  // a third constant row per item

template <int AGG, int EF>
__device__ __forceinline__ float edge_step(float acc, float w, float x, float m, float c1, float c2, float c3)
{
    if constexpr (EF == kEfGate) return accumulate<AGG>(acc, sigmoid_f32(x + c1), m);
    if constexpr (EF == kEfGateGrad || EF == kEfGateGradMax) {
        float g, slope;
        sigmoid_and_slope_f32(x + c1, g, slope);
        const float r = fmaf(slope, c2 * m, acc);
        if constexpr (EF == kEfGateGradMax) return sigmoid_f32(x + c1) * m == c3 ? r : acc;
        return r;
    }
    if constexpr (EF == kEfMaxGrad) {
        const float msg = w * c1;
        return msg == x ? fmaf(w, m, acc) : acc;
    }
    return accumulate<AGG>(acc, w, x);
}
template <int EF>
__device__ __forceinline__ void edge_step_both(float& acc, float& acc2, float x, float m, float c1, float c2, float t)
{
    float g, slope;
    sigmoid_and_slope_f32(x + c1, g, slope);
    const float r = fmaf(slope, c2 * m, acc), r2 = fmaf(g, m, acc2);
    if constexpr (EF == kEfGateBothMax) {
        const bool hit = sigmoid_f32(x + c1) * c2 == t;
        acc = hit ? r : acc;
        acc2 = hit ? r2 : acc2;
    } else {
        acc = r;
        acc2 = r2;
    }
}

// One group of up to U edges: issue every row load first, then consume.
// TAIL guards each edge with the wave-uniform predicate e + k < e1.
template <typename T, int VEC, int RC, int AGG, int EF, int U, bool TAIL>
__device__ __forceinline__ void wide_group(const T* __restrict__ X, const int64_t ld, const T* __restrict__ X2, const int64_t ld2,
                                           const T* __restrict__ X3, const int64_t ld3, const int (&u)[U], const int e, const int e1,
                                           const int (&col)[RC], Frag<T, VEC> (&x)[U][RC], Frag<T, VEC> (&m)[EF ? U : 1][EF ? RC : 1],
                                           Frag<T, VEC> (&t3)[ef_third_row(EF) ? U : 1][ef_third_row(EF) ? RC : 1])
{
#pragma unroll
    for (int k = 0; k < U; ++k) {
        if (TAIL && e + k >= e1) continue;
        const T* row = X + (int64_t)u[k] * ld;
        const T* row2 = X2 + (int64_t)u[k] * ld2;
        const T* row3 = X3 + (int64_t)u[k] * ld3;
#pragma unroll
        for (int c = 0; c < RC; ++c) {
            x[k][c].load(row + col[c]);
            if constexpr (EF != kEfLinear) m[k][c].load(row2 + col[c]);
            if constexpr (ef_third_row(EF)) t3[k][c].load(row3 + col[c]);
        }
    }
}
template <typename T, int VEC, int RC, int AGG, int EF, int U, bool TAIL>
__device__ __forceinline__ void wide_consume(const float (&w)[U], const int e, const int e1, const float (&c1)[RC][VEC],
                                             const float (&c2)[RC][VEC], const float (&c3)[RC][VEC], float (&acc)[RC][VEC],
                                             float (&acc2)[ef_is_both(EF) ? RC : 1][VEC], const Frag<T, VEC> (&x)[U][RC],
                                             const Frag<T, VEC> (&m)[EF ? U : 1][EF ? RC : 1],
                                             const Frag<T, VEC> (&t3)[ef_third_row(EF) ? U : 1][ef_third_row(EF) ? RC : 1])
{
#pragma unroll
    for (int k = 0; k < U; ++k) {
        if (TAIL && e + k >= e1) continue;
#pragma unroll
        for (int c = 0; c < RC; ++c)
#pragma unroll
            for (int jj = 0; jj < VEC; ++jj) {
                float mv = 0.f, tv = 0.f;
                if constexpr (EF != kEfLinear) mv = m[k][c].get(jj);
                if constexpr (ef_third_row(EF)) tv = t3[k][c].get(jj);
                if constexpr (ef_is_both(EF))
                    edge_step_both<EF>(acc[c][jj], acc2[c][jj], x[k][c].get(jj), mv, c1[c][jj], c2[c][jj], tv);
                else
                    acc[c][jj] = edge_step<AGG, EF>(acc[c][jj], w[k], x[k][c].get(jj), mv, c1[c][jj], c2[c][jj], c3[c][jj]);
            }
    }
}

template <typename T, int VEC, int RC, int AGG, int EF>
__global__ __launch_bounds__(256) void k_gather_wide(const GatherArgs a)
{
    ItemView it;
    if (!fetch_item(a, &it)) return;
    const int lane = threadIdx.x & 63;
    const int F = a.F;
    const int nvec = (F + VEC - 1) / VEC;
    constexpr bool GATED = EF != kEfLinear;
    constexpr bool ROW3 = ef_third_row(EF);
    constexpr int LOADS_PER_EDGE = RC * (ROW3 ? 3 : GATED ? 2 : 1);
    constexpr int U = (kInFlight / LOADS_PER_EDGE) > 0 ? (kInFlight / LOADS_PER_EDGE) : 1;
    const T* __restrict__ X = static_cast<const T*>(a.src);
    const T* __restrict__ X2 = GATED ? static_cast<const T*>(a.src2) : X;
    const int64_t ld2 = GATED ? a.ld_src2 : 0;
    const T* __restrict__ X3 = ROW3 ? static_cast<const T*>(a.src3) : X;
    const int64_t ld3 = ROW3 ? a.ld_src3 : 0;
    const const_i32_ptr ridx = (const_i32_ptr)(uintptr_t)a.row_idx;
    const const_f32_ptr ew = (GATED && EF != kEfMaxGrad) ? (const_f32_ptr)0 : (const_f32_ptr)(uintptr_t)a.edge_w;
    __shared__ float red[(kWavesPerBlock - 1) * 64 * RC * VEC];

    for (int cb = 0; cb < nvec; cb += 64 * RC) {
        float acc[RC][VEC];
        float acc2[ef_is_both(EF) ? RC : 1][VEC];
        float pd[RC][VEC], c2[RC][VEC], c3[RC][VEC];
        bool ok[RC];
#pragma unroll
        for (int c = 0; c < (ef_is_both(EF) ? RC : 1); ++c)
#pragma unroll
            for (int j = 0; j < VEC; ++j) acc2[c][j] = 0.f;
        int col[RC];
        int ldcol[RC];  // lanes past the end of the row re-read its first fragment and drop the result
#pragma unroll
        for (int c = 0; c < RC; ++c) {
            col[c] = (cb + lane + 64 * c) * VEC;
            ok[c] = (cb + lane + 64 * c) < nvec;
            ldcol[c] = ok[c] ? col[c] : 0;
#pragma unroll
            for (int j = 0; j < VEC; ++j) {
                acc[c][j] = identity<AGG>();
                pd[c][j] = 0.f;
                c2[c][j] = 0.f;
                c3[c][j] = 0.f;
            }
            if constexpr (GATED) {
                Frag<float, VEC> f;
                f.zero();
                if (ok[c]) f.load(a.dst + (int64_t)it.v * a.ld_dst + col[c]);
#pragma unroll
                for (int j = 0; j < VEC; ++j) pd[c][j] = f.get(j);
                if constexpr (EF == kEfMaxGrad)
                    if (a.dst_sigmoid) {  // the same function of the same fp32 value as the product that made the pooled rows
#pragma unroll
                        for (int j = 0; j < VEC; ++j) pd[c][j] = sigmoid_f32(pd[c][j]);
                    }
            }
            if constexpr (ef_is_grad(EF)) {
                Frag<float, VEC> f;
                f.zero();
                if (ok[c]) f.load(a.dst2 + (int64_t)it.v * a.ld_dst2 + col[c]);
#pragma unroll
                for (int j = 0; j < VEC; ++j) c2[c][j] = f.get(j);
            }
            if constexpr (ef_third_const(EF)) {
                Frag<float, VEC> f;
                f.zero();
                if (ok[c]) f.load(a.dst3 + (int64_t)it.v * a.ld_dst3 + col[c]);
#pragma unroll
                for (int j = 0; j < VEC; ++j) c3[c][j] = f.get(j);
            }
        }
        Frag<T, VEC> x[U][RC];
        Frag<T, VEC> m[GATED ? U : 1][GATED ? RC : 1];
        Frag<T, VEC> t3[ROW3 ? U : 1][ROW3 ? RC : 1];
        int u[U], un[U];
        float w[U], wn[U];
        int e = it.e0;
        if (e + U <= it.e1) fetch_ids<U, false>(ridx, ew, e, it.e1, un, wn);
        for (; e + U <= it.e1; e += U) {
#pragma unroll
            for (int k = 0; k < U; ++k) {
                u[k] = un[k];
                w[k] = wn[k];
            }
            wide_group<T, VEC, RC, AGG, EF, U, false>(X, a.ld_src, X2, ld2, X3, ld3, u, e, it.e1, ldcol, x, m, t3);
            // ids of the next full group travel while this group's rows do
            if (e + 2 * U <= it.e1) fetch_ids<U, false>(ridx, ew, e + U, it.e1, un, wn);
            wide_consume<T, VEC, RC, AGG, EF, U, false>(w, e, it.e1, pd, c2, c3, acc, acc2, x, m, t3);
        }
        if (e < it.e1) {
            fetch_ids<U, true>(ridx, ew, e, it.e1, u, w);
            wide_group<T, VEC, RC, AGG, EF, U, true>(X, a.ld_src, X2, ld2, X3, ld3, u, e, it.e1, ldcol, x, m, t3);
            wide_consume<T, VEC, RC, AGG, EF, U, true>(w, e, it.e1, pd, c2, c3, acc, acc2, x, m, t3);
        }
        if (it.team) {  // the same for every wavefront of the block, so the barriers are uniform
#pragma unroll
            for (int c = 0; c < RC; ++c) team_park<VEC>(red, 64 * RC * VEC, c * 64 + lane, ok[c], acc[c]);
            __syncthreads();
            if ((threadIdx.x >> 6) == 0) {
#pragma unroll
                for (int c = 0; c < RC; ++c)
                    if (ok[c]) {
                        team_collect<AGG, VEC>(red, 64 * RC * VEC, c * 64 + lane, acc[c]);
                        store_row<VEC>(a, it.v, it.slot, col[c], acc[c], AGG, false);
                    }
            }
            if constexpr (ef_is_both(EF)) {  // the second row through the same LDS space
                __syncthreads();
#pragma unroll
                for (int c = 0; c < RC; ++c) team_park<VEC>(red, 64 * RC * VEC, c * 64 + lane, ok[c], acc2[c]);
                __syncthreads();
                if ((threadIdx.x >> 6) == 0) {
#pragma unroll
                    for (int c = 0; c < RC; ++c)
                        if (ok[c]) {
                            team_collect<AGG, VEC>(red, 64 * RC * VEC, c * 64 + lane, acc2[c]);
                            store_row2<VEC>(a, it.v, it.slot, col[c], acc2[c]);
                        }
                }
            }
            if (cb + 64 * RC < nvec) __syncthreads();  // LDS is reused by the next block of columns
        } else {
#pragma unroll
            for (int c = 0; c < RC; ++c)
                if (ok[c]) {
                    store_row<VEC>(a, it.v, it.slot, col[c], acc[c], AGG, it.empty_item);
                    if constexpr (ef_is_both(EF)) store_row2<VEC>(a, it.v, it.slot, col[c], acc2[c]);
                }
        }
    }
}

// ---------------------------------------------------------------------------
// bf16 rows, sum over linear messages, with the multiply-accumulate on the matrix unit. The loads are
// those of k_gather_wide / k_gather_narrow; what changes is who does the arithmetic. Unpacking a bf16
// and one FMA per element costs two vector-ALU instructions per element (the narrow kernel on 512-byte
// rows keeps the vector ALUs busy 100 % of the time); here a lane only interleaves the halves of its
// registers (one byte-permute per two elements) and a 16x16x32 bf16 MFMA forms `acc += w_e * x` for
// four edges and two features per lane at once:
//
//   B (32 x 16, the data): column n = lane % 16, rows k = 8 (lane / 16) + j. A lane supplies, from its
//     own fragments, j = 0..3: feature 2p of its edges 4h..4h+3, j = 4..7: feature 2p + 1 of the same
//     edges (p = 0..3 feature pair, h = 0..1 half of a group of eight loads: eight MFMAs per group).
//   A (16 x 32, the weights): row i serves lane group kg = (i & 7) / 2 and feature 2p + (i & 1); it holds
//     that group's four edge weights at k = 8 kg + 4 (i & 1) + 0..3 and zero elsewhere, so that a lane
//     group only ever meets its own rows (and may work on other edges than its neighbours). Rows 0..7
//     carry the weights rounded to bf16, rows 8..15 the bf16-rounded remainder: w = hi + lo to 2^-18
//     relative, and the two partial sums are added at the end of the item.
//   C (16 x 16 fp32): lane (n, g) register r is row 4 g + r: all 256 values are in use.
//
// At the end of the item the rows of C go back to the lanes that own the features through a
// wavefront-private piece of LDS. Products of two bf16 values are exact in fp32 and the accumulation
// is fp32, as before. A non-finite feature of one source row turns every feature that shares a C
// column with it into NaN (0 x inf inside the dot product), not only its own.
// ---------------------------------------------------------------------------
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

constexpr uint32_t kPermLowHalves = 0x05040100u;   // (s0.lo16 << 16) | s1.lo16
constexpr uint32_t kPermHighHalves = 0x07060302u;  // (s0.hi16 << 16) | s1.hi16
constexpr uint32_t kPermZero = 0x0c0c0c0cu;

// What a lane contributes to the A operand: row i = lane % 16 belongs to lane group (i & 7) / 2, and only the
// lanes of that group hold its k range. `sel_part` picks this row's part of a weight out of a dword.
struct MmaLane {
    uint32_t sel0, sel1;  // byte selectors of the dwords 0..1 and 2..3 of A (zero selectors for lanes that supply nothing)
    bool low_rows;        // rows 8..15: the remainder part
};
__device__ __forceinline__ MmaLane mma_lane(const int lane, const uint32_t sel_hi, const uint32_t sel_lo)
{
    const int i = lane & 15, g = lane >> 4;
    const bool mine = ((i & 7) >> 1) == g;
    const uint32_t sel = i >= 8 ? sel_lo : sel_hi;
    return MmaLane{(mine && !(i & 1)) ? sel : kPermZero, (mine && (i & 1)) ? sel : kPermZero, i >= 8};
}

// Eight fragments (one per load of the group) and the eight weights that go with them, as dwords from which the
// lane's selectors take its part: acc[p] += sum over the loads of w * (features 2p, 2p + 1 of the fragment).
__device__ __forceinline__ void mma_consume(const Frag<uint16_t, 8> (&x)[8], const uint32_t (&wv)[8], const MmaLane ml,
                                            const bool second_half, f32x4_t (&acc)[4])
{
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        if (h == 1 && !second_half) break;  // the same for the whole wavefront
        u32x4_t av;
        av.x = __builtin_amdgcn_perm(wv[4 * h + 1], wv[4 * h], ml.sel0);
        av.y = __builtin_amdgcn_perm(wv[4 * h + 3], wv[4 * h + 2], ml.sel0);
        av.z = __builtin_amdgcn_perm(wv[4 * h + 1], wv[4 * h], ml.sel1);
        av.w = __builtin_amdgcn_perm(wv[4 * h + 3], wv[4 * h + 2], ml.sel1);
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const uint32_t d0 = p == 0 ? x[4 * h].r.x : p == 1 ? x[4 * h].r.y : p == 2 ? x[4 * h].r.z : x[4 * h].r.w;
            const uint32_t d1 = p == 0 ? x[4 * h + 1].r.x : p == 1 ? x[4 * h + 1].r.y : p == 2 ? x[4 * h + 1].r.z : x[4 * h + 1].r.w;
            const uint32_t d2 = p == 0 ? x[4 * h + 2].r.x : p == 1 ? x[4 * h + 2].r.y : p == 2 ? x[4 * h + 2].r.z : x[4 * h + 2].r.w;
            const uint32_t d3 = p == 0 ? x[4 * h + 3].r.x : p == 1 ? x[4 * h + 3].r.y : p == 2 ? x[4 * h + 3].r.z : x[4 * h + 3].r.w;
            u32x4_t bv;
            bv.x = __builtin_amdgcn_perm(d1, d0, kPermLowHalves);
            bv.y = __builtin_amdgcn_perm(d3, d2, kPermLowHalves);
            bv.z = __builtin_amdgcn_perm(d1, d0, kPermHighHalves);
            bv.w = __builtin_amdgcn_perm(d3, d2, kPermHighHalves);
            acc[p] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8_t, av), __builtin_bit_cast(bf16x8_t, bv),
                                                             acc[p], 0, 0, 0);
        }
    }
}

// End of an item: C row 4 g + r of column n belongs to lane 16 kg + n, feature 2 p + (row & 1), part row / 8.
// Every lane leaves with the eight sums of its own fragment (both parts added).
__device__ __forceinline__ void mma_collect(const f32x4_t (&acc)[4], float* const xw, const int lane, float (&val)[8])
{
    const int n = lane & 15, g = lane >> 4;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int row = 4 * g + r;
        const int owner = 16 * ((row & 7) >> 1) + n;
        float* const q = xw + ((row >> 3) * 64 + owner) * 8 + (row & 1);
#pragma unroll
        for (int p = 0; p < 4; ++p) q[2 * p] = acc[p][r];
    }
    // the exchange stays inside one wavefront, whose LDS operations complete in order
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int j = 0; j < 8; ++j) val[j] = xw[lane * 8 + j] + xw[(64 + lane) * 8 + j];
}

// Rows of 33..64 fragments: one edge per wave-wide load, ids and weights in scalar registers.
template <bool TAIL>
__device__ __forceinline__ void mma_wide_group(const uint16_t* __restrict__ X, const int64_t ld, const int (&u)[8], const float (&w)[8],
                                               const int cnt, const int ldcol, const MmaLane ml, f32x4_t (&acc)[4])
{
    Frag<uint16_t, 8> x[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        if (TAIL && k >= cnt)
            x[k].zero();
        else
            x[k].load(X + (int64_t)u[k] * ld + ldcol);
    }
    // this lane's part of every weight in the upper half of a dword: hi = bf16(w) for the rows 0..7,
    // bf16(w - hi) for the rows 8..15 (adding 0x8000 before the truncation rounds)
    const uint32_t lo_mask = ml.low_rows ? 0xffff0000u : 0u;
    uint32_t part[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        const float wk = (TAIL && k >= cnt) ? 0.f : w[k];
        const uint32_t hi = (__float_as_uint(wk) + 0x8000u) & 0xffff0000u;
        part[k] = __float_as_uint(wk - __uint_as_float(hi & lo_mask)) + 0x8000u;
    }
    mma_consume(x, part, ml, !TAIL || cnt > 4, acc);
}

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(7, 8))) void k_gather_wide_mma(const GatherArgs a)
{
    ItemView it;
    if (!fetch_item(a, &it)) return;  // launched without team items
    const int lane = threadIdx.x & 63;
    const int nvec = a.F / 8;  // 33..64
    const bool ok = lane < nvec;
    const int col = lane * 8;
    const int ldcol = ok ? col : 0;  // lanes past the end of the row re-read its first fragment and drop the result
    const uint16_t* __restrict__ X = static_cast<const uint16_t*>(a.src);
    const const_i32_ptr ridx = (const_i32_ptr)(uintptr_t)a.row_idx;
    const const_f32_ptr ew = (const_f32_ptr)(uintptr_t)a.edge_w;
    __shared__ float xch[kWavesPerBlock][2 * 64 * 8];
    const MmaLane ml = mma_lane(lane, kPermHighHalves, kPermHighHalves);

    f32x4_t acc[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) acc[p] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    int u[8], un[8];
    float w[8], wn[8];
    int e = it.e0;
    if (e + 8 <= it.e1) fetch_ids<8, false>(ridx, ew, e, it.e1, un, wn);
    for (; e + 8 <= it.e1; e += 8) {
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            u[k] = un[k];
            w[k] = wn[k];
        }
        // ids of the next full group travel while this group's rows do
        if (e + 16 <= it.e1) fetch_ids<8, false>(ridx, ew, e + 8, it.e1, un, wn);
        mma_wide_group<false>(X, a.ld_src, u, w, 8, ldcol, ml, acc);
    }
    if (e < it.e1) {
        fetch_ids<8, true>(ridx, ew, e, it.e1, u, w);
        mma_wide_group<true>(X, a.ld_src, u, w, it.e1 - e, ldcol, ml, acc);
    }
    float val[8];
    mma_collect(acc, xch[threadIdx.x >> 6], lane, val);
    if (ok) store_row<8>(a, it.v, it.slot, col, val, SAGA_AGG_SUM, false);
}

// Rows of 9..32 fragments: 2 or 4 edges side by side in one wave-wide load (lpr = 32 or 16 lanes per row, so a
// lane group of the MFMA never straddles two edges). Ids and weights of 64 edges are read one per lane and travel
// by lane permutes.
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(6, 8))) void k_gather_narrow_mma(const GatherArgs a, const int lpr_log2)
{
    ItemView it;
    if (!fetch_item(a, &it)) return;  // launched without team items
    const int lane = threadIdx.x & 63;
    const int nvec = a.F / 8;
    const int lpr = 1 << lpr_log2;
    const int sub = lane & (lpr - 1);
    const int grp = lane >> lpr_log2;
    const int epw_log2 = 6 - lpr_log2;  // 2 or 4 edges per wave-wide load
    const bool colok = sub < nvec;
    const int col = sub * 8;
    const int ldcol = colok ? col : 0;
    const uint16_t* __restrict__ X = static_cast<const uint16_t*>(a.src);
    const int32_t* __restrict__ ridx = a.row_idx;
    const float* __restrict__ ew = a.edge_w;
    const char* const xbase = reinterpret_cast<const char*>(X + ldcol);  // see k_gather_narrow
    const uint32_t ldb = (uint32_t)(a.ld_src * 2);
    const int grp4 = grp << 2;  // slot s < 64 of a batch lives in lane s: byte address 4 s of the lane permute
    __shared__ float xch[kWavesPerBlock][2 * 64 * 8];
    const MmaLane ml = mma_lane(lane, kPermHighHalves, kPermLowHalves);

    f32x4_t acc[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) acc[p] = f32x4_t{0.f, 0.f, 0.f, 0.f};

    // Ids and weights of a batch of 64 edges, one per lane. Slots past the end of the item repeat its last edge with
    // weight 0, so that every load step can run unguarded. The loaded values are not touched before the batch they
    // belong to starts: the next batch's are requested right after the first rows of this one.
    auto fetch_batch = [&](const int eb, int& id_out, float& w_out) {
        const int my = eb + lane;
        id_out = __builtin_nontemporal_load(ridx + min(my, it.e1 - 1));  // read once: kept out of the rows' way in the L2
        w_out = my < it.e1 ? (ew ? __builtin_nontemporal_load(ew + my) : 1.0f) : 0.f;
    };
    int idx_next = 0;
    float wt_next = 0.f;
    if (it.e0 < it.e1) fetch_batch(it.e0, idx_next, wt_next);
    for (int eb = it.e0; eb < it.e1; eb += 64) {
        const int idx = idx_next;
        // both bf16 parts of the weight in one dword, split once per edge (not once per use)
        const uint32_t w_hi = f32_to_bf16_rne(wt_next);
        const uint32_t wt = (w_hi << 16) | f32_to_bf16_rne(wt_next - __uint_as_float(w_hi << 16));
        const int cnt = min(64, it.e1 - eb);
        // groups of eight load steps, all issued before the first is consumed
        for (int j0 = 0; (j0 << epw_log2) < cnt; j0 += 8) {
            Frag<uint16_t, 8> x[8];
            uint32_t wv[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const uint32_t u = (uint32_t)__builtin_amdgcn_ds_bpermute(((j0 + k) << (epw_log2 + 2)) + grp4, idx);
                x[k].load(reinterpret_cast<const uint16_t*>(xbase + (uint64_t)u * ldb));
            }
            if (j0 == 0 && eb + 64 < it.e1) fetch_batch(eb + 64, idx_next, wt_next);
            // the weights are only needed when the rows are there: fetching them after the loads keeps their
            // registers free while the row addresses are formed
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int k = 0; k < 8; ++k) wv[k] = (uint32_t)__builtin_amdgcn_ds_bpermute(((j0 + k) << (epw_log2 + 2)) + grp4, (int)wt);
            mma_consume(x, wv, ml, ((j0 + 4) << epw_log2) < cnt, acc);
        }
    }
    float val[8];
    mma_collect(acc, xch[threadIdx.x >> 6], lane, val);
    for (int off = lpr; off < 64; off <<= 1)
#pragma unroll
        for (int j = 0; j < 8; ++j) val[j] += __shfl_xor(val[j], off);
    if (grp == 0 && colok) store_row<8>(a, it.v, it.slot, col, val, SAGA_AGG_SUM, false);
}

// ---------------------------------------------------------------------------
// rows of <= 32 fragments: lpr = 2^lpr_log2 lanes cover a row, 64 / lpr edges
// sit side by side in one wave-wide load; a butterfly over the lane groups
// finishes the reduction.
// ---------------------------------------------------------------------------
// Eight wavefronts per SIMD (64 registers) where the variant fits them without spilling: on graphs of many light columns
// a wavefront's life is one chain of three memory round trips (work item, source ids, rows) for a dozen edges, and the
// throughput is the number of resident wavefronts over that chain (CommNet on R-MAT 20: 19 wavefronts per compute unit
// on average at six per SIMD, propagation 1.24 ms; 1.18 ms at eight). The gate-gradient variants and the bf16 maximum
// need more registers: five and six.
constexpr int narrow_min_waves(int elem_bytes, int agg, int ef)
{
    return ef_is_grad(ef) ? 5 : (elem_bytes == 2 && agg == SAGA_AGG_MAX) ? 6 : 8;
}
template <typename T, int VEC, int AGG, int EF>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(narrow_min_waves(sizeof(T), AGG, EF), 8))) void k_gather_narrow(
    const GatherArgs a, const int lpr_log2)
{
    constexpr bool GATED = EF != kEfLinear;
    ItemView it;
    if (!fetch_item(a, &it)) return;
    const int lane = threadIdx.x & 63;
    const int F = a.F;
    const int nvec = (F + VEC - 1) / VEC;
    const int lpr = 1 << lpr_log2;
    const int sub = lane & (lpr - 1);
    const int grp = lane >> lpr_log2;
    const int epw_log2 = 6 - lpr_log2;
    const int epw = 1 << epw_log2;
    const bool colok = sub < nvec;
    const int col = sub * VEC;
    const int ldcol = colok ? col : 0;
    constexpr bool ROW3 = ef_third_row(EF);
    constexpr int U = ROW3 ? kInFlight / 3 : GATED ? kInFlight / 2 : kInFlight;
    const T* __restrict__ X = static_cast<const T*>(a.src);
    const T* __restrict__ X2 = GATED ? static_cast<const T*>(a.src2) : X;
    const int64_t ld2 = GATED ? a.ld_src2 : 0;
    const T* __restrict__ X3 = ROW3 ? static_cast<const T*>(a.src3) : X;
    const int64_t ld3 = ROW3 ? a.ld_src3 : 0;
    const int32_t* __restrict__ ridx = a.row_idx;
    const float* __restrict__ ew = a.edge_w;
    // row address = this lane's fragment of row 0 + id * bytes per row: one 32 x 32 -> 64-bit multiply-add
    // (the launcher checks that a row stride fits 32 bits)
    const char* const xbase = reinterpret_cast<const char*>(X + ldcol);
    const char* const xbase2 = reinterpret_cast<const char*>(X2 + ldcol);
    const char* const xbase3 = reinterpret_cast<const char*>(X3 + ldcol);
    const uint32_t ldb = (uint32_t)(a.ld_src * (int64_t)sizeof(T));
    const uint32_t ldb2 = (uint32_t)(ld2 * (int64_t)sizeof(T));
    const uint32_t ldb3 = (uint32_t)(ld3 * (int64_t)sizeof(T));
    const int grp4 = grp << 2;

    float acc[VEC], acc2[VEC], pd[VEC], c2[VEC], c3[VEC];
#pragma unroll
    for (int j = 0; j < VEC; ++j) {
        acc[j] = identity<AGG>();
        acc2[j] = 0.f;
        pd[j] = 0.f;
        c2[j] = 0.f;
        c3[j] = 0.f;
    }
    if constexpr (GATED) {
        Frag<float, VEC> f;
        f.zero();
        if (colok) f.load(a.dst + (int64_t)it.v * a.ld_dst + col);
#pragma unroll
        for (int j = 0; j < VEC; ++j) pd[j] = f.get(j);
        if constexpr (EF == kEfMaxGrad)
            if (a.dst_sigmoid) {
#pragma unroll
                for (int j = 0; j < VEC; ++j) pd[j] = sigmoid_f32(pd[j]);
            }
    }
    if constexpr (ef_is_grad(EF)) {
        Frag<float, VEC> f;
        f.zero();
        if (colok) f.load(a.dst2 + (int64_t)it.v * a.ld_dst2 + col);
#pragma unroll
        for (int j = 0; j < VEC; ++j) c2[j] = f.get(j);
    }
    if constexpr (ef_third_const(EF)) {
        Frag<float, VEC> f;
        f.zero();
        if (colok) f.load(a.dst3 + (int64_t)it.v * a.ld_dst3 + col);
#pragma unroll
        for (int j = 0; j < VEC; ++j) c3[j] = f.get(j);
    }

    // ids and weights of a batch of 64 edges, one per lane; the next batch's travel while this one's rows do
    auto fetch_batch = [&](const int eb, int& id_out, float& w_out) {
        const int my = eb + lane;
        id_out = 0;
        w_out = 1.0f;
        if (my < it.e1) {  // read once: keep them out of the way of the rows in the L2
            id_out = __builtin_nontemporal_load(ridx + my);
            if ((!GATED || EF == kEfMaxGrad) && ew) w_out = __builtin_nontemporal_load(ew + my);
        }
    };
    int idx_next;
    float wt_next;
    fetch_batch(it.e0, idx_next, wt_next);
    for (int eb = it.e0; eb < it.e1; eb += 64) {
        const int idx = idx_next;
        const float wt = wt_next;
        if (eb + 64 < it.e1) fetch_batch(eb + 64, idx_next, wt_next);
        const int cnt = min(64, it.e1 - eb);
        // `count` load steps starting at step j0, all issued before the first is consumed. CHECK: a step may reach past
        // the batch (only its last step can), so every lane tests its own slot; otherwise nothing is tested per lane.
        // Lanes past the end of a row (colok false) accumulate what they load from the row's first fragment and are
        // never stored, and the closing butterfly only mixes lanes of equal `sub`.
        auto steps = [&](const int j0, const int count, auto check_tag) {
            constexpr bool CHECK = decltype(check_tag)::value;
            Frag<T, VEC> x[U];
            Frag<T, VEC> m[GATED ? U : 1];
            Frag<T, VEC> t3[ROW3 ? U : 1];
            float w[U];
            bool ok[U];
#pragma unroll
            for (int k = 0; k < U; ++k) {
                if (k < count) {
                    const int s = ((j0 + k) << epw_log2) + grp;
                    ok[k] = !CHECK || s < cnt;
                    // slots past the end of the batch hold id 0: a valid row, loaded and dropped
                    // slot s < 64 of the batch lives in lane s: byte address 4 s of the lane permute
                    const int from = ((j0 + k) << (epw_log2 + 2)) + grp4;
                    const uint32_t u = (uint32_t)__builtin_amdgcn_ds_bpermute(from, idx);
                    w[k] = __int_as_float(__builtin_amdgcn_ds_bpermute(from, __float_as_int(wt)));
                    x[k].load(reinterpret_cast<const T*>(xbase + (uint64_t)u * ldb));
                    if constexpr (GATED) m[k].load(reinterpret_cast<const T*>(xbase2 + (uint64_t)u * ldb2));
                    if constexpr (ROW3) t3[k].load(reinterpret_cast<const T*>(xbase3 + (uint64_t)u * ldb3));
                }
            }
#pragma unroll
            for (int k = 0; k < U; ++k) {
                if (k < count) {
#pragma unroll
                    for (int j = 0; j < VEC; ++j) {
                        float mv = 0.f, tv = 0.f;
                        if constexpr (GATED) mv = m[k].get(j);
                        if constexpr (ROW3) tv = t3[k].get(j);
                        if constexpr (ef_is_both(EF)) {
                            float r = acc[j], r2 = acc2[j];
                            edge_step_both<EF>(r, r2, x[k].get(j), mv, pd[j], c2[j], tv);
                            acc[j] = (!CHECK || ok[k]) ? r : acc[j];
                            acc2[j] = (!CHECK || ok[k]) ? r2 : acc2[j];
                        } else {
                            const float r = edge_step<AGG, EF>(acc[j], w[k], x[k].get(j), mv, pd[j], c2[j], c3[j]);
                            acc[j] = (!CHECK || ok[k]) ? r : acc[j];
                        }
                    }
                }
            }
        };
        const int nfull = cnt >> epw_log2;  // steps whose slots all lie inside the batch
        int j0 = 0;
        for (; j0 + U <= nfull; j0 += U) steps(j0, U, std::false_type{});
        if (j0 < nfull) steps(j0, nfull - j0, std::false_type{});
        if (cnt & (epw - 1)) steps(nfull, 1, std::true_type{});
    }
    for (int off = lpr; off < 64; off <<= 1)
#pragma unroll
        for (int j = 0; j < VEC; ++j) {
            acc[j] = combine<AGG>(acc[j], __shfl_xor(acc[j], off));
            if constexpr (ef_is_both(EF)) acc2[j] += __shfl_xor(acc2[j], off);
        }
    if (it.team) {
        __shared__ float red[(kWavesPerBlock - 1) * 32 * VEC];
        team_park<VEC>(red, 32 * VEC, sub, grp == 0 && colok, acc);
        __syncthreads();
        if ((threadIdx.x >> 6) == 0 && grp == 0 && colok) {
            team_collect<AGG, VEC>(red, 32 * VEC, sub, acc);
            store_row<VEC>(a, it.v, it.slot, col, acc, AGG, false);
        }
        if constexpr (ef_is_both(EF)) {
            __syncthreads();
            team_park<VEC>(red, 32 * VEC, sub, grp == 0 && colok, acc2);
            __syncthreads();
            if ((threadIdx.x >> 6) == 0 && grp == 0 && colok) {
                team_collect<AGG, VEC>(red, 32 * VEC, sub, acc2);
                store_row2<VEC>(a, it.v, it.slot, col, acc2);
            }
        }
    } else if (grp == 0 && colok) {
        store_row<VEC>(a, it.v, it.slot, col, acc, AGG, it.empty_item);
        if constexpr (ef_is_both(EF)) store_row2<VEC>(a, it.v, it.slot, col, acc2);
    }
}

// ---------------------------------------------------------------------------
// combine the partial rows of split vertices, in slot order
// ---------------------------------------------------------------------------
// One thread per 16-byte fragment of a row (per element when the row does not allow fragments); the rows of as many
// cut columns as fit share a block. The partial rows are added strictly in slot order; four loads are issued before
// the first of them is added.
template <int AGG, int VEC>
__global__ __launch_bounds__(256) void k_combine(const CombineArgs a, const int tpr, const int rows_per_block)
{
    int hv, frag;
    if (rows_per_block == 1) {
        hv = blockIdx.x;
        frag = blockIdx.y * 256 + threadIdx.x;
    } else {
        hv = blockIdx.x * rows_per_block + threadIdx.x / tpr;
        frag = threadIdx.x % tpr;
        if ((int)threadIdx.x >= rows_per_block * tpr) return;
    }
    if (hv >= a.n_heavy || frag >= tpr) return;
    const HeavyVertex h = a.heavy[hv];
    const int f = frag * VEC;
    const float* p = a.partials + (int64_t)h.slot0 * a.F + f;
    auto load = [&](int slot, float (&v)[VEC]) {
        if constexpr (VEC == 4) {
            const f32x4_t x = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(p + (int64_t)slot * a.F));
            v[0] = x.x, v[1] = x.y, v[2] = x.z, v[3] = x.w;
        } else {
            v[0] = __builtin_nontemporal_load(p + (int64_t)slot * a.F);
        }
    };
    float r[VEC];
    load(0, r);
    int s = 1;
    for (; s + 4 <= h.nslots; s += 4) {
        float x0[VEC], x1[VEC], x2[VEC], x3[VEC];
        load(s, x0);
        load(s + 1, x1);
        load(s + 2, x2);
        load(s + 3, x3);
#pragma unroll
        for (int j = 0; j < VEC; ++j) r[j] = combine<AGG>(combine<AGG>(combine<AGG>(combine<AGG>(r[j], x0[j]), x1[j]), x2[j]), x3[j]);
    }
    for (; s < h.nslots; ++s) {
        float x[VEC];
        load(s, x);
#pragma unroll
        for (int j = 0; j < VEC; ++j) r[j] = combine<AGG>(r[j], x[j]);
    }
#pragma unroll
    for (int j = 0; j < VEC; ++j) {
        if (a.accumulate) r[j] = combine<AGG>(a.out[(int64_t)h.v * a.ld_out + f + j], r[j]);
        if (a.bias || a.act != SAGA_ACT_NONE) r[j] = finish_vertex(r[j], a.bias ? a.bias[f + j] : 0.f, a.act);
    }
    if (a.out) {
        float* o = a.out + (int64_t)h.v * a.ld_out + f;
        if constexpr (VEC == 4)
            store_stream4(o, r[0], r[1], r[2], r[3]);
        else
            o[0] = r[0];
    }
    if (a.out16) {
        uint16_t* o = a.out16 + (int64_t)h.v * a.ld_out16 + f;
        if constexpr (VEC == 4) {
            uint2 pk;
            pk.x = f32_to_bf16_rne(r[0]) | ((uint32_t)f32_to_bf16_rne(r[1]) << 16);
            pk.y = f32_to_bf16_rne(r[2]) | ((uint32_t)f32_to_bf16_rne(r[3]) << 16);
            *reinterpret_cast<uint2*>(o) = pk;
        } else {
            o[0] = f32_to_bf16_rne(r[0]);
        }
    }
}

__global__ __launch_bounds__(256) void k_fill_f32(float* p, int64_t count, float value)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (int64_t)gridDim.x * 256) p[i] = value;
}
__global__ __launch_bounds__(256) void k_neg_inf_to_zero(float* p, int64_t count)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (int64_t)gridDim.x * 256)
        if (p[i] == neg_inf()) p[i] = 0.f;
}
__global__ __launch_bounds__(256) void k_f32_to_bf16(const float* in, uint16_t* out, int64_t count)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (int64_t)gridDim.x * 256)
        out[i] = f32_to_bf16_rne(in[i]);
}
// The stages run one by one, for the comparison with the fused operator (Section 3.2; the paper's baseline without
// the optimised propagation, Section 6.2): Scatter writes the per-edge tensor S[e] = X[src e] (fp32), ApplyEdge
// turns it into the messages in place (one fp32 multiply by the edge weight), and Gather then reads the messages
// as rows of their own (edge e reads row e).
template <typename T>
__global__ __launch_bounds__(256) void k_stage_scatter(const T* __restrict__ X, int64_t ldx, const int32_t* __restrict__ src,
                                                       float* __restrict__ S, int F, int64_t n_edges)
{
    const int64_t total = n_edges * F;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int64_t e = i / F;
        const int f = (int)(i - e * F);
        const T x = X[(int64_t)src[e] * ldx + f];
        if constexpr (sizeof(T) == 4)
            S[i] = x;
        else
            S[i] = __uint_as_float((uint32_t)x << 16);
    }
}
__global__ __launch_bounds__(256) void k_stage_apply_edge(float* __restrict__ S, const float* __restrict__ w, int F, int64_t n_edges)
{
    const int64_t total = n_edges * F;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) S[i] = w[i / F] * S[i];
}
__global__ __launch_bounds__(256) void k_iota_i32(int32_t* p, int64_t count)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (int64_t)gridDim.x * 256) p[i] = (int32_t)i;
}
__global__ __launch_bounds__(256) void k_copy_u128(uint4* dst, const uint4* src, int64_t count)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (int64_t)gridDim.x * 256) dst[i] = src[i];
}
__global__ __launch_bounds__(256) void k_zero_u32(uint32_t* p, int64_t count)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (int64_t)gridDim.x * 256) p[i] = 0u;
}

// One wavefront per column: ids in range and strictly ascending.
__global__ __launch_bounds__(256) void k_validate_columns(const int64_t* col_ptr, int64_t n_cols, const int32_t* row_idx,
                                                          int64_t n_src, int32_t* flag)
{
    const int64_t v = (int64_t)blockIdx.x * kWavesPerBlock + (threadIdx.x >> 6);
    if (v >= n_cols) return;
    const int64_t e0 = col_ptr[v], e1 = col_ptr[v + 1];
    bool bad = false;
    for (int64_t e = e0 + (threadIdx.x & 63); e < e1; e += 64) {
        const int u = row_idx[e];
        if (u < 0 || u >= n_src) bad = true;
        if (e > e0 && row_idx[e - 1] >= u) bad = true;
    }
    if (bad) *flag = 1;
}

int grid_for(int64_t count) { return (int)std::min<int64_t>((count + 255) / 256, 65535 * 8); }

int ceil_log2(int x)
{
    int l = 0;
    while ((1 << l) < x) ++l;
    return l;
}

template <typename T, int VEC, int AGG, int EF>
hipError_t launch_shape(const GatherArgs& a, hipStream_t s)
{
    const int nvec = (a.F + VEC - 1) / VEC;
    const int64_t blocks = a.n_team + (a.n_items - a.n_team + kWavesPerBlock - 1) / kWavesPerBlock;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    const dim3 grid((unsigned)blocks), block(256);
    if (nvec <= 32) {
        hipLaunchKernelGGL((k_gather_narrow<T, VEC, AGG, EF>), grid, block, 0, s, a, ceil_log2(nvec));
    } else if (nvec <= 64) {
        hipLaunchKernelGGL((k_gather_wide<T, VEC, 1, AGG, EF>), grid, block, 0, s, a);
    } else if (nvec <= 128) {
        hipLaunchKernelGGL((k_gather_wide<T, VEC, 2, AGG, EF>), grid, block, 0, s, a);
    } else {
        hipLaunchKernelGGL((k_gather_wide<T, VEC, 4, AGG, EF>), grid, block, 0, s, a);
    }
    return hipGetLastError();
}

template <typename T, int VEC>
hipError_t launch_op(const GatherArgs& a, hipStream_t s)
{
    if constexpr (sizeof(T) == 4) {  // the gated forms work on fp32 hoisted rows only
        if (a.op == SAGA_EDGE_GATED)
            return a.agg == SAGA_AGG_SUM ? launch_shape<T, VEC, SAGA_AGG_SUM, kEfGate>(a, s)
                                         : launch_shape<T, VEC, SAGA_AGG_MAX, kEfGate>(a, s);
        if (a.op == kGatherOpGateGrad) return launch_shape<T, VEC, SAGA_AGG_SUM, kEfGateGrad>(a, s);
        if (a.op == kGatherOpGateBoth) return launch_shape<T, VEC, SAGA_AGG_SUM, kEfGateBoth>(a, s);
        if (a.op == kGatherOpMaxGrad) return launch_shape<T, VEC, SAGA_AGG_SUM, kEfMaxGrad>(a, s);
        if (a.op == kGatherOpGateGradMax) return launch_shape<T, VEC, SAGA_AGG_SUM, kEfGateGradMax>(a, s);
        if (a.op == kGatherOpGateBothMax) return launch_shape<T, VEC, SAGA_AGG_SUM, kEfGateBothMax>(a, s);
    }
    return a.agg == SAGA_AGG_SUM ? launch_shape<T, VEC, SAGA_AGG_SUM, kEfLinear>(a, s)
                                 : launch_shape<T, VEC, SAGA_AGG_MAX, kEfLinear>(a, s);
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

hipError_t launch_gather(const GatherArgs& a, hipStream_t s)
{
    if (a.n_items <= 0) return hipSuccess;
    const int esize = a.dtype == SAGA_F32 ? 4 : 2;
    const int vec = 16 / esize;
    bool vec_ok = a.F % vec == 0 && (a.ld_src * esize) % 16 == 0 && aligned16(a.src);
    if (a.out) vec_ok = vec_ok && (a.ld_out * 4) % 16 == 0 && aligned16(a.out);
    if (a.out16) vec_ok = vec_ok && (a.ld_out16 * 2) % 16 == 0 && aligned16(a.out16);
    if (a.partials) vec_ok = vec_ok && aligned16(a.partials);
    if ((a.bias || a.act != SAGA_ACT_NONE) && a.accumulate) return hipErrorInvalidValue;
    if (a.ld_src < 0 || a.ld_src >= (1LL << 30) || a.ld_src2 < 0 || a.ld_src2 >= (1LL << 30))
        return hipErrorInvalidValue;  // the kernels form row offsets in bytes with 32-bit row strides
    const bool both = a.op == kGatherOpGateBoth || a.op == kGatherOpGateBothMax;
    const bool grad = a.op == kGatherOpGateGrad || a.op == kGatherOpGateGradMax || both;
    const bool gated = a.op == SAGA_EDGE_GATED || grad || a.op == kGatherOpMaxGrad;
    if (gated) {
        if (!a.src2 || !a.dst || (grad && (!a.dst2 || a.agg != SAGA_AGG_SUM))) return hipErrorInvalidValue;
        if (a.op == kGatherOpMaxGrad && a.agg != SAGA_AGG_SUM) return hipErrorInvalidValue;
        vec_ok = vec_ok && (a.ld_dst * 4) % 16 == 0 && aligned16(a.dst) && (a.ld_src2 * 4) % 16 == 0 && aligned16(a.src2);
        if (grad) vec_ok = vec_ok && (a.ld_dst2 * 4) % 16 == 0 && aligned16(a.dst2);
        if (a.op == kGatherOpGateGradMax) {
            if (!a.dst3) return hipErrorInvalidValue;
            vec_ok = vec_ok && (a.ld_dst3 * 4) % 16 == 0 && aligned16(a.dst3);
        }
        if (a.op == kGatherOpGateBothMax) {
            if (!a.src3 || a.ld_src3 < 0 || a.ld_src3 >= (1LL << 30)) return hipErrorInvalidValue;
            vec_ok = vec_ok && (a.ld_src3 * 4) % 16 == 0 && aligned16(a.src3);
        }
        if (both) {
            if (!a.out || !a.out2 || a.out16 || (a.partials && !a.partials2)) return hipErrorInvalidValue;
            vec_ok = vec_ok && (a.ld_out2 * 4) % 16 == 0 && aligned16(a.out2) && (!a.partials2 || aligned16(a.partials2));
        }
    }
    if (a.dtype == SAGA_F32) return vec_ok ? launch_op<float, 4>(a, s) : launch_op<float, 1>(a, s);
    if (gated) return hipErrorInvalidValue;
    if (a.mma && vec_ok && a.agg == SAGA_AGG_SUM && a.n_team == 0 && a.F > 8 * 8 && a.F <= 64 * 8) {
        const int64_t blocks = (a.n_items + kWavesPerBlock - 1) / kWavesPerBlock;
        if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
        const int nvec = a.F / 8;
        if (nvec > 32)
            hipLaunchKernelGGL(k_gather_wide_mma, dim3((unsigned)blocks), dim3(256), 0, s, a);
        else
            hipLaunchKernelGGL(k_gather_narrow_mma, dim3((unsigned)blocks), dim3(256), 0, s, a, nvec > 16 ? 5 : 4);
        return hipGetLastError();
    }
    return vec_ok ? launch_op<uint16_t, 8>(a, s) : launch_op<uint16_t, 1>(a, s);
}

hipError_t launch_combine(const CombineArgs& a, hipStream_t s)
{
    if (a.n_heavy <= 0) return hipSuccess;
    bool vec = a.F % 4 == 0 && aligned16(a.partials);
    if (a.out) vec = vec && a.ld_out % 4 == 0 && aligned16(a.out);
    if (a.out16) vec = vec && a.ld_out16 % 4 == 0 && (reinterpret_cast<uintptr_t>(a.out16) & 7u) == 0;
    const int tpr = vec ? a.F / 4 : a.F;  // threads per row
    const int rows_per_block = tpr >= 256 ? 1 : 256 / tpr;
    const dim3 grid(rows_per_block == 1 ? (unsigned)a.n_heavy : (unsigned)((a.n_heavy + rows_per_block - 1) / rows_per_block),
                    rows_per_block == 1 ? (unsigned)((tpr + 255) / 256) : 1u),
        block(256);
    if (a.agg == SAGA_AGG_SUM) {
        if (vec)
            hipLaunchKernelGGL((k_combine<SAGA_AGG_SUM, 4>), grid, block, 0, s, a, tpr, rows_per_block);
        else
            hipLaunchKernelGGL((k_combine<SAGA_AGG_SUM, 1>), grid, block, 0, s, a, tpr, rows_per_block);
    } else {
        if (vec)
            hipLaunchKernelGGL((k_combine<SAGA_AGG_MAX, 4>), grid, block, 0, s, a, tpr, rows_per_block);
        else
            hipLaunchKernelGGL((k_combine<SAGA_AGG_MAX, 1>), grid, block, 0, s, a, tpr, rows_per_block);
    }
    return hipGetLastError();
}

hipError_t launch_fill_f32(float* p, int64_t count, float value, hipStream_t s)
{
    if (count <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_fill_f32, dim3(grid_for(count)), dim3(256), 0, s, p, count, value);
    return hipGetLastError();
}
hipError_t launch_neg_inf_to_zero(float* p, int64_t count, hipStream_t s)
{
    if (count <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_neg_inf_to_zero, dim3(grid_for(count)), dim3(256), 0, s, p, count);
    return hipGetLastError();
}
hipError_t launch_f32_to_bf16(const float* in, uint16_t* out, int64_t count, hipStream_t s)
{
    if (count <= 0) return hipSuccess;
    hipLaunchKernelGGL(k_f32_to_bf16, dim3(grid_for(count)), dim3(256), 0, s, in, out, count);
    return hipGetLastError();
}
hipError_t launch_stage_scatter_apply(const void* X, int64_t ldx, int32_t dtype, const int32_t* src, const float* edge_w, float* S,
                                      int32_t* iota, int32_t F, int64_t n_edges, hipStream_t s)
{
    if (n_edges <= 0 || F <= 0) return hipSuccess;
    const int64_t total = n_edges * F;
    if (dtype == SAGA_F32)
        hipLaunchKernelGGL(k_stage_scatter<float>, dim3(grid_for(total)), dim3(256), 0, s, static_cast<const float*>(X), ldx, src, S, F, n_edges);
    else
        hipLaunchKernelGGL(k_stage_scatter<uint16_t>, dim3(grid_for(total)), dim3(256), 0, s, static_cast<const uint16_t*>(X), ldx, src, S, F,
                           n_edges);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (edge_w) {
        hipLaunchKernelGGL(k_stage_apply_edge, dim3(grid_for(total)), dim3(256), 0, s, S, edge_w, F, n_edges);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    hipLaunchKernelGGL(k_iota_i32, dim3(grid_for(n_edges)), dim3(256), 0, s, iota, n_edges);
    return hipGetLastError();
}
hipError_t launch_zero_bytes(void* p, size_t bytes, hipStream_t s)
{
    // a fill kernel rather than hipMemsetAsync, so the call is safe under graph capture
    if (bytes == 0) return hipSuccess;
    if (bytes % 4 != 0 || !((reinterpret_cast<uintptr_t>(p) & 3u) == 0)) return hipErrorInvalidValue;
    const int64_t count = (int64_t)(bytes / 4);
    hipLaunchKernelGGL(k_zero_u32, dim3(grid_for(count)), dim3(256), 0, s, static_cast<uint32_t*>(p), count);
    return hipGetLastError();
}
hipError_t launch_copy_bytes(void* dst, const void* src, size_t bytes, hipStream_t s)
{
    if (bytes == 0) return hipSuccess;
    if (bytes % 16 != 0 || (reinterpret_cast<uintptr_t>(dst) & 15u) || (reinterpret_cast<uintptr_t>(src) & 15u))
        return hipErrorInvalidValue;
    const int64_t count = (int64_t)(bytes / 16);
    hipLaunchKernelGGL(k_copy_u128, dim3(grid_for(count)), dim3(256), 0, s, static_cast<uint4*>(dst),
                       static_cast<const uint4*>(src), count);
    return hipGetLastError();
}
hipError_t launch_validate_columns(const int64_t* col_ptr, int64_t n_cols, const int32_t* row_idx, int64_t n_src,
                                   int32_t* flag, hipStream_t s)
{
    if (n_cols <= 0) return hipSuccess;
    const int64_t blocks = (n_cols + kWavesPerBlock - 1) / kWavesPerBlock;
    hipLaunchKernelGGL(k_validate_columns, dim3((unsigned)blocks), dim3(256), 0, s, col_ptr, n_cols, row_idx, n_src, flag);
    return hipGetLastError();
}

// Parameter gradients of backward-ApplyVertex (Section 2.2): C[FP x FQ] = P^T Q, a
// contraction over all vertices of two row-major fp32 matrices (P = the Gather output or
// the vertices' own features, Q = the gradient of the pre-activation). Both operands are
// read the way they are stored, a vertex's features contiguous, so neither is transposed:
// for the 32x32x2 MFMA a lane's operand is one element (feature l % 32, vertex l / 32),
// which is a row-contiguous read of a K tile staged in LDS as [vertex][feature].
//
// The vertex range is divided over gridDim splits (the output is tiny, the contraction
// long); every split writes its own FP x FQ partial and a second kernel adds the partials
// in split order, so the result does not depend on scheduling. The same file holds the
// two small reductions beside it: the activation's derivative applied to the incoming
// gradient, and the column sums that give the bias gradient.
#include "saga_internal.h"
#include "device_math.h"

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kKT = 16;       // vertices per K tile
constexpr int kPadCols = 32;  // LDS row padding (floats): consecutive vertices start 32 banks apart

// One K tile, global -> registers. Thread t owns 4-float chunks t, t + 256, ... of the
// [kKT][BM + BN] tile. Rows past the split's end and columns past the matrix are zero.
template <int BM, int BN, bool ALIGNED, int CH>
__device__ __forceinline__ void tn_load(const GemmTnArgs& a, int64_t v0, int64_t v_end, int i0, int j0, int tid, f32x4 (&r)[CH])
{
    constexpr int CPR = (BM + BN) / 4;  // chunks per tile row
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const int id = tid + 256 * c;
        const int k = id / CPR, cc = id % CPR;
        const bool isq = cc >= BM / 4;
        const int col = isq ? j0 + (cc - BM / 4) * 4 : i0 + cc * 4;
        const int lim = isq ? a.FQ : a.FP;
        const float* base = isq ? a.Q : a.P;
        const int64_t ld = isq ? a.ldq : a.ldp;
        const int64_t v = v0 + k;
        f32x4 x = {0.f, 0.f, 0.f, 0.f};
        if (id < kKT * CPR && v < v_end) {
            const float* p = base + v * ld + col;
            if (ALIGNED) {
                if (col + 4 <= lim) x = *reinterpret_cast<const f32x4*>(p);  // lim % 4 == 0: a chunk is inside or outside
            } else {
                if (col + 0 < lim) x.x = p[0];
                if (col + 1 < lim) x.y = p[1];
                if (col + 2 < lim) x.z = p[2];
                if (col + 3 < lim) x.w = p[3];
            }
        }
        r[c] = x;
    }
}

template <int BM, int BN, int CH>
__device__ __forceinline__ void tn_store(float* buf, int tid, const f32x4 (&r)[CH])
{
    constexpr int CPR = (BM + BN) / 4, LD = BM + BN + kPadCols;
#pragma unroll
    for (int c = 0; c < CH; ++c) {
        const int id = tid + 256 * c;
        if (kKT * CPR % 256 == 0 || id < kKT * CPR) *reinterpret_cast<f32x4*>(buf + (id / CPR) * LD + (id % CPR) * 4) = r[c];
    }
}

template <int BM, int BN, int WM, int WN, bool ALIGNED>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(1, 3))) void k_gemm_tn(const GemmTnArgs a, const int tiles_m, const int tiles_n)
{
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32, LD = BM + BN + kPadCols;
    constexpr int CH = (kKT * (BM + BN) / 4 + 255) / 256;
    static_assert(WM * WN == 4 && TM >= 1 && TN >= 1, "tile shape");
    __shared__ __attribute__((aligned(16))) float lds[2][kKT * LD];

    // blocks b, b + 8, b + 16, ... run on one XCD: give them the tiles of one split, which
    // read the same vertex rows
    const int T = tiles_m * tiles_n;
    const int64_t b = blockIdx.x;
    const int64_t grp = b / (8 * (int64_t)T);
    const int within = (int)(b % (8 * (int64_t)T));
    const int64_t split = grp * 8 + (within & 7);
    const int tile = within >> 3;
    if (split >= a.n_split) return;
    const int i0 = (tile / tiles_n) * BM, j0 = (tile % tiles_n) * BN;
    const int64_t v_begin = split * a.rows_per_split;
    const int64_t v_end = v_begin + a.rows_per_split < a.n ? v_begin + a.rows_per_split : a.n;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WM, wn = wave / WM;

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    f32x4 regs[CH];
    const int64_t nk = (v_end - v_begin + kKT - 1) / kKT;
    if (nk > 0) {
        tn_load<BM, BN, ALIGNED>(a, v_begin, v_end, i0, j0, tid, regs);
        tn_store<BM, BN>(lds[0], tid, regs);
    }
    __syncthreads();
    for (int64_t kt = 0; kt < nk; ++kt) {
        // the last iteration loads past the end of the split: all zeros, never used
        tn_load<BM, BN, ALIGNED>(a, v_begin + (kt + 1) * kKT, kt + 1 < nk ? v_end : 0, i0, j0, tid, regs);
        __builtin_amdgcn_sched_barrier(0);
        const float* base = lds[kt & 1] + (lane >> 5) * LD + (lane & 31);
#pragma unroll
        for (int kk = 0; kk < kKT / 2; ++kk) {
            float fa[TM], fb[TN];
#pragma unroll
            for (int i = 0; i < TM; ++i) fa[i] = base[kk * 2 * LD + (wm * TM + i) * 32];
#pragma unroll
            for (int j = 0; j < TN; ++j) fb[j] = base[kk * 2 * LD + BM + (wn * TN + j) * 32];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        tn_store<BM, BN>(lds[(kt + 1) & 1], tid, regs);
        __syncthreads();
    }

    // this split's partial: lane holds column (lane & 31) of 16 rows of each 32 x 32 block
    float* __restrict__ out = a.part + split * (int64_t)a.FP * a.FQ;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int col = j0 + (wn * TN + j) * 32 + (lane & 31);
        if (col >= a.FQ) continue;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int row0 = i0 + (wm * TM + i) * 32 + (lane >> 5) * 4;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int row = row0 + (r >> 2) * 8 + (r & 3);
                if (row < a.FP) out[(int64_t)row * a.FQ + col] = acc[i][j][r];
            }
        }
    }
}

// C[r][c] = sum over splits. A block owns 64 consecutive elements; its four wavefronts each add
// every fourth split in order, and wavefront 0 adds the four sums in order: the grouping is fixed
// by n_split alone.
__global__ __launch_bounds__(256) void k_sum_splits(const float* __restrict__ part, int64_t count, int n_split, int FQ, float* __restrict__ C,
                                                    int64_t ldc, int accumulate)
{
    __shared__ float red[4][64];
    const int e = threadIdx.x & 63, q = threadIdx.x >> 6;
    const int64_t i = (int64_t)blockIdx.x * 64 + e;
    float s = 0.f;
    if (i < count)
        for (int k = q; k < n_split; k += 4) s += part[(int64_t)k * count + i];
    red[q][e] = s;
    __syncthreads();
    if (q == 0 && i < count) {
        float* c = C + (i / FQ) * ldc + (i % FQ);
        const float r = ((red[0][e] + red[1][e]) + red[2][e]) + red[3][e];
        *c = accumulate ? *c + r : r;  // accumulate: a later tile of rows adds to what earlier tiles left (streamed calls)
    }
}

// backward-ApplyVertex's elementwise part over a slab of rows: the activation's derivative taken from the
// layer's output (MODE 1, ReLU: dZ = dY where Y > 0, else 0; MODE 2, sigmoid: dZ = dY * Y (1 - Y); MODE 0: dZ
// is dY itself and nothing is stored), and the slab's column sums of dZ for the bias gradient. A thread owns VEC consecutive columns
// and every RL-th row of the slab (RL row lanes when the matrix is narrower than the block); the
// row lanes' sums are added in lane order.
__device__ __forceinline__ float act_grad(int mode, float g, float y)
{
    if (mode == 1) return y > 0.f ? g : 0.f;
    return g * (y * (1.0f - y));
}

template <int VEC, int MODE>
__global__ __launch_bounds__(256) void k_dz_colsum(const float* __restrict__ dY, int64_t lddy, const float* __restrict__ Y, int64_t ldy,
                                                   float* __restrict__ dZ, int64_t lddz, int64_t rows, int F, int64_t R,
                                                   float* __restrict__ part)
{
    __shared__ float red[256 * VEC];
    const int ncg = (F + VEC - 1) / VEC;                  // column groups
    const int RL = ncg >= 256 ? 1 : 256 / ncg;            // row lanes
    const int64_t r0 = (int64_t)blockIdx.x * R;
    const int64_t r1 = r0 + R < rows ? r0 + R : rows;
    for (int cg0 = 0; cg0 < ncg; cg0 += 256) {            // one pass unless the matrix is wider than 256 groups
        const int t = threadIdx.x;
        const int cg = cg0 + (RL == 1 ? t : t % ncg), rl = RL == 1 ? 0 : t / ncg;
        const bool live = cg < ncg && rl < RL;
        float sum[VEC];
#pragma unroll
        for (int j = 0; j < VEC; ++j) sum[j] = 0.f;
        if (live) {
            const int c = cg * VEC;
            for (int64_t r = r0 + rl; r < r1; r += RL) {
                float g[VEC];
                if constexpr (VEC == 4) {
                    const float4 a = *reinterpret_cast<const float4*>(dY + r * lddy + c);
                    g[0] = a.x, g[1] = a.y, g[2] = a.z, g[3] = a.w;
                    if (MODE) {
                        const float4 y = *reinterpret_cast<const float4*>(Y + r * ldy + c);
                        g[0] = act_grad(MODE, g[0], y.x), g[1] = act_grad(MODE, g[1], y.y);
                        g[2] = act_grad(MODE, g[2], y.z), g[3] = act_grad(MODE, g[3], y.w);
                        *reinterpret_cast<float4*>(dZ + r * lddz + c) = make_float4(g[0], g[1], g[2], g[3]);
                    }
                } else {
                    g[0] = dY[r * lddy + c];
                    if (MODE) {
                        g[0] = act_grad(MODE, g[0], Y[r * ldy + c]);
                        dZ[r * lddz + c] = g[0];
                    }
                }
#pragma unroll
                for (int j = 0; j < VEC; ++j) sum[j] += g[j];
            }
        }
        if (part) {
            __syncthreads();
#pragma unroll
            for (int j = 0; j < VEC; ++j) red[t * VEC + j] = sum[j];
            __syncthreads();
            if (live && rl == 0) {
#pragma unroll
                for (int j = 0; j < VEC; ++j) {
                    float s = 0.f;
                    for (int l = 0; l < RL; ++l) s += red[(RL == 1 ? t : l * ncg + (cg - cg0)) * VEC + j];
                    if (cg * VEC + j < F) part[(int64_t)blockIdx.x * F + cg * VEC + j] = s;
                }
            }
        }
    }
}

// bf16 layers: dZ = dY where Y > 0 (or dY itself without Y), written twice, as fp32 for the parameter-gradient product
// and the bias sums, and as bf16 (the same values) for the propagation and the products that run in bf16
__global__ __launch_bounds__(256) void k_dz_bf16(const uint16_t* __restrict__ dY, int64_t lddy, const uint16_t* __restrict__ Y, int64_t ldy,
                                                 float* __restrict__ dZ32, uint16_t* __restrict__ dZ16, int64_t rows, int F)
{
    const int64_t total = rows * F;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int64_t r = i / F;
        const int c = (int)(i % F);
        uint16_t g = dY[r * lddy + c];
        if (Y) {
            const uint16_t y = Y[r * ldy + c];
            const bool pos = (y & 0x7fffu) != 0 && (y & 0x8000u) == 0 && (y & 0x7fffu) <= 0x7f80u;  // y > 0, not NaN
            g = pos ? g : (uint16_t)0;
        }
        if (dZ16) dZ16[i] = g;  // NULL: only the fp32 copy is wanted (the rows of X for dW_self)
        dZ32[i] = __uint_as_float((uint32_t)g << 16);
    }
}

// out[i] = in[perm[i]]
__global__ __launch_bounds__(256) void k_permute_f32(const float* __restrict__ in, const int32_t* __restrict__ perm, float* __restrict__ out,
                                                     int64_t count)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (int64_t)gridDim.x * 256) out[i] = in[perm[i]];
}

// d[i] *= sigmoid'(z[i]). The slope is formed from the pre-activation, not from a stored sigmoid h as h (1 - h): an
// fp32 h close to 1 has lost 1 - h (z = 9: 1 - h = 1.2e-4 known to 2^-25, a relative error of 2.4e-4 in the slope).
__global__ __launch_bounds__(256) void k_sigmoid_grad(float* __restrict__ d, const float* __restrict__ z, int64_t count)
{
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < count; i += (int64_t)gridDim.x * 256) {
        float g, slope;
        sigmoid_and_slope_f32(z[i], g, slope);
        d[i] *= slope;
    }
}

template <int BM, int BN, int WM, int WN>
hipError_t launch_tn_cfg(const GemmTnArgs& a, bool aligned, hipStream_t s)
{
    const int tiles_m = (a.FP + BM - 1) / BM, tiles_n = (a.FQ + BN - 1) / BN;
    const int64_t groups = (a.n_split + 7) / 8;
    const int64_t blocks = groups * 8 * tiles_m * tiles_n;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    if (aligned)
        hipLaunchKernelGGL((k_gemm_tn<BM, BN, WM, WN, true>), dim3((unsigned)blocks), dim3(256), 0, s, a, tiles_m, tiles_n);
    else
        hipLaunchKernelGGL((k_gemm_tn<BM, BN, WM, WN, false>), dim3((unsigned)blocks), dim3(256), 0, s, a, tiles_m, tiles_n);
    return hipGetLastError();
}

}  // namespace

void gemm_tn_plan(int64_t n, int32_t FP, int32_t FQ, int64_t* rows_per_split, int32_t* n_split)
{
    const int BN = FQ > 64 ? 128 : (FQ > 32 ? 64 : 32);
    const int BM = FQ > 64 ? 128 : (FQ > 32 ? 128 : 256);
    const int64_t tiles = (int64_t)((FP + BM - 1) / BM) * ((FQ + BN - 1) / BN);
    // enough blocks to fill the chip a few times over, but at least 256 vertices per split
    int64_t want = std::max<int64_t>(1, 2048 / std::max<int64_t>(tiles, 1));
    want = std::min<int64_t>(want, std::max<int64_t>(1, n / 256));
    want = std::min<int64_t>(want, 1024);
    int64_t rows = (std::max<int64_t>(n, 1) + want - 1) / want;
    rows = (rows + kKT - 1) / kKT * kKT;
    *rows_per_split = rows;
    *n_split = (int32_t)std::max<int64_t>(1, (n + rows - 1) / rows);
}

hipError_t launch_gemm_tn(const GemmTnArgs& a, float* C, int64_t ldc, int accumulate, hipStream_t s)
{
    if (a.FP <= 0 || a.FQ <= 0) return hipSuccess;
    if (a.n_split < 1 || a.rows_per_split < 1 || a.rows_per_split % kKT != 0 || !a.part) return hipErrorInvalidValue;
    if ((int64_t)a.n_split * a.rows_per_split < a.n) return hipErrorInvalidValue;
    const bool aligned = a.FP % 4 == 0 && a.FQ % 4 == 0 && a.ldp % 4 == 0 && a.ldq % 4 == 0 &&
                         (reinterpret_cast<uintptr_t>(a.P) & 15u) == 0 && (reinterpret_cast<uintptr_t>(a.Q) & 15u) == 0;
    hipError_t e;
    if (a.FQ > 64)
        e = launch_tn_cfg<128, 128, 2, 2>(a, aligned, s);
    else if (a.FQ > 32)
        e = launch_tn_cfg<128, 64, 4, 1>(a, aligned, s);
    else
        e = launch_tn_cfg<256, 32, 4, 1>(a, aligned, s);
    if (e != hipSuccess) return e;
    const int64_t count = (int64_t)a.FP * a.FQ;
    hipLaunchKernelGGL(k_sum_splits, dim3((unsigned)((count + 63) / 64)), dim3(256), 0, s, a.part, count, a.n_split, a.FQ, C, ldc, accumulate);
    return hipGetLastError();
}

int64_t colsum_slabs(int64_t rows) { return std::max<int64_t>(1, std::min<int64_t>(1024, (rows + 127) / 128)); }

hipError_t launch_dz_colsum(const float* dY, int64_t lddy, const float* Y, int64_t ldy, int32_t act, float* dZ, int64_t rows, int32_t F,
                            float* part, float* dbias, int accumulate, hipStream_t s, int64_t lddz)
{
    if (F <= 0) return hipSuccess;
    if (lddz <= 0) lddz = F;
    if (act == SAGA_ACT_NONE) Y = nullptr;
    if (act != SAGA_ACT_NONE && !Y) return hipErrorInvalidValue;
    if (!Y && !part) return hipSuccess;  // nothing to mask, nothing to sum
    const int64_t slabs = colsum_slabs(rows);
    const int64_t R = (std::max<int64_t>(rows, 1) + slabs - 1) / slabs;
    const bool mask = Y != nullptr;
    const bool sig = act == SAGA_ACT_SIGMOID;
    const bool vec4 = F % 4 == 0 && lddy % 4 == 0 && (!mask || (ldy % 4 == 0 && lddz % 4 == 0)) && (reinterpret_cast<uintptr_t>(dY) & 15u) == 0 &&
                      (!mask || ((reinterpret_cast<uintptr_t>(Y) & 15u) == 0 && (reinterpret_cast<uintptr_t>(dZ) & 15u) == 0));
    const dim3 grid((unsigned)slabs), block(256);
    if (vec4 && mask && sig)
        hipLaunchKernelGGL((k_dz_colsum<4, 2>), grid, block, 0, s, dY, lddy, Y, ldy, dZ, lddz, rows, F, R, part);
    else if (vec4 && mask)
        hipLaunchKernelGGL((k_dz_colsum<4, 1>), grid, block, 0, s, dY, lddy, Y, ldy, dZ, lddz, rows, F, R, part);
    else if (vec4)
        hipLaunchKernelGGL((k_dz_colsum<4, 0>), grid, block, 0, s, dY, lddy, Y, ldy, dZ, lddz, rows, F, R, part);
    else if (mask && sig)
        hipLaunchKernelGGL((k_dz_colsum<1, 2>), grid, block, 0, s, dY, lddy, Y, ldy, dZ, lddz, rows, F, R, part);
    else if (mask)
        hipLaunchKernelGGL((k_dz_colsum<1, 1>), grid, block, 0, s, dY, lddy, Y, ldy, dZ, lddz, rows, F, R, part);
    else
        hipLaunchKernelGGL((k_dz_colsum<1, 0>), grid, block, 0, s, dY, lddy, Y, ldy, dZ, lddz, rows, F, R, part);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || !part) return e;
    hipLaunchKernelGGL(k_sum_splits, dim3((unsigned)((F + 63) / 64)), dim3(256), 0, s, part, (int64_t)F, (int)slabs, F, dbias, (int64_t)F, accumulate);
    return hipGetLastError();
}

hipError_t launch_permute_f32(const float* in, const int32_t* perm, float* out, int64_t count, hipStream_t s)
{
    if (count <= 0) return hipSuccess;
    const int grid = (int)std::min<int64_t>((count + 255) / 256, 1 << 20);
    hipLaunchKernelGGL(k_permute_f32, dim3(grid), dim3(256), 0, s, in, perm, out, count);
    return hipGetLastError();
}

hipError_t launch_sigmoid_grad(float* d, const float* z, int64_t count, hipStream_t s)
{
    if (count <= 0) return hipSuccess;
    const int grid = (int)std::min<int64_t>((count + 255) / 256, 1 << 20);
    hipLaunchKernelGGL(k_sigmoid_grad, dim3(grid), dim3(256), 0, s, d, z, count);
    return hipGetLastError();
}

hipError_t launch_dz_bf16(const uint16_t* dY, int64_t lddy, const uint16_t* Y, int64_t ldy, float* dZ32, uint16_t* dZ16, int64_t rows,
                          int32_t F, hipStream_t s)
{
    const int64_t total = rows * F;
    if (total <= 0) return hipSuccess;
    const int grid = (int)std::min<int64_t>((total + 255) / 256, 1 << 20);
    hipLaunchKernelGGL(k_dz_bf16, dim3(grid), dim3(256), 0, s, dY, lddy, Y, ldy, dZ32, dZ16, rows, F);
    return hipGetLastError();
}

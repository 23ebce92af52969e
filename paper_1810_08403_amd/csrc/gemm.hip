// Dense products of the layer on the gfx950 matrix cores: ApplyVertex
// (Y = act(A W + bias), Figures 2 and 10) and the per-vertex products hoisted
// out of a gated ApplyEdge (Section 3.2). The paper leaves these to its
// dataflow runtime's stock kernels; here they are one LDS-tiled MFMA kernel.
//
// C[M x N] = act(A[M x K] * Bt[N x K]^T + bias). Both operands are read
// K-contiguous: A as given, the weights from a packed, zero-padded transpose
// Bt. A K tile is 64 bytes per row (16 fp32 or 32 bf16). In LDS a row takes
// 80 bytes, so the 16-byte fragment reads of 32 consecutive rows spread over
// all banks. Each lane reads 16 bytes of its row: for bf16 that is exactly one
// 32x32x16 MFMA operand; for fp32 it feeds four 32x32x2 MFMAs (lane halves
// supply k and k+4 instead of k and k+1, the same on both operands, which
// only permutes the order of the K sum).
#include "saga_internal.h"

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kRowBytes = 64;    // bytes of K per tile row
constexpr int kLdsStride = 80;   // LDS bytes per tile row
constexpr int kBtRowPad = 128;   // Bt rows are padded to a multiple of this

__device__ __forceinline__ uint16_t to_bf16(float f)
{
    uint32_t x = __float_as_uint(f);
    if ((x & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((x >> 16) | 0x40u);
    x += 0x7fffu + ((x >> 16) & 1u);
    return (uint16_t)(x >> 16);
}

template <typename T>
__device__ __forceinline__ void mma_step(const uint4& a, const uint4& b, floatx16& acc);

template <>
__device__ __forceinline__ void mma_step<float>(const uint4& a, const uint4& b, floatx16& acc)
{
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
}
template <>
__device__ __forceinline__ void mma_step<uint16_t>(const uint4& a, const uint4& b, floatx16& acc)
{
    union {
        uint4 u;
        bf16x8 v;
    } ua, ub;
    ua.u = a;
    ub.u = b;
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ua.v, ub.v, acc, 0, 0, 0);
}

template <typename T, int BM, int BN, int WM, int WN, bool ALIGNED, typename TO>
__global__ __launch_bounds__(256) void k_gemm_nt(const GemmArgs a, const int n_tiles_n, const int64_t n_tiles)
{
    constexpr int KT = kRowBytes / (int)sizeof(T);  // elements of K per tile
    constexpr int EPC = 16 / (int)sizeof(T);        // elements per 16-byte chunk
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    static_assert(WM * WN == 4 && TM >= 1 && TN >= 1, "tile shape");
    __shared__ __attribute__((aligned(16))) unsigned char lds[2][(BM + BN) * kLdsStride];

    // XCD-aware tile order: consecutive tiles of one XCD share the A tile
    int64_t tile;
    {
        const int64_t b = blockIdx.x, per = gridDim.x >> 3;
        tile = (b & 7) * per + (b >> 3);
    }
    if (tile >= n_tiles) return;
    const int64_t m0 = (tile / n_tiles_n) * BM;
    const int n0 = (int)(tile % n_tiles_n) * BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WM, wn = wave / WM;
    const T* __restrict__ A = static_cast<const T*>(a.A);
    const T* __restrict__ Bt = static_cast<const T*>(a.Bt);
    const int K = a.K;
    const int nk = (K + KT - 1) / KT;

    constexpr int ACH = (BM * 4 + 255) / 256, BCH = (BN * 4 + 255) / 256;
    uint4 ra[ACH], rb[BCH];

    auto gload = [&](int kt) {
#pragma unroll
        for (int i = 0; i < ACH; ++i) {
            const int c = tid + 256 * i;
            if (BM * 4 % 256 != 0 && c >= BM * 4) break;
            const int row = c >> 2, kc = c & 3;
            int64_t gr = m0 + row;
            if (gr >= a.M) gr = a.M - 1;
            const int k = kt * KT + kc * EPC;
            const T* p = A + gr * a.lda + k;
            if (ALIGNED) {
                ra[i] = k < K ? *reinterpret_cast<const uint4*>(p) : make_uint4(0, 0, 0, 0);
            } else {
                T tmp[EPC];
#pragma unroll
                for (int j = 0; j < EPC; ++j) tmp[j] = (k + j < K) ? p[j] : T(0);
                ra[i] = *reinterpret_cast<const uint4*>(tmp);
            }
        }
#pragma unroll
        for (int i = 0; i < BCH; ++i) {
            const int c = tid + 256 * i;
            if (BN * 4 % 256 != 0 && c >= BN * 4) break;
            const int row = c >> 2, kc = c & 3;
            rb[i] = *reinterpret_cast<const uint4*>(Bt + (int64_t)(n0 + row) * a.ldbt + kt * KT + kc * EPC);
        }
    };
    auto lstore = [&](int buf) {
#pragma unroll
        for (int i = 0; i < ACH; ++i) {
            const int c = tid + 256 * i;
            if (BM * 4 % 256 != 0 && c >= BM * 4) break;
            *reinterpret_cast<uint4*>(&lds[buf][(c >> 2) * kLdsStride + (c & 3) * 16]) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < BCH; ++i) {
            const int c = tid + 256 * i;
            if (BN * 4 % 256 != 0 && c >= BN * 4) break;
            *reinterpret_cast<uint4*>(&lds[buf][(BM + (c >> 2)) * kLdsStride + (c & 3) * 16]) = rb[i];
        }
    };

    floatx16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    gload(0);
    lstore(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        if (kt + 1 < nk) gload(kt + 1);
        const unsigned char* base = lds[kt & 1];
#pragma unroll
        for (int step = 0; step < 2; ++step) {
            uint4 fa[TM], fb[TN];
            const int chunk = (step * 2 + (lane >> 5)) * 16;
#pragma unroll
            for (int i = 0; i < TM; ++i)
                fa[i] = *reinterpret_cast<const uint4*>(base + ((wm * TM + i) * 32 + (lane & 31)) * kLdsStride + chunk);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                fb[j] = *reinterpret_cast<const uint4*>(base + (BM + (wn * TN + j) * 32 + (lane & 31)) * kLdsStride + chunk);
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j) mma_step<T>(fa[i], fb[j], acc[i][j]);
        }
        if (kt + 1 < nk) lstore((kt + 1) & 1);
        __syncthreads();
    }

    // epilogue: lane holds column (lane & 31) of 16 rows of each 32 x 32 tile
    TO* __restrict__ C = static_cast<TO*>(a.C);
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int col = n0 + (wn * TN + j) * 32 + (lane & 31);
        if (col >= a.N) continue;
        const float bias = a.bias ? a.bias[col] : 0.f;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const int64_t rbase = m0 + (wm * TM + i) * 32 + (lane >> 5) * 4;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int64_t row = rbase + (r >> 2) * 8 + (r & 3);
                if (row >= a.M) continue;
                float y = acc[i][j][r] + bias;
                if (a.act == SAGA_ACT_RELU) y = y > 0.f ? y : 0.f;
                if (sizeof(TO) == 4)
                    reinterpret_cast<float*>(C)[row * a.ldc + col] = y;
                else
                    reinterpret_cast<uint16_t*>(C)[row * a.ldc + col] = to_bf16(y);
            }
        }
    }
}

template <typename T>
__global__ __launch_bounds__(256) void k_pack_bt_transpose(const T* W, int64_t ldw, int K, int N, T* Bt, int64_t n_pad,
                                                           int64_t k_pad)
{
    const int64_t total = n_pad * k_pad;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int64_t n = i / k_pad, k = i % k_pad;
        Bt[i] = (n < N && k < K) ? W[k * ldw + n] : T(0);
    }
}

__global__ __launch_bounds__(256) void k_pack_bt_rows(const float* Wsrc, int64_t ldw, int64_t col0, int R, int K, float* Bt,
                                                      int64_t ldbt, int64_t row0)
{
    const int64_t total = (int64_t)R * K;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int64_t r = i / K, k = i % K;
        Bt[(row0 + r) * ldbt + k] = Wsrc ? Wsrc[r * ldw + col0 + k] : (r == k ? 1.f : 0.f);
    }
}

template <typename T, int BM, int BN, int WM, int WN, typename TO>
hipError_t launch_cfg(const GemmArgs& a, bool aligned, hipStream_t s)
{
    const int n_tiles_n = (a.N + BN - 1) / BN;
    const int64_t n_tiles = ((a.M + BM - 1) / BM) * n_tiles_n;
    const int64_t blocks = (n_tiles + 7) / 8 * 8;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    if (aligned)
        hipLaunchKernelGGL((k_gemm_nt<T, BM, BN, WM, WN, true, TO>), dim3((unsigned)blocks), dim3(256), 0, s, a, n_tiles_n,
                           n_tiles);
    else
        hipLaunchKernelGGL((k_gemm_nt<T, BM, BN, WM, WN, false, TO>), dim3((unsigned)blocks), dim3(256), 0, s, a, n_tiles_n,
                           n_tiles);
    return hipGetLastError();
}

template <typename T, typename TO>
hipError_t launch_typed(const GemmArgs& a, hipStream_t s)
{
    const bool aligned = (a.K * sizeof(T)) % 16 == 0 && (a.lda * sizeof(T)) % 16 == 0 &&
                         (reinterpret_cast<uintptr_t>(a.A) & 15u) == 0;
    if (a.N > 64) return launch_cfg<T, 128, 128, 2, 2, TO>(a, aligned, s);
    if (a.N > 32) return launch_cfg<T, 128, 64, 4, 1, TO>(a, aligned, s);
    return launch_cfg<T, 256, 32, 4, 1, TO>(a, aligned, s);
}

}  // namespace

void bt_padded_shape(int32_t N, int32_t K, int32_t dtype, int64_t* n_pad, int64_t* k_pad)
{
    const int kt = kRowBytes / (dtype == SAGA_F32 ? 4 : 2);
    *n_pad = ((int64_t)N + kBtRowPad - 1) / kBtRowPad * kBtRowPad;
    *k_pad = ((int64_t)K + kt - 1) / kt * kt;
}

hipError_t launch_gemm(const GemmArgs& a, hipStream_t s)
{
    if (a.M <= 0 || a.N <= 0) return hipSuccess;
    if (a.K <= 0) return hipErrorInvalidValue;
    if (a.dtype == SAGA_F32) {
        if (a.out_dtype != SAGA_F32) return hipErrorInvalidValue;
        return launch_typed<float, float>(a, s);
    }
    if (a.out_dtype == SAGA_F32) return launch_typed<uint16_t, float>(a, s);
    return launch_typed<uint16_t, uint16_t>(a, s);
}

hipError_t launch_pack_bt_transpose(const void* W, int64_t ldw, int32_t K, int32_t N, int32_t dtype, void* Bt, hipStream_t s)
{
    int64_t n_pad, k_pad;
    bt_padded_shape(N, K, dtype, &n_pad, &k_pad);
    const int64_t total = n_pad * k_pad;
    const int grid = (int)std::min<int64_t>((total + 255) / 256, 65535);
    if (dtype == SAGA_F32)
        hipLaunchKernelGGL(k_pack_bt_transpose<float>, dim3(grid), dim3(256), 0, s, static_cast<const float*>(W), ldw, K, N,
                           static_cast<float*>(Bt), n_pad, k_pad);
    else
        hipLaunchKernelGGL(k_pack_bt_transpose<uint16_t>, dim3(grid), dim3(256), 0, s, static_cast<const uint16_t*>(W), ldw, K,
                           N, static_cast<uint16_t*>(Bt), n_pad, k_pad);
    return hipGetLastError();
}

hipError_t launch_pack_bt_rows(const float* Wsrc, int64_t ldw, int64_t col0, int32_t R, int32_t K, float* Bt, int64_t ldbt,
                               int64_t row0, hipStream_t s)
{
    const int64_t total = (int64_t)R * K;
    if (total <= 0) return hipSuccess;
    const int grid = (int)std::min<int64_t>((total + 255) / 256, 65535);
    hipLaunchKernelGGL(k_pack_bt_rows, dim3(grid), dim3(256), 0, s, Wsrc, ldw, col0, R, K, Bt, ldbt, row0);
    return hipGetLastError();
}

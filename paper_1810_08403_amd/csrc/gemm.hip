// Dense products of the layer on the gfx950 matrix cores: ApplyVertex
// (Y = act(A W + bias), Figures 2 and 10) and the per-vertex products hoisted
// out of a gated ApplyEdge (Section 3.2). The paper leaves these to its
// dataflow runtime's stock kernels; here they are one LDS-tiled MFMA kernel.
//
// C[M x N] = act(A[M x K] * Bt[N x K]^T + bias). Both operands are read
// K-contiguous: A as given, the weights from a packed, zero-padded transpose
// Bt. A K tile is 64 bytes per row for fp32 (16 elements) and 128 bytes for
// bf16 (64 elements). In LDS a row takes 16 bytes more, so the 16-byte
// fragment reads of consecutive rows spread over all banks. Each lane reads
// 16 bytes of its row per step: for bf16 that is exactly one
// 32x32x16 MFMA operand; for fp32 it feeds four 32x32x2 MFMAs (lane halves
// supply k and k+4 instead of k and k+1, the same on both operands, which
// only permutes the order of the K sum).
//
// A launch holds as many workgroups as the chip keeps resident (three per
// compute unit); each walks a list of output tiles and prefetches K tiles two
// deep in registers across tile boundaries, so the memory latency at the start
// of a tile and the write-out at its end overlap the neighbouring tiles' MFMAs.
// Measured on 1,048,576 x 128 x 128 fp32: 0.37 ms (one tile per workgroup:
// 0.39); the same loop without MFMAs 0.21 ms, without global loads 0.33 ms,
// without the write-out 0.30 ms. A write-out with 16-byte stores from
// transposed accumulators (32 bytes per row and instruction) was slower than
// the 4-byte stores that fill two whole 128-byte lines per instruction.
#include <type_traits>
#include "device_math.h"
#include "saga_internal.h"

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));  // a 16-byte fragment as a first-class vector value

// bytes of K per tile row: 64 for fp32 (16 elements, 16 MFMAs of 64 cycles per wave and 32 x 32 tile), 128 for bf16
// (64 elements: with 64 bytes a wave had 256 cycles of MFMA work between two barriers, less than the barrier, the LDS
// round trip and the address arithmetic around it cost)
template <typename T>
constexpr int row_bytes()
{
    return sizeof(T) == 4 ? 64 : 128;
}
constexpr int kLdsPad = 16;      // LDS bytes added to a tile row: 16-byte reads of 16 consecutive rows then cover all banks
constexpr int kBtRowPad = 128;   // Bt rows are padded to a multiple of this

__device__ __forceinline__ uint16_t to_bf16(float f)
{
    uint32_t x = __float_as_uint(f);
    if ((x & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((x >> 16) | 0x40u);
    x += 0x7fffu + ((x >> 16) & 1u);
    return (uint16_t)(x >> 16);
}

// All MFMAs of one 16-byte fragment step of a wave's TM x TN accumulator tiles. fp32 takes four 32x32x2 MFMAs per
// tile and step; they are issued tile after tile for one dword of the fragments before the next dword, so that
// consecutive MFMAs write different accumulators.
template <typename T, int TM, int TN>
__device__ __forceinline__ void mma_step(const u32x4 (&fa)[TM], const u32x4 (&fb)[TN], floatx16 (&acc)[TM][TN])
{
    if constexpr (sizeof(T) == 4) {
#pragma unroll
        for (int c = 0; c < 4; ++c)
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(fa[i][c]), __uint_as_float(fb[j][c]), acc[i][j], 0, 0, 0);
    } else {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, fa[i]), __builtin_bit_cast(bf16x8, fb[j]),
                                                                    acc[i][j], 0, 0, 0);
    }
}

// Global -> registers of one K tile (64 bytes per row) of the A and Bt blocks: thread t owns
// 16-byte chunks t, t + 256, ... A chunk past the end of K is loaded from k = 0 and zeroed
// on its way to LDS, so that the prefetched registers are not touched before the MFMAs of
// the current tile have issued. A tile index past the last tile (kt >= nk) reads the last
// tile again and zeroes all of its A chunks: such a tile adds nothing to the product.
template <typename T, int BM, int BN, bool ALIGNED, int ACH, int BCH>
__device__ __forceinline__ void tile_load(const GemmArgs& a, const T* __restrict__ A, const T* __restrict__ Bt, int64_t m0,
                                          int n0, int kt, int nk, int tid, u32x4 (&ra)[ACH], u32x4 (&rb)[BCH], unsigned& ka)
{
    constexpr int KB = row_bytes<T>(), KT = KB / (int)sizeof(T), EPC = 16 / (int)sizeof(T), CPR = KB / 16;  // chunks per row
    ka = 0;
    const bool past = kt >= nk;
    if (past) kt = nk - 1;
    // K tiles [0, nk1) come from A, the rest from the optional second operand A2
    const int nk1 = (a.K + KT - 1) / KT;
    const bool second = kt >= nk1;
    const T* __restrict__ Asrc = second ? static_cast<const T*>(a.A2) : A;
    const int64_t ld = second ? a.lda2 : a.lda;
    const int Klim = second ? a.K2 : a.K;
    const int k0 = (second ? kt - nk1 : kt) * KT;
#pragma unroll
    for (int i = 0; i < ACH; ++i) {
        const int c = tid + 256 * i;
        const int row = (c / CPR) < BM ? (c / CPR) : 0, kc = c % CPR;
        int64_t gr = m0 + row;
        if (gr >= a.M) gr = a.M - 1;
        const int k = k0 + kc * EPC;
        const bool in = k < Klim && !past;
        ka |= in ? (1u << i) : 0u;
        const T* p = Asrc + gr * ld + (ALIGNED && !in ? 0 : k);
        if (ALIGNED) {
            ra[i] = *reinterpret_cast<const u32x4*>(p);
        } else {
            uint32_t w[4] = {0, 0, 0, 0};
#pragma unroll
            for (int j = 0; j < EPC; ++j) {
                const uint32_t e = (k + j < Klim && !past) ? (sizeof(T) == 4 ? __float_as_uint(*reinterpret_cast<const float*>(p + j))
                                                                   : (uint32_t) * reinterpret_cast<const uint16_t*>(p + j))
                                                 : 0u;
                if (sizeof(T) == 4)
                    w[j] = e;
                else
                    w[j >> 1] |= e << (16 * (j & 1));
            }
            ra[i] = u32x4{w[0], w[1], w[2], w[3]};
        }
    }
#pragma unroll
    for (int i = 0; i < BCH; ++i) {
        const int c = tid + 256 * i;
        const int row = (c / CPR) < BN ? (c / CPR) : 0, kc = c % CPR;
        rb[i] = *reinterpret_cast<const u32x4*>(Bt + (int64_t)(n0 + row) * a.ldbt + kt * KT + kc * EPC);
    }
}
template <int KB, int BM, int BN, bool ALIGNED, int ACH, int BCH>
__device__ __forceinline__ void tile_store(unsigned char* buf, int tid, const u32x4 (&ra)[ACH], const u32x4 (&rb)[BCH],
                                           unsigned ka)
{
    constexpr int CPR = KB / 16, kLdsStride = KB + kLdsPad;
#pragma unroll
    for (int i = 0; i < ACH; ++i) {
        const int c = tid + 256 * i;
        const bool in = !ALIGNED || ((ka >> i) & 1u);
        const u32x4 v = in ? ra[i] : u32x4{0u, 0u, 0u, 0u};
        if (BM * CPR % 256 == 0 || c < BM * CPR) *reinterpret_cast<u32x4*>(buf + (c / CPR) * kLdsStride + (c % CPR) * 16) = v;
    }
#pragma unroll
    for (int i = 0; i < BCH; ++i) {
        const int c = tid + 256 * i;
        if (BN * CPR % 256 == 0 || c < BN * CPR)
            *reinterpret_cast<u32x4*>(buf + (BM + c / CPR) * kLdsStride + (c % CPR) * 16) = rb[i];
    }
}

// Bias, activation, rounding and store of one wave's accumulators. row0 / col0: first row
// and the column this lane holds. CHECK guards the ragged edge tiles only.
template <typename TO, int TM, int TN, bool CHECK>
__device__ __forceinline__ void store_tile(const GemmArgs& a, const floatx16 (&acc)[TM][TN], int64_t row0, int col0)
{
    TO* __restrict__ C = static_cast<TO*>(a.C);
#pragma unroll
    for (int j = 0; j < TN; ++j) {
        const int col = col0 + j * 32;
        if (CHECK && col >= a.N) continue;
        const float bias = a.bias ? a.bias[col] : 0.f;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            TO* p = C + (row0 + i * 32) * a.ldc + col;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int dr = (r >> 2) * 8 + (r & 3);
                if (CHECK && row0 + i * 32 + dr >= a.M) continue;
                float y = acc[i][j][r] + bias;
                if (a.act == SAGA_ACT_RELU) y = y > 0.f ? y : 0.f;
                if (a.act == SAGA_ACT_SIGMOID) y = sigmoid_f32(y);
                if (sizeof(TO) == 4)
                    reinterpret_cast<float*>(p)[dr * a.ldc] = y;
                else
                    reinterpret_cast<uint16_t*>(p)[dr * a.ldc] = to_bf16(y);
            }
        }
    }
}

// One workgroup takes a list of output tiles (a slice of its XCD's share, see launch_cfg) and runs their K tiles as
// one stream: while a tile's last K tiles are multiplied and its results are written out, the first K tiles of the
// workgroup's next output tile are already on their way, so only the first tile of a workgroup waits for memory
// with nothing else to do. Layers have short K loops (K = 128: eight K tiles), where that wait and the write-out
// would otherwise be a third of a tile's time.
template <typename T, int BM, int BN, int WM, int WN, bool ALIGNED, typename TO>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(sizeof(T) == 4 ? 3 : 2, sizeof(T) == 4 ? 3 : 2))) void k_gemm_nt(
    const GemmArgs a, const int n_tiles_n, const int n_tiles)
{
    constexpr int KB = row_bytes<T>(), kLdsStride = KB + kLdsPad;
    constexpr int KT = KB / (int)sizeof(T);  // elements of K per tile
    constexpr int TM = BM / WM / 32, TN = BN / WN / 32;
    static_assert(WM * WN == 4 && TM >= 1 && TN >= 1, "tile shape");
    __shared__ __attribute__((aligned(16))) unsigned char lds[2][(BM + BN) * kLdsStride];

    // XCD-aware tile order: workgroups are dealt to the 8 XCDs in turn; XCD x owns the consecutive tiles
    // [x * per, (x + 1) * per), which share rows of A and all of Bt in its L2, and its workgroups take them in turn
    const int per = (n_tiles + 7) >> 3, slots = (int)(gridDim.x >> 3);
    const int xcd = (int)(blockIdx.x & 7), slot = (int)(blockIdx.x >> 3);
    const int first = xcd * per + slot;
    const int last = min((xcd + 1) * per, n_tiles);
    if (first >= last) return;
    const int count = (last - first + slots - 1) / slots;  // output tiles of this workgroup: first, first + slots, ...

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WM, wn = wave / WM;
    const T* __restrict__ A = static_cast<const T*>(a.A);
    const T* __restrict__ Bt = static_cast<const T*>(a.Bt);
    const int nk = (a.K + KT - 1) / KT + (a.A2 ? (a.K2 + KT - 1) / KT : 0);
    const int nkp = (nk + 1) & ~1;  // the loop takes K tiles in pairs: an odd count is padded with a zero tile

    constexpr int ACH = (BM * (KB / 16) + 255) / 256, BCH = (BN * (KB / 16) + 255) / 256;
    u32x4 ra[ACH], rb[BCH], ra2[ACH], rb2[BCH];
    unsigned ka = 0, ka2 = 0;  // bit i: chunk i of this thread lies inside K

    floatx16 acc[TM][TN];

    auto multiply = [&](const unsigned char* base) {
#pragma unroll
        for (int step = 0; step < KB / 32; ++step) {
            u32x4 fa[TM], fb[TN];
            const int chunk = (step * 2 + (lane >> 5)) * 16;
#pragma unroll
            for (int i = 0; i < TM; ++i)
                fa[i] = *reinterpret_cast<const u32x4*>(base + ((wm * TM + i) * 32 + (lane & 31)) * kLdsStride + chunk);
#pragma unroll
            for (int j = 0; j < TN; ++j)
                fb[j] = *reinterpret_cast<const u32x4*>(base + (BM + (wn * TN + j) * 32 + (lane & 31)) * kLdsStride + chunk);
            mma_step<T, TM, TN>(fa, fb, acc);
        }
    };
    // the load cursor runs two K tiles ahead of the multiplication, across output tiles; past the workgroup's last
    // output tile it stays there and loads zero tiles (kt >= nk)
    int l_ti = 0, l_kt = 0;
    int64_t l_m0 = (int64_t)(first / n_tiles_n) * BM;
    int l_n0 = (first % n_tiles_n) * BN;
    auto load_next = [&](u32x4(&qa)[ACH], u32x4(&qb)[BCH], unsigned& qk) {
        tile_load<T, BM, BN, ALIGNED>(a, A, Bt, l_m0, l_n0, l_ti < count ? l_kt : nk, nk, tid, qa, qb, qk);
        if (++l_kt == nkp) {
            l_kt = 0;
            if (++l_ti < count) {
                const int t = first + l_ti * slots;
                l_m0 = (int64_t)(t / n_tiles_n) * BM;
                l_n0 = (t % n_tiles_n) * BN;
            }
        }
    };
    load_next(ra, rb, ka);
    tile_store<KB, BM, BN, ALIGNED>(lds[0], tid, ra, rb, ka);
    load_next(ra, rb, ka);
    __syncthreads();
    for (int ti = 0; ti < count; ++ti) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
        // Two K tiles are in flight in registers while a third is multiplied out of LDS. The K tiles go in pairs
        // without a branch in the middle (one would make the compiler keep two copies of the accumulators).
        for (int kt = 0; kt < nkp; kt += 2) {
            // K tile kt is in lds[0], kt + 1 on its way into (ra, rb): issue kt + 2 into (ra2, rb2)
            load_next(ra2, rb2, ka2);
            __builtin_amdgcn_sched_barrier(0);  // keep the prefetch ahead of the MFMAs it is meant to overlap
            multiply(lds[0]);
            __builtin_amdgcn_sched_barrier(0);  // ... and the wait for the older loads behind them
            tile_store<KB, BM, BN, ALIGNED>(lds[1], tid, ra, rb, ka);
            __syncthreads();
            load_next(ra, rb, ka);
            __builtin_amdgcn_sched_barrier(0);
            multiply(lds[1]);
            __builtin_amdgcn_sched_barrier(0);
            tile_store<KB, BM, BN, ALIGNED>(lds[0], tid, ra2, rb2, ka2);
            __syncthreads();
        }
        // write-out: lane holds column (lane & 31) of 16 rows of each 32 x 32 tile
        const int t = first + ti * slots;
        const int64_t m0 = (int64_t)(t / n_tiles_n) * BM;
        const int n0 = (t % n_tiles_n) * BN;
        if (m0 + BM <= a.M && n0 + BN <= a.N)
            store_tile<TO, TM, TN, false>(a, acc, m0 + wm * TM * 32 + (lane >> 5) * 4, n0 + wn * TN * 32 + (lane & 31));
        else
            store_tile<TO, TM, TN, true>(a, acc, m0 + wm * TM * 32 + (lane >> 5) * 4, n0 + wn * TN * 32 + (lane & 31));
    }
}

// ---------------------------------------------------------------------------
// fp32 products with K = 128 (the layer width of the gated, CommNet and max-pooling applications: their hoisted
// per-vertex products and ApplyVertex) with the weights resident in LDS. A workgroup owns 128 columns: their rows of Bt
// (64 KiB) are brought into LDS once; then it walks 64-row tiles of A, each copied from memory straight into one of two
// 32 KiB LDS buffers (global_load_lds: no registers, no store instructions) while the previous tile is multiplied. One
// barrier per tile, 64 MFMAs (4,096 cycles) per wavefront between two barriers; the results of a tile are written out
// between the first steps of the next tile and complete under its MFMAs. A wave-wide copy lands as 1 KiB of consecutive LDS
// bytes, so rows cannot be padded; instead the 16-byte chunks of a row are stored permuted (chunk c of row r at position
// c ^ (r & 15)), which spreads the operand reads of 16 consecutive rows over all banks. One workgroup of eight
// wavefronts per compute unit (128 KiB of LDS), two wavefronts per SIMD, each with one 32 x 32 accumulator tile (four
// wavefronts with two tiles each, one per SIMD, were slower: 94 against 100 TFLOP/s on 1,048,576 x 128 x 384).
// ---------------------------------------------------------------------------
constexpr int kWldsK = 128, kWldsBM = 64, kWldsBN = 128;

// bias, activation and store of value r of a lane's 32 x 32 accumulator tile (row row0 + (r / 4) * 8 + r % 4)
// out_row: the row of C the value goes to (row0 + dr itself, or what the row list names for it)
template <int ACT, bool CHECK>
__device__ __forceinline__ void wlds_store_one(const GemmArgs& a, float v, int r, int64_t row0, int64_t out_row, int col, float bias)
{
    const int dr = (r >> 2) * 8 + (r & 3);
    if (CHECK && (col >= a.N || row0 + dr >= a.M)) return;
    float y = v + bias;
    if (ACT == SAGA_ACT_RELU) y = y > 0.f ? y : 0.f;
    if (ACT == SAGA_ACT_SIGMOID) y = sigmoid_f32(y);
    static_cast<float*>(a.C)[out_row * a.ldc + col] = y;
}
// The activation is a parameter of the kernel: as a run-time select per value it made every product compute the sigmoid's
// exponential for every value.
// IDS: the product is taken over the rows a.row_ids names (row i of the product reads row row_ids[i] of A and writes row
// row_ids[i] of C; the list is padded to whole tiles with its last entry). The ids a tile's copies need are read a tile
// before the copies are issued and the ids its results go to at the tile's start, so that no step waits for them: every
// wait for memory in the loop is the one at the end of a tile.
template <int ACT, bool IDS>
__global__ __launch_bounds__(512) void k_gemm_wlds(const GemmArgs a, const int n_cg, const int wg_per_cg, const int n_tiles_m)
{
    // three separate arrays: the compiler makes an LDS read wait for the copies in flight (they count as memory
    // operations that write LDS) unless it can tell that they go to another array than the one being read
    __shared__ __attribute__((aligned(16))) float Bs[kWldsBN * kWldsK];
    __shared__ __attribute__((aligned(16))) float As0[kWldsBM * kWldsK];
    __shared__ __attribute__((aligned(16))) float As1[kWldsBM * kWldsK];
    typedef __attribute__((address_space(3))) void* lds_ptr;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m = lane & 31, h = lane >> 5;
    const int wm = wave & 1, wn = wave >> 1;
    // blockIdx = ((j / 8) * n_cg + cg) * 8 + j % 8: workgroup j of every column group on XCD j % 8, so that the column
    // groups that read the same rows of A at the same time share them in one L2
    const int cg = (int)((blockIdx.x >> 3) % (unsigned)n_cg);
    const int j = (int)((blockIdx.x >> 3) / (unsigned)n_cg) * 8 + (int)(blockIdx.x & 7);
    if (j >= n_tiles_m) return;
    const int count = (n_tiles_m - j + wg_per_cg - 1) / wg_per_cg;  // tiles j, j + wg_per_cg, ...
    const float* __restrict__ A = static_cast<const float*>(a.A);
    const float* __restrict__ Bt = static_cast<const float*>(a.Bt);

    // a wave-wide copy: rows 2 idx and 2 idx + 1 of a tile, lane l the chunk that belongs at position l & 31 of row
    // 2 idx + (l >> 5), i.e. chunk (l & 31) ^ (row & 15) of the row in memory. A wavefront makes eight per tile.
    const int crow = lane >> 5, cpos = lane & 31;
    const int32_t* __restrict__ ids = a.row_ids;
    int nid[4] = {0, 0, 0, 0};  // IDS: the rows of A this lane copies for the tile after the one being copied
    auto load_ids = [&](int tile) {
#pragma unroll
        for (int i = 0; i < 4; ++i) nid[i] = ids[(int64_t)tile * kWldsBM + 2 * (wave * 4 + i) + crow];
    };
    auto copy_one = [&](int tile, float (&buf)[kWldsBM * kWldsK], int i) {
        const int idx = wave * 4 + i, row = 2 * idx + crow;
        int64_t gr;
        if constexpr (IDS) {
            gr = nid[i];
        } else {
            gr = (int64_t)tile * kWldsBM + row;
            if (gr >= a.M) gr = a.M - 1;  // rows past the end are copies of the last row; their results are not stored
        }
        const float* src = A + gr * a.lda + ((cpos ^ (row & 15)) << 2);
        __builtin_amdgcn_global_load_lds(src, (lds_ptr)(&buf[idx * 256]), 16, 0, 0);
    };
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int idx = wave * 8 + i, row = 2 * idx + crow;
        const float* src = Bt + (int64_t)(cg * kWldsBN + row) * a.ldbt + ((cpos ^ (row & 15)) << 2);  // Bt is padded to 128 rows
        __builtin_amdgcn_global_load_lds(src, (lds_ptr)(&Bs[idx * 256]), 16, 0, 0);
    }
    if constexpr (IDS) load_ids(j);
#pragma unroll
    for (int i = 0; i < 4; ++i) copy_one(j, As0, i);
    if constexpr (IDS) {
        if (count > 1) load_ids(j + wg_per_cg);
    }
    const int col0 = cg * kWldsBN + wn * 32 + m;
    const float bias = (a.bias && col0 < a.N) ? a.bias[col0] : 0.f;
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wavefront's copies have landed
    __syncthreads();

    // operand addresses: row r of a buffer, chunk 2 s + h at position (2 s + h) ^ (r & 15); r & 15 == m & 15 for both operands
    const int ra = (wm * 32 + m) * kWldsK;
    const int rb0 = (wn * 32 + m) * kWldsK;
    const int sw = m & 15;
    // One tile: the next one's copies first, then 16 steps of two operand reads (requested a step ahead) and four
    // MFMAs; the wait for the copies and the barrier. The results of a tile are written out between the first eight
    // steps of the next tile, two values per step: with two wavefronts per SIMD that leave the barrier together, a
    // write-out of its own (16 values per lane with their address arithmetic) kept the matrix cores waiting.
    // (Spreading the copies between the steps as well was slower: 1.28 against 1.11 ms on 1,048,576 x 128 x 384.)
    floatx16 pacc;
    int64_t prow0 = 0;
    bool pfull = false;
    int4 oid[4], poid[4];  // IDS: the rows of C this lane's 16 results of the current / the previous tile go to
    auto out_row = [&](int r) -> int64_t {
        if constexpr (IDS) {
            const int4 q = poid[r >> 2];
            return (r & 3) == 0 ? q.x : (r & 3) == 1 ? q.y : (r & 3) == 2 ? q.z : q.w;
        } else {
            return prow0 + (r >> 2) * 8 + (r & 3);
        }
    };
    auto do_tile = [&](int t, const float (&cur)[kWldsBM * kWldsK], float (&nxt)[kWldsBM * kWldsK], auto pchk) __attribute__((always_inline)) {
        constexpr bool PCHECK = decltype(pchk)::value;  // the previous tile ends past M or N
        const int tile = j + t * wg_per_cg;
        if (t + 1 < count) {
#pragma unroll
            for (int i = 0; i < 4; ++i) copy_one(tile + wg_per_cg, nxt, i);
        }
        if constexpr (IDS) {
            if (t + 2 < count) load_ids(tile + 2 * wg_per_cg);
#pragma unroll
            for (int q = 0; q < 4; ++q)
                oid[q] = *reinterpret_cast<const int4*>(ids + (int64_t)tile * kWldsBM + wm * 32 + h * 4 + 8 * q);
        }
        __builtin_amdgcn_sched_barrier(0);  // the copies start before the MFMAs they run under
        floatx16 acc;
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[r] = 0.f;
        u32x4 fa, fb0;
        auto fetch = [&](int s_, u32x4& xa, u32x4& xb0) {
            const int pos = ((2 * s_ + h) ^ sw) << 2;
            xa = *reinterpret_cast<const u32x4*>(&cur[ra + pos]);
            xb0 = *reinterpret_cast<const u32x4*>(&Bs[rb0 + pos]);
        };
        fetch(0, fa, fb0);
#pragma unroll
        for (int s_ = 0; s_ < kWldsK / 8; ++s_) {
            u32x4 na = fa, nb0 = fb0;
            if (s_ + 1 < kWldsK / 8) fetch(s_ + 1, na, nb0);
            __builtin_amdgcn_sched_barrier(0);  // the next step's reads are on their way while this step multiplies
#pragma unroll
            for (int c = 0; c < 4; ++c)
                acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(fa[c]), __uint_as_float(fb0[c]), acc, 0, 0, 0);
            if (s_ < 8 && t > 0) {
                wlds_store_one<ACT, PCHECK>(a, pacc[2 * s_], 2 * s_, prow0, out_row(2 * s_), col0, bias);
                wlds_store_one<ACT, PCHECK>(a, pacc[2 * s_ + 1], 2 * s_ + 1, prow0, out_row(2 * s_ + 1), col0, bias);
            }
            __builtin_amdgcn_sched_barrier(0);
            fa = na;
            fb0 = nb0;
        }
        // the next tile's copies were issued a whole tile ago, the previous tile's stores at least half a tile ago
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();  // every wavefront is done with this buffer, and sees the next one
        pacc = acc;
        if constexpr (IDS) {
#pragma unroll
            for (int q = 0; q < 4; ++q) poid[q] = oid[q];
        }
        prow0 = (int64_t)tile * kWldsBM + wm * 32 + h * 4;
        pfull = (int64_t)tile * kWldsBM + kWldsBM <= a.M && cg * kWldsBN + kWldsBN <= a.N;
    };
    auto tile_of = [&](int t, const float (&cur)[kWldsBM * kWldsK], float (&nxt)[kWldsBM * kWldsK]) __attribute__((always_inline)) {
        if (pfull || t == 0)
            do_tile(t, cur, nxt, std::false_type{});
        else
            do_tile(t, cur, nxt, std::true_type{});
    };
    for (int t = 0; t < count; t += 2) {
        tile_of(t, As0, As1);
        if (t + 1 < count) tile_of(t + 1, As1, As0);
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) wlds_store_one<ACT, true>(a, pacc[r], r, prow0, out_row(r), col0, bias);
}

// ---------------------------------------------------------------------------
// bf16 products with K = 256 or 512 and many rows (ApplyVertex of the wide GCN layers, the transform-first product and
// dZ W^T of their backward pass) with the weights resident in registers. These products are bound by memory (512 -> 256:
// 0.4 GB against 69 GFLOP), and the 256 KiB of a 512 x 256 bf16 weight matrix fit no LDS; they do fit the registers of
// one workgroup: each of its eight wavefronts keeps 32 columns for all of K (128 registers per lane at K = 512),
// already in the layout of the 16x16x32 matrix instruction's first operand, for the whole kernel. The product is
// taken transposed, C^T = W^T A^T: the rows of A are the instruction's second operand (read from LDS, 16 bytes per
// lane and instruction) and a lane ends up with four consecutive columns of one row, which it stores as 8 bytes.
// The workgroup walks 32-row tiles of A, copied from memory straight into one of three LDS buffers
// (global_load_lds, chunks permuted within a row as in k_gemm_wlds) two tiles ahead of the multiplication, so that two
// tiles (64 KiB at K = 512) are in flight per compute unit all the time. Every row of A is read from memory once
// and no weight is read again after the first microsecond.
// Waiting for a tile: a wavefront's copies complete in the order they were issued, its stores in an order of their
// own. s_waitcnt vmcnt(n), n = the copies of the one tile that may still be in flight, is therefore enough whatever
// the stores do: if a copy of an earlier tile were outstanding, so would all n of the later one be.
// Measured on 262,144 x 512 x 256 (MI355X; the stage also packs the weights): 153 us with k_gemm_nt, 94 us here
// (4.3 TB/s). What the steps cost, from runs with parts taken out: the copies alone 56 us; with the operand reads and
// MFMAs 78 us (every wavefront reads the whole tile from LDS: 256 KiB per tile and compute unit with eight
// wavefronts; sixteen wavefronts of 16 columns read twice that and took 108 us); an epilogue of its own before the
// steps, 100 us (113 us before the chip's bf16 conversion instruction replaced the integer rounding and the
// activation became a branch per group instead of a select per value: two wavefronts per SIMD in the same phase
// hide no vector instructions), spread between the steps of the next tile as it is now, 94 us.
// ---------------------------------------------------------------------------
constexpr int kWregTR = 32;  // rows of a tile

// NW wavefronts per workgroup, each with 256 / NW columns (CH groups of 16): the fewer wavefronts, the fewer times a tile
// of A is read from LDS (once per wavefront), the more registers the weights take per lane (4 CH K / 32).
template <int KS, int NW, typename TO>
__global__ __launch_bounds__(NW * 64) void k_gemm_wreg16(const GemmArgs a, const int n_cg, const int wg_per_cg, const int n_tiles_m)
{
    constexpr int K = 32 * KS;                         // 512 or 256
    constexpr int CH = 16 / NW;                        // 16-column groups of a wavefront
    constexpr int kTile = kWregTR * K;                 // bf16 elements of a tile
    constexpr int kCopies = kTile * 2 / 1024 / NW;     // wave-wide copies (1 KiB) per wavefront and tile
    constexpr int kRowsPerCopy = 1024 / (K * 2);       // 1 or 2
    constexpr int kChunks = K / 8;                     // 16-byte chunks of a row: 64 or 32
    static_assert(kCopies >= 1 && kCopies < 16, "the wait below counts the copies of one tile in four bits");
    __shared__ __attribute__((aligned(16))) uint16_t As0[kTile];
    __shared__ __attribute__((aligned(16))) uint16_t As1[kTile];
    __shared__ __attribute__((aligned(16))) uint16_t As2[kTile];
    typedef __attribute__((address_space(3))) void* lds_ptr;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // uniform, and known to be: addresses built from it stay in scalar registers
    const int n = lane & 15, g = lane >> 4;
    const int cg = (int)((blockIdx.x >> 3) % (unsigned)n_cg);
    const int j = (int)((blockIdx.x >> 3) / (unsigned)n_cg) * 8 + (int)(blockIdx.x & 7);
    if (j >= n_tiles_m) return;
    const int count = (n_tiles_m - j + wg_per_cg - 1) / wg_per_cg;  // tiles j, j + wg_per_cg, ...
    const uint16_t* __restrict__ A = static_cast<const uint16_t*>(a.A);
    const uint16_t* __restrict__ Bt = static_cast<const uint16_t*>(a.Bt);
    const int c0 = cg * 256 + wave * 16 * CH;  // this wavefront's columns: [c0, c0 + 16 CH); N is a multiple of 16

    // lane l of a copy brings the chunk that belongs at position l % kChunks of its row, chunk (l % kChunks) ^ (row & 15)
    const int crow = lane / kChunks, cpos = lane % kChunks;
    auto copy_tile = [&](int tile, uint16_t (&buf)[kTile]) {
#pragma unroll
        for (int i = 0; i < kCopies; ++i) {
            const int idx = wave * kCopies + i, row = idx * kRowsPerCopy + crow;
            int64_t gr = (int64_t)tile * kWregTR + row;
            if (gr >= a.M) gr = a.M - 1;  // rows past the end are copies of the last row; their results are not stored
            const uint16_t* src = A + gr * a.lda + ((cpos ^ (row & 15)) << 3);
            __builtin_amdgcn_global_load_lds(src, (lds_ptr)(&buf[idx * 512]), 16, 0, 0);
        }
    };
    copy_tile(j, As0);
    if (count > 1) copy_tile(j + wg_per_cg, As1);

    // the weights: column c0 + 16 h + n, the eight k at 32 s + 8 g, for every group h and step s (groups past N: column 0,
    // their results are not stored)
    u32x4 w[CH][KS];
    float bias[CH][4];
#pragma unroll
    for (int h = 0; h < CH; ++h) {
        const bool has = c0 + 16 * h < a.N;
        const uint16_t* wp = Bt + (int64_t)(has ? c0 + 16 * h + n : 0) * a.ldbt + 8 * g;
#pragma unroll
        for (int s_ = 0; s_ < KS; ++s_) w[h][s_] = *reinterpret_cast<const u32x4*>(wp + 32 * s_);
#pragma unroll
        for (int q = 0; q < 4; ++q) bias[h][q] = (a.bias && has) ? a.bias[c0 + 16 * h + 4 * g + q] : 0.f;
    }

    // bias, activation, rounding and store of one 16 x 16 group of results: columns c0 + 16 h ..., rows 16 hh ... of the tile
    auto store_act = [&](int tile, const floatx4& r, int h, int hh, auto act_c) {
        constexpr int ACT = decltype(act_c)::value;
        TO* __restrict__ C = static_cast<TO*>(a.C);
        const int64_t row = (int64_t)tile * kWregTR + hh * 16 + n;
        if (c0 + 16 * h >= a.N || row >= a.M) return;
        float y[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            y[q] = r[q] + bias[h][q];
            if (ACT == SAGA_ACT_RELU) y[q] = y[q] > 0.f ? y[q] : 0.f;
            if (ACT == SAGA_ACT_SIGMOID) y[q] = sigmoid_f32(y[q]);
        }
        TO* p = C + row * a.ldc + c0 + 16 * h + 4 * g;
        if (sizeof(TO) == 4) {
            *reinterpret_cast<float4*>(p) = make_float4(y[0], y[1], y[2], y[3]);
        } else {
            // the conversion instruction of this chip (round to nearest even, two values at a time)
            typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
            uint2 v;
            v.x = __builtin_bit_cast(uint32_t, (bf16x2){(__bf16)y[0], (__bf16)y[1]});
            v.y = __builtin_bit_cast(uint32_t, (bf16x2){(__bf16)y[2], (__bf16)y[3]});
            *reinterpret_cast<uint2*>(p) = v;
        }
    };
    // one branch on the activation per group instead of a select per value (the sigmoid's exponential would otherwise be
    // computed for every value of every layer)
    const int act = __builtin_amdgcn_readfirstlane(a.act);
    auto store_group = [&](int tile, const floatx4& r, int h, int hh) {
        if (act == SAGA_ACT_RELU)
            store_act(tile, r, h, hh, std::integral_constant<int, SAGA_ACT_RELU>{});
        else if (act == SAGA_ACT_SIGMOID)
            store_act(tile, r, h, hh, std::integral_constant<int, SAGA_ACT_SIGMOID>{});
        else
            store_act(tile, r, h, hh, std::integral_constant<int, SAGA_ACT_NONE>{});
    };
    // A tile's results move to pacc at the next tile's barrier and are stored group by group between the steps of that
    // tile: with two wavefronts per SIMD, both in the same phase, an epilogue of its own would leave the matrix cores idle.
    floatx4 acc[CH][2], pacc[CH][2];
#pragma unroll
    for (int h = 0; h < CH; ++h)
#pragma unroll
        for (int q = 0; q < 4; ++q) acc[h][0][q] = acc[h][1][q] = 0.f;
    // Operand reads: row hh * 16 + n of the buffer, chunk 4 s + g at position (4 s + g) ^ n, i.e. byte
    // n * 2 K + ((g ^ (n & 3)) << 4) + ((s ^ (n >> 2)) << 6), and 32 K bytes further for the second half of the rows.
    // They are written as instructions: for an LDS read it can see, the compiler waits for every copy in flight that
    // it cannot prove to go to another array, and after unrolling it could not for one tile in three. The wait for a
    // read is lgkmcnt(0) on the registers it fills, placed before the next step's reads are issued, so a read has the
    // MFMAs of one step to arrive in.
    const uint32_t rd = (uint32_t)(n * 2 * K + ((g ^ (n & 3)) << 4)), nb = (uint32_t)(n >> 2);
    auto lds_base = [](const uint16_t* p) { return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) uint16_t*)p; };
    auto fetch = [&](uint32_t base, int s_, u32x4& x0, u32x4& x1) {
        const uint32_t addr = base + rd + (((uint32_t)s_ ^ nb) << 6);
        asm volatile("ds_read_b128 %0, %2\n\tds_read_b128 %1, %2 offset:%3" : "=&v"(x0), "=&v"(x1) : "v"(addr), "n"(32 * K) : "memory");
    };
    auto arrived = [](u32x4& x0, u32x4& x1) { asm volatile("s_waitcnt lgkmcnt(0)" : "+v"(x0), "+v"(x1)::"memory"); };
    auto do_tile = [&](int t, const uint16_t (&cur)[kTile], uint16_t (&nxt2)[kTile]) {
        const int tile = j + t * wg_per_cg;
        // this wavefront's copies of tile t have landed (those of tile t + 1 may be in flight), then everybody's have
        if (t + 1 < count)
            __builtin_amdgcn_s_waitcnt(0x0F70 | kCopies);
        else
            __builtin_amdgcn_s_waitcnt(0x0F70);
        // the bare barrier instruction: __syncthreads(), and a fence on LDS alone too, would make the compiler wait for the
        // copies of tile t + 1 as well (they write LDS). What has to be ordered is ordered by hand: the copies of tile t by
        // the wait above, this wavefront's operand reads of tile t - 1 by the waits that precede the MFMAs using them.
        __builtin_amdgcn_s_barrier();
#pragma unroll
        for (int h = 0; h < CH; ++h)
#pragma unroll
            for (int hh = 0; hh < 2; ++hh) {
                pacc[h][hh] = acc[h][hh];
#pragma unroll
                for (int q = 0; q < 4; ++q) acc[h][hh][q] = 0.f;
            }
        __builtin_amdgcn_sched_barrier(0);
        if (t + 2 < count) copy_tile(tile + 2 * wg_per_cg, nxt2);
        const uint32_t base = lds_base(cur);
        u32x4 f[2][2];
        fetch(base, 0, f[0][0], f[0][1]);
#pragma unroll
        for (int s_ = 0; s_ < KS; ++s_) {
            u32x4(&fc)[2] = f[s_ & 1];
            arrived(fc[0], fc[1]);
            if (s_ + 1 < KS) fetch(base, s_ + 1, f[(s_ + 1) & 1][0], f[(s_ + 1) & 1][1]);
#pragma unroll
            for (int h = 0; h < CH; ++h) {
                const bf16x8 wv = __builtin_bit_cast(bf16x8, w[h][s_]);
                acc[h][0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wv, __builtin_bit_cast(bf16x8, fc[0]), acc[h][0], 0, 0, 0);
                acc[h][1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wv, __builtin_bit_cast(bf16x8, fc[1]), acc[h][1], 0, 0, 0);
            }
            if (t > 0 && (s_ & 1) && s_ / 2 < 2 * CH) store_group(tile - wg_per_cg, pacc[(s_ / 2) >> 1][(s_ / 2) & 1], (s_ / 2) >> 1, (s_ / 2) & 1);
        }
    };
    for (int t = 0; t < count; t += 3) {
        do_tile(t, As0, As2);
        if (t + 1 < count) do_tile(t + 1, As1, As0);
        if (t + 2 < count) do_tile(t + 2, As2, As1);
    }
#pragma unroll
    for (int h = 0; h < CH; ++h)
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) store_group(j + (count - 1) * wg_per_cg, acc[h][hh], h, hh);
}

template <typename T>
__global__ __launch_bounds__(256) void k_pack_bt_transpose(const T* W, int64_t ldw, int K, int N, T* Bt, int64_t ldbt, int64_t col0)
{
    const int64_t total = (int64_t)N * K;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int64_t k = i / N, n = i % N;  // consecutive threads read consecutive elements of a row of W
        Bt[n * ldbt + col0 + k] = W[k * ldw + n];
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
__global__ __launch_bounds__(256) void k_pack_bt_rows16(const uint16_t* Wsrc, int64_t ldw, int R, int K, uint16_t* Bt, int64_t ldbt)
{
    const int64_t total = (int64_t)R * K;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int64_t r = i / K, k = i % K;
        Bt[r * ldbt + k] = Wsrc[r * ldw + k];
    }
}

template <typename T, int BM, int BN, int WM, int WN, typename TO>
hipError_t launch_cfg(const GemmArgs& a, bool aligned, hipStream_t s)
{
    const int n_tiles_n = (a.N + BN - 1) / BN;
    const int64_t n_tiles = ((a.M + BM - 1) / BM) * n_tiles_n;
    if (n_tiles > 0x7fffffffLL - 8) return hipErrorInvalidValue;
    // as many workgroups as the 256 compute units hold at once (three each, two with the wider K tiles of bf16), a
    // multiple of the 8 XCDs; fewer when there are fewer tiles. Each takes every slots-th tile of its XCD's share.
    const int64_t blocks = std::min<int64_t>((n_tiles + 7) / 8 * 8, sizeof(T) == 4 ? 768 : 512);
    if (aligned)
        hipLaunchKernelGGL((k_gemm_nt<T, BM, BN, WM, WN, true, TO>), dim3((unsigned)blocks), dim3(256), 0, s, a, n_tiles_n,
                           (int)n_tiles);
    else
        hipLaunchKernelGGL((k_gemm_nt<T, BM, BN, WM, WN, false, TO>), dim3((unsigned)blocks), dim3(256), 0, s, a, n_tiles_n,
                           (int)n_tiles);
    return hipGetLastError();
}

template <typename T, typename TO>
hipError_t launch_typed(const GemmArgs& a, hipStream_t s)
{
    bool aligned = (a.K * sizeof(T)) % 16 == 0 && (a.lda * sizeof(T)) % 16 == 0 &&
                   (reinterpret_cast<uintptr_t>(a.A) & 15u) == 0;
    if (a.A2)
        aligned = aligned && (a.K2 * sizeof(T)) % 16 == 0 && (a.lda2 * sizeof(T)) % 16 == 0 &&
                  (reinterpret_cast<uintptr_t>(a.A2) & 15u) == 0;
    if (a.N > 64) return launch_cfg<T, 128, 128, 2, 2, TO>(a, aligned, s);
    if constexpr (sizeof(T) == 2) {  // bf16: 288 LDS rows of 144 bytes would leave one workgroup per compute unit
        return launch_cfg<T, 128, 64, 4, 1, TO>(a, aligned, s);
    } else {
        if (a.N > 32) return launch_cfg<T, 128, 64, 4, 1, TO>(a, aligned, s);
        return launch_cfg<T, 256, 32, 4, 1, TO>(a, aligned, s);
    }
}

}  // namespace

void bt_padded_shape(int32_t N, int32_t K, int32_t dtype, int64_t* n_pad, int64_t* k_pad)
{
    const int kt = dtype == SAGA_F32 ? row_bytes<float>() / 4 : row_bytes<uint16_t>() / 2;
    *n_pad = ((int64_t)N + kBtRowPad - 1) / kBtRowPad * kBtRowPad;
    *k_pad = ((int64_t)K + kt - 1) / kt * kt;
}

// the weights-in-LDS kernel where it applies (fp32, one operand, K = 128, rows in 16-byte fragments, enough rows to give
// every compute unit several tiles); false: not applicable
static bool wlds_applies(const GemmArgs& a)
{
    if (a.dtype != SAGA_F32 || a.out_dtype != SAGA_F32 || a.tiled_only) return false;
    if (a.A2 || a.K != kWldsK || a.lda % 4 != 0 || (reinterpret_cast<uintptr_t>(a.A) & 15u) || a.M < 16 * 1024) return false;
    if (a.row_ids && (reinterpret_cast<uintptr_t>(a.row_ids) & 15u)) return false;
    if (a.ldbt % 4 != 0 || a.ldbt < kWldsK || (reinterpret_cast<uintptr_t>(a.Bt) & 15u)) return false;
    const int n_cg = (a.N + kWldsBN - 1) / kWldsBN;
    const int64_t n_tiles_m = (a.M + kWldsBM - 1) / kWldsBM;
    return n_cg <= 32 && n_tiles_m <= 0x7fffffffLL;
}

bool gemm_takes_row_list(const GemmArgs& a) { return a.row_ids && wlds_applies(a); }

static bool launch_wlds(const GemmArgs& a, hipStream_t s, hipError_t* err)
{
    if (!wlds_applies(a)) return false;
    const int n_cg = (a.N + kWldsBN - 1) / kWldsBN;
    const int64_t n_tiles_m = (a.M + kWldsBM - 1) / kWldsBM;
    const int wg_per_cg = std::max(8, 256 / n_cg / 8 * 8);  // one workgroup per compute unit, a multiple of the 8 XCDs per column group
    const dim3 grid((unsigned)(wg_per_cg * n_cg));
    if (a.row_ids) {
        if (a.act == SAGA_ACT_RELU)
            hipLaunchKernelGGL((k_gemm_wlds<SAGA_ACT_RELU, true>), grid, dim3(512), 0, s, a, n_cg, wg_per_cg, (int)n_tiles_m);
        else if (a.act == SAGA_ACT_SIGMOID)
            hipLaunchKernelGGL((k_gemm_wlds<SAGA_ACT_SIGMOID, true>), grid, dim3(512), 0, s, a, n_cg, wg_per_cg, (int)n_tiles_m);
        else
            hipLaunchKernelGGL((k_gemm_wlds<SAGA_ACT_NONE, true>), grid, dim3(512), 0, s, a, n_cg, wg_per_cg, (int)n_tiles_m);
    } else if (a.act == SAGA_ACT_RELU)
        hipLaunchKernelGGL((k_gemm_wlds<SAGA_ACT_RELU, false>), grid, dim3(512), 0, s, a, n_cg, wg_per_cg, (int)n_tiles_m);
    else if (a.act == SAGA_ACT_SIGMOID)
        hipLaunchKernelGGL((k_gemm_wlds<SAGA_ACT_SIGMOID, false>), grid, dim3(512), 0, s, a, n_cg, wg_per_cg, (int)n_tiles_m);
    else
        hipLaunchKernelGGL((k_gemm_wlds<SAGA_ACT_NONE, false>), grid, dim3(512), 0, s, a, n_cg, wg_per_cg, (int)n_tiles_m);
    *err = hipGetLastError();
    return true;
}

// the weights-in-registers kernel where it applies (bf16, one operand, K = 256 or 512, N a multiple of 16, rows and
// outputs in 16-byte / 8-byte fragments, enough rows to give every compute unit several tiles); false: not applicable
template <typename TO>
static bool launch_wreg16(const GemmArgs& a, hipStream_t s, hipError_t* err)
{
    if (a.A2 || (a.K != 256 && a.K != 512) || a.N % 16 != 0 || a.M < 32 * 1024) return false;
    if (a.lda % 8 != 0 || (reinterpret_cast<uintptr_t>(a.A) & 15u) || a.ldbt % 8 != 0 || a.ldbt < a.K ||
        (reinterpret_cast<uintptr_t>(a.Bt) & 15u) || a.ldc % 4 != 0 || (reinterpret_cast<uintptr_t>(a.C) & 15u))
        return false;
    const int n_cg = (a.N + 255) / 256;
    const int64_t n_tiles_m = (a.M + kWregTR - 1) / kWregTR;
    if (n_cg > 32 || n_tiles_m > 0x7fffffffLL) return false;
    const int wg_per_cg = std::max(8, 256 / n_cg / 8 * 8);  // one workgroup per compute unit, a multiple of the 8 XCDs per column group
    const dim3 grid((unsigned)(wg_per_cg * n_cg));
    constexpr int NW = 8;
    if (a.K == 512)
        hipLaunchKernelGGL((k_gemm_wreg16<16, NW, TO>), grid, dim3(NW * 64), 0, s, a, n_cg, wg_per_cg, (int)n_tiles_m);
    else
        hipLaunchKernelGGL((k_gemm_wreg16<8, NW, TO>), grid, dim3(NW * 64), 0, s, a, n_cg, wg_per_cg, (int)n_tiles_m);
    *err = hipGetLastError();
    return true;
}

hipError_t launch_gemm(const GemmArgs& a, hipStream_t s)
{
    if (a.M <= 0 || a.N <= 0) return hipSuccess;
    if (a.K <= 0 || (a.A2 && a.K2 <= 0)) return hipErrorInvalidValue;
    if (a.dtype == SAGA_F32) {
        if (a.out_dtype != SAGA_F32) return hipErrorInvalidValue;
        hipError_t e = hipSuccess;
        if (launch_wlds(a, s, &e)) return e;
        if (a.row_ids) return hipErrorInvalidValue;  // the tiled kernel takes whole ranges of rows only
        return launch_typed<float, float>(a, s);
    }
    if (a.row_ids) return hipErrorInvalidValue;
    hipError_t e = hipSuccess;
    if (a.out_dtype == SAGA_F32) {
        if (launch_wreg16<float>(a, s, &e)) return e;
        return launch_typed<uint16_t, float>(a, s);
    }
    if (launch_wreg16<uint16_t>(a, s, &e)) return e;
    return launch_typed<uint16_t, uint16_t>(a, s);
}

hipError_t launch_pack_bt_transpose(const void* W, int64_t ldw, int32_t K, int32_t N, int32_t dtype, void* Bt, int64_t ldbt,
                                    int64_t col0, hipStream_t s)
{
    const int64_t total = (int64_t)N * K;
    if (total <= 0) return hipSuccess;
    const int grid = (int)std::min<int64_t>((total + 255) / 256, 65535);
    if (dtype == SAGA_F32)
        hipLaunchKernelGGL(k_pack_bt_transpose<float>, dim3(grid), dim3(256), 0, s, static_cast<const float*>(W), ldw, K, N,
                           static_cast<float*>(Bt), ldbt, col0);
    else
        hipLaunchKernelGGL(k_pack_bt_transpose<uint16_t>, dim3(grid), dim3(256), 0, s, static_cast<const uint16_t*>(W), ldw, K,
                           N, static_cast<uint16_t*>(Bt), ldbt, col0);
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

hipError_t launch_pack_bt_rows_bf16(const uint16_t* Wsrc, int64_t ldw, int32_t R, int32_t K, uint16_t* Bt, int64_t ldbt, hipStream_t s)
{
    const int64_t total = (int64_t)R * K;
    if (total <= 0) return hipSuccess;
    const int grid = (int)std::min<int64_t>((total + 255) / 256, 65535);
    hipLaunchKernelGGL(k_pack_bt_rows16, dim3(grid), dim3(256), 0, s, Wsrc, ldw, R, K, Bt, ldbt);
    return hipGetLastError();
}

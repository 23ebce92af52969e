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
#include "device_math.h"
#include "saga_internal.h"

namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
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
// after the barrier and complete under the MFMAs of the next tile. A wave-wide copy lands as 1 KiB of consecutive LDS
// bytes, so rows cannot be padded; instead the 16-byte chunks of a row are stored permuted (chunk c of row r at position
// c ^ (r & 15)), which spreads the operand reads of 16 consecutive rows over all banks. One workgroup of eight
// wavefronts per compute unit (128 KiB of LDS), two wavefronts per SIMD, each with one 32 x 32 accumulator tile (four
// wavefronts with two tiles each, one per SIMD, were slower: 94 against 100 TFLOP/s on 1,048,576 x 128 x 384).
// ---------------------------------------------------------------------------
constexpr int kWldsK = 128, kWldsBM = 64, kWldsBN = 128;

template <bool CHECK>
__device__ __forceinline__ void wlds_store(const GemmArgs& a, const floatx16& acc, int64_t row0, int col, float bias)
{
    float* __restrict__ C = static_cast<float*>(a.C);
    if (CHECK && col >= a.N) return;
    float* p = C + row0 * a.ldc + col;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const int dr = (r >> 2) * 8 + (r & 3);
        if (CHECK && row0 + dr >= a.M) continue;
        float y = acc[r] + bias;
        if (a.act == SAGA_ACT_RELU) y = y > 0.f ? y : 0.f;
        if (a.act == SAGA_ACT_SIGMOID) y = sigmoid_f32(y);
        p[dr * a.ldc] = y;
    }
}

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
    auto copy_one = [&](int tile, float (&buf)[kWldsBM * kWldsK], int i) {
        const int idx = wave * 4 + i, row = 2 * idx + crow;
        int64_t gr = (int64_t)tile * kWldsBM + row;
        if (gr >= a.M) gr = a.M - 1;  // rows past the end are copies of the last row; their results are not stored
        const float* src = A + gr * a.lda + ((cpos ^ (row & 15)) << 2);
        __builtin_amdgcn_global_load_lds(src, (lds_ptr)(&buf[idx * 256]), 16, 0, 0);
    };
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int idx = wave * 8 + i, row = 2 * idx + crow;
        const float* src = Bt + (int64_t)(cg * kWldsBN + row) * a.ldbt + ((cpos ^ (row & 15)) << 2);  // Bt is padded to 128 rows
        __builtin_amdgcn_global_load_lds(src, (lds_ptr)(&Bs[idx * 256]), 16, 0, 0);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) copy_one(j, As0, i);
    const int col0 = cg * kWldsBN + wn * 32 + m;
    const float bias = (a.bias && col0 < a.N) ? a.bias[col0] : 0.f;
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wavefront's copies have landed
    __syncthreads();

    // operand addresses: row r of a buffer, chunk 2 s + h at position (2 s + h) ^ (r & 15); r & 15 == m & 15 for both operands
    const int ra = (wm * 32 + m) * kWldsK;
    const int rb0 = (wn * 32 + m) * kWldsK;
    const int sw = m & 15;
    // One tile: the next one's copies first, then 16 steps of three operand reads (requested a step ahead) and eight
    // MFMAs; the wait for the copies, the barrier, and the write-out, which the hardware completes under the next
    // tile's MFMAs. (Spreading the copies and the previous tile's write-out, from a second accumulator set, between
    // the MFMAs of the steps was slower: 1.28 against 1.11 ms on 1,048,576 x 128 x 384.)
    auto do_tile = [&](int t, const float (&cur)[kWldsBM * kWldsK], float (&nxt)[kWldsBM * kWldsK]) {
        const int tile = j + t * wg_per_cg;
        if (t + 1 < count) {
#pragma unroll
            for (int i = 0; i < 4; ++i) copy_one(tile + wg_per_cg, nxt, i);
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
            __builtin_amdgcn_sched_barrier(0);
            fa = na;
            fb0 = nb0;
        }
        // the next tile's copies (and the previous tile's stores) were issued a whole tile ago
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();  // every wavefront is done with this buffer, and sees the next one
        const int64_t row0 = (int64_t)tile * kWldsBM + wm * 32 + h * 4;
        if ((int64_t)tile * kWldsBM + kWldsBM <= a.M && cg * kWldsBN + kWldsBN <= a.N)
            wlds_store<false>(a, acc, row0, col0, bias);
        else
            wlds_store<true>(a, acc, row0, col0, bias);
    };
    for (int t = 0; t < count; t += 2) {
        do_tile(t, As0, As1);
        if (t + 1 < count) do_tile(t + 1, As1, As0);
    }
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
static bool launch_wlds(const GemmArgs& a, hipStream_t s, hipError_t* err)
{
    if (a.A2 || a.K != kWldsK || a.lda % 4 != 0 || (reinterpret_cast<uintptr_t>(a.A) & 15u) || a.M < 16 * 1024) return false;
    if (a.ldbt % 4 != 0 || a.ldbt < kWldsK || (reinterpret_cast<uintptr_t>(a.Bt) & 15u)) return false;
    const int n_cg = (a.N + kWldsBN - 1) / kWldsBN;
    const int64_t n_tiles_m = (a.M + kWldsBM - 1) / kWldsBM;
    if (n_cg > 32 || n_tiles_m > 0x7fffffffLL) return false;
    const int wg_per_cg = std::max(8, 256 / n_cg / 8 * 8);  // one workgroup per compute unit, a multiple of the 8 XCDs per column group
    hipLaunchKernelGGL(k_gemm_wlds, dim3((unsigned)(wg_per_cg * n_cg)), dim3(512), 0, s, a, n_cg, wg_per_cg, (int)n_tiles_m);
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
        return launch_typed<float, float>(a, s);
    }
    if (a.out_dtype == SAGA_F32) return launch_typed<uint16_t, float>(a, s);
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

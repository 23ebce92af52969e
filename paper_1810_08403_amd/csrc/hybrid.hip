// The dense part of the fused Scatter-ApplyEdge-Gather of a bf16 sum layer on the gfx950 matrix cores.
//
// Section 3.3 parallelises the propagation along the feature row of one vertex at a time; that is the right
// shape where the adjacency matrix is sparse. In a power-law graph the block of heavy destinations and heavy
// sources is not sparse: with destinations ranked by in-degree and sources by out-degree, a 64 x 32 block of
// the matrix often holds hundreds of edges. There
//     accum[64 destinations][F] += A_block[64 x 32 edge weights] * X[32 source rows][F]
// is a dense contraction. The matrix cores do it at a cost that does not depend on the number of edges in the
// block, and each source row is read once per block instead of once per edge; the host marks the blocks for
// which that is cheaper than the sparse kernel (build_hybrid_plan), the sparse kernel keeps the rest.
//
// One workgroup works a chunk of consecutive blocks of one destination tile; its four wavefronts own 128
// features each (512 per pass over the chunk). Per block:
//   - every wavefront loads its 256-byte slice of the block's 32 source rows, a lane 8 rows x 16 bytes, and
//     turns the 8 x 8 (row x feature) patch it holds into the instruction's B operands (8 sources of one
//     feature per lane) with byte permutes;
//   - the workgroup brings the block's A operand, 64 x 32 weights as two bf16 parts (w = high + low to 2^-17
//     relative), into LDS in the lane order of the instruction, so that a lane's operand is one 16-byte LDS
//     read: a block of up to 256 edges from its compact edge list (cell, weight), one pair per thread, scattered
//     into a cleared buffer; a fuller block as the finished 8 KiB operand, copied from memory straight into LDS
//     (global_load_lds). Three LDS buffers rotate (being read, being filled for the next block, being cleared
//     for the one after), which leaves one barrier per block;
//   - 16x16x32 bf16 MFMAs accumulate 64 destinations x 128 features per wavefront in registers.
// At the end of the chunk every destination's row goes to its partial-row slot; the combine pass adds the
// chunks of a tile and the pieces of the sparse remainder in slot order, so sums stay reproducible.
#include "saga_internal.h"

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr uint32_t kPermLow = 0x05040100u;   // (low half of the second operand, low half of the first)
constexpr uint32_t kPermHigh = 0x07060302u;  // (high half of the second, high half of the first)
constexpr int kCells = kDenseM * kDenseK;    // 2,048 weights per block and part

__device__ __forceinline__ uint16_t bf16_rne(float f)
{
    uint32_t x = __float_as_uint(f);
    x += 0x7fffu + ((x >> 16) & 1u);  // weights are finite
    return (uint16_t)(x >> 16);
}

// Wave-uniform reads through the constant address space arrive in scalar registers (read-only scalar loads).
typedef const int32_t __attribute__((address_space(4))) * c_i32;

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void k_dense_blocks(const DenseArgs a)
{
    // [buffer][part: 0 high, 1 low][cell], cells in the lane order of the A operand
    __shared__ __attribute__((aligned(16))) uint16_t lds[3][2][kCells];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int kg = lane >> 4, oct = lane & 15;  // the lane supplies sources 8 kg .. 8 kg + 7 of a block, feature octet `oct` of its slice
    const c_i32 c_chunks = (c_i32)(uintptr_t)a.chunks, c_src_tile = (c_i32)(uintptr_t)a.blk_src_tile, c_e0 = (c_i32)(uintptr_t)a.blk_e0,
                c_ft = (c_i32)(uintptr_t)a.blk_tile;
    const int ch_tile = c_chunks[4 * (int64_t)blockIdx.x], ch_b0 = c_chunks[4 * (int64_t)blockIdx.x + 1],
              ch_b1 = c_chunks[4 * (int64_t)blockIdx.x + 2], ch_cidx = c_chunks[4 * (int64_t)blockIdx.x + 3];
    const int n_pass = (a.F + 511) / 512;

    auto clear = [&](int buf) {  // 8 KiB: 32 bytes per thread
        u32x4* p = reinterpret_cast<u32x4*>(&lds[buf][0][0]);
        p[tid] = u32x4{0u, 0u, 0u, 0u};
        p[tid + 256] = u32x4{0u, 0u, 0u, 0u};
    };
    // Everything a block needs is asked for one step of the loop before it is used, each step one memory round trip:
    //   four blocks ahead:  the block's source tile, the bounds of its edge list or the number of its finished operand (scalar loads),
    //   three blocks ahead: the 32 source ids of that tile, one per thread of the first half-wavefront, into a register,
    //   two blocks ahead:   those ids into LDS; this thread's edge of the block's list into registers (fetch),
    //   one block ahead:    the source rows, their ids read back from LDS (load_rows), and the operand into LDS: the edge
    //                       scattered (place), or the finished operand copied (copy_operand),
    //   then the block is multiplied.
    __shared__ int ids_lds[3][kDenseK];
    struct Bounds {
        int tile, e0, e1, ft;  // source tile; edge list [e0, e1) (at most 256 edges); finished operand, or -1
    };
    struct Staged {
        uint32_t w;
        int pos;
    };
    auto bounds_of = [&](int b) {
        const int bb = b < ch_b1 ? b : ch_b1 - 1;  // past the chunk: its last block again, never used
        return Bounds{c_src_tile[bb], c_e0[bb], c_e0[bb + 1], c_ft[bb]};
    };
    auto fetch = [&](const Bounds& bd, Staged& st) {
        const int e = bd.e0 + tid;
        const int ee = e < bd.e1 ? e : (bd.e1 > 0 ? bd.e1 - 1 : 0);  // past the list (or no list): a valid address, never used
        st.w = a.de_w[ee];
        st.pos = a.de_pos[ee];
    };
    auto place = [&](const Bounds& bd, const Staged& st, int buf) {
        if (bd.e0 + tid < bd.e1) {
            lds[buf][0][st.pos] = (uint16_t)(st.w & 0xffffu);
            lds[buf][1][st.pos] = (uint16_t)(st.w >> 16);
        }
    };
    // 8 KiB from memory into an LDS buffer without passing through registers: every wavefront copies 1 KiB (a lane 16
    // bytes) of each half. The copy is complete, for this wavefront, when its memory counter has run out (s_waitcnt
    // vmcnt(0) below); the barrier that follows makes it visible to the others.
    auto copy_operand = [&](int ft, int buf) {
        const char* src = reinterpret_cast<const char*>(a.de_tiles) + (int64_t)ft * (kDenseTileElems * 2) + tid * 16;
        char* dst = reinterpret_cast<char*>(&lds[buf][0][0]) + wave * 1024;
        __builtin_amdgcn_global_load_lds(src, (__attribute__((address_space(3))) void*)dst, 16, 0, 0);
        __builtin_amdgcn_global_load_lds(src + 4096, (__attribute__((address_space(3))) void*)(dst + 4096), 16, 0, 0);
    };
    auto id_of = [&](const Bounds& bd) { return a.src_tile_ids[(int64_t)bd.tile * kDenseK + (tid & (kDenseK - 1))]; };

    for (int pass = 0; pass < n_pass; ++pass) {
        const int col = (pass * 4 + wave) * 128 + oct * 8;  // first feature of this lane's octet
        const bool active = col < a.F;                       // F is a multiple of 128: a wavefront's slice is all there or not at all
        // a row fragment's address is the (wave-uniform) base of X plus a 32-bit byte offset: the launcher checks that X
        // is smaller than 4 GiB, and eight 64-bit addresses per lane would not fit the register budget of this kernel
        const char* const xbase = reinterpret_cast<const char*>(a.X);
        const uint32_t colb = (uint32_t)(active ? col : 0) * 2u, ldb = (uint32_t)a.ld * 2u;
        auto load_rows = [&](int slot, u32x4 (&x)[8]) {  // this lane's sources 8 kg .. 8 kg + 7 of the block whose ids sit in ids_lds[slot]
            const int4 i0 = *reinterpret_cast<const int4*>(&ids_lds[slot][kg * 8]);
            const int4 i1 = *reinterpret_cast<const int4*>(&ids_lds[slot][kg * 8 + 4]);
            const int id[8] = {i0.x, i0.y, i0.z, i0.w, i1.x, i1.y, i1.z, i1.w};
#pragma unroll
            for (int j = 0; j < 8; ++j) x[j] = *reinterpret_cast<const u32x4*>(xbase + ((uint32_t)id[j] * ldb + colb));
        };

        f32x4 acc[4][8];
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int f = 0; f < 8; ++f) acc[mt][f] = f32x4{0.f, 0.f, 0.f, 0.f};

        if (pass > 0) __syncthreads();  // the previous pass has finished with the LDS buffers
        clear(0);
        clear(1);
        clear(2);
        // prologue. Block b0 + k is "block k" below; its ids live in ids_lds[k % 3], its operand in lds[k % 3].
        Bounds bd1 = bounds_of(ch_b0 + 1), bd2 = bounds_of(ch_b0 + 2), bd3 = bounds_of(ch_b0 + 3);
        {
            const Bounds bd0 = bounds_of(ch_b0);
            Staged st0;
            fetch(bd0, st0);
            if (tid < kDenseK) {
                ids_lds[0][tid] = id_of(bd0);
                ids_lds[1][tid] = id_of(bd1);
            }
            __syncthreads();  // the buffers are cleared, the ids of blocks 0 and 1 are in place
            if (bd0.ft >= 0)
                copy_operand(bd0.ft, 0);
            else
                place(bd0, st0, 0);
        }
        Staged st;        // this thread's edge of block 1's list
        fetch(bd1, st);
        int id_reg = id_of(bd2);  // ids of block 2
        u32x4 xc[8], xn[8];
        if (active) load_rows(0, xc);
        __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): a copied operand has landed
        __syncthreads();

        for (int b = ch_b0; b < ch_b1; ++b) {
            // at the top: bd1 / bd2 / bd3 describe blocks b + 1 / b + 2 / b + 3, st is this thread's edge of block b + 1,
            // id_reg an id of block b + 2, ids_lds holds the ids of blocks b and b + 1, lds[cur] the operand of block b
            const int it = b - ch_b0;
            const int cur = it % 3, nxt = (it + 1) % 3, old = (it + 2) % 3;
            const bool more = b + 1 < ch_b1;
            if (more && active) load_rows(nxt, xn);
            const bool copied = more && bd1.ft >= 0;
            if (copied)
                copy_operand(bd1.ft, nxt);                // (every byte of the buffer is overwritten)
            else if (more)
                place(bd1, st, nxt);                      // (the buffer was cleared two blocks ago)
            if (tid < kDenseK) ids_lds[old][tid] = id_reg;  // ids of block b + 2 (the slot's last reader was block b - 1's row loads)
            fetch(bd2, st);                               // this thread's edge of block b + 2
            id_reg = id_of(bd3);                          // ids of block b + 3
            const Bounds bd4 = bounds_of(b + 4);
            clear(old);                                   // (read for the last time in the previous block)
            if (active) {
                // the high parts of the weights, then the low parts, with the same B operands formed twice: byte permutes
                // are cheaper than the 16 registers that keeping both parts of A (or the operands) would cost
#pragma unroll
                for (int part = 0; part < 2; ++part) {
                    if (part == 1 && !a.use_low) break;
                    u32x4 av[4];
#pragma unroll
                    for (int mt = 0; mt < 4; ++mt) av[mt] = *reinterpret_cast<const u32x4*>(&lds[cur][part][(mt * 64 + lane) * 8]);
#pragma unroll
                    for (int p = 0; p < 4; ++p) {  // feature pair (2p, 2p + 1) of the octet: dword p of every row fragment
                        u32x4 blo, bhi;
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            blo[q] = __builtin_amdgcn_perm(xc[2 * q + 1][p], xc[2 * q][p], kPermLow);
                            bhi[q] = __builtin_amdgcn_perm(xc[2 * q + 1][p], xc[2 * q][p], kPermHigh);
                        }
                        const bf16x8 b0v = __builtin_bit_cast(bf16x8, blo), b1v = __builtin_bit_cast(bf16x8, bhi);
#pragma unroll
                        for (int mt = 0; mt < 4; ++mt) {
                            const bf16x8 a8 = __builtin_bit_cast(bf16x8, av[mt]);
                            acc[mt][2 * p] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a8, b0v, acc[mt][2 * p], 0, 0, 0);
                            acc[mt][2 * p + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a8, b1v, acc[mt][2 * p + 1], 0, 0, 0);
                        }
                    }
                }
            }
            if (copied) __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): this wavefront's share of the copied operand has landed
            __syncthreads();
#pragma unroll
            for (int j = 0; j < 8; ++j) xc[j] = xn[j];
            bd1 = bd2;
            bd2 = bd3;
            bd3 = bd4;
        }

        // the accumulators of sub-tile mt hold, in lane (kg, oct), destinations 16 mt + 4 kg + r (r = register) at
        // features col .. col + 7 (one per accumulator f): eight consecutive floats of that destination's partial row
        if (active) {
#pragma unroll
            for (int mt = 0; mt < 4; ++mt)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int m = mt * 16 + kg * 4 + r;
                    const int slot0 = a.tile_row_slot0[(int64_t)ch_tile * kDenseM + m];
                    if (slot0 < 0) continue;
                    float* p = a.partials + (int64_t)(slot0 + ch_cidx) * a.F + col;
                    const f32x4 lo = {acc[mt][0][r], acc[mt][1][r], acc[mt][2][r], acc[mt][3][r]};
                    const f32x4 hi = {acc[mt][4][r], acc[mt][5][r], acc[mt][6][r], acc[mt][7][r]};
                    __builtin_nontemporal_store(lo, reinterpret_cast<f32x4*>(p));
                    __builtin_nontemporal_store(hi, reinterpret_cast<f32x4*>(p + 4));
                }
        }
    }
}

// The edge data in the orders and forms the two kernels read them.
__global__ __launch_bounds__(256) void k_pack_hybrid_weights(const PackArgs a)
{
    const int64_t total = a.n_list + a.n_tile + a.n_rem;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        if (i < a.n_list + a.n_tile) {
            const bool list = i < a.n_list;
            const int64_t k = list ? i : i - a.n_list;
            const float x = a.w ? a.w[list ? a.de_edge[k] : a.dt_edge[k]] : 1.0f;
            const uint16_t hi = bf16_rne(x);
            const uint16_t lo = bf16_rne(x - __uint_as_float((uint32_t)hi << 16));
            if (list) {
                a.de_w[k] = (uint32_t)hi | ((uint32_t)lo << 16);
            } else {
                const int at = a.dt_addr[k];
                a.de_tiles[at] = hi;
                a.de_tiles[at + kCells] = lo;
            }
        } else {
            const int64_t k = i - a.n_list - a.n_tile;
            a.rem_w[k] = a.w[a.rem_edge[k]];
        }
    }
}

}  // namespace

hipError_t launch_dense_blocks(const DenseArgs& a, hipStream_t s)
{
    if (a.n_chunks <= 0) return hipSuccess;
    if (a.F <= 0 || a.F % 128 != 0 || a.ld % 8 != 0 || (reinterpret_cast<uintptr_t>(a.X) & 15u) || (reinterpret_cast<uintptr_t>(a.partials) & 15u) ||
        (reinterpret_cast<uintptr_t>(a.de_tiles) & 15u) || a.n_chunks > 0x7fffffffLL)
        return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_dense_blocks, dim3((unsigned)a.n_chunks), dim3(256), 0, s, a);
    return hipGetLastError();
}

hipError_t launch_pack_hybrid_weights(const PackArgs& in, hipStream_t s)
{
    PackArgs a = in;
    if (!a.w) a.n_rem = 0;  // without edge data the remainder is read unweighted
    const int64_t total = a.n_list + a.n_tile + a.n_rem;
    if (total <= 0) return hipSuccess;
    const int grid = (int)std::min<int64_t>((total + 255) / 256, 1 << 20);
    hipLaunchKernelGGL(k_pack_hybrid_weights, dim3(grid), dim3(256), 0, s, a);
    return hipGetLastError();
}

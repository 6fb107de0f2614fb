// Matrix-core kernel of the block-pruned matrix product (paper, section 2.1.2), gfx950, binary16 storage.
//
// A workgroup of four wavefronts computes a 64-row x 512-column tile of y.  The plan has gathered, per
// row tile, the columns of the weight matrix that any block of the tile keeps into one compact list
// and packed the weights at those columns in MFMA operand order (zeros where a block pruned the row).
// The kernel walks the list 16 entries at a time: the 16 rows of x the entries name are copied
// memory-to-LDS (one direct-load instruction per row: 512 columns are 1 KB, the most one instruction
// moves), the two weight operands likewise, into a ring of stages; the x operand is read from LDS
// with the transposing read, which turns [list entry][column] storage into the MFMA's per-column
// fragments.  Pruned columns therefore cost no traffic and no arithmetic; pruned rows inside a kept
// column are zero operands.  v_mfma_f32_32x32x16_f16 accumulates in fp32; bias is the accumulators'
// initial value; ReLU, the rounding to binary16 and a transposition through LDS (so that stores are
// 256-byte runs) finish the tile.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>
#include <type_traits>

#include "block_plan.hpp"

namespace ppc {

struct K4Args {
    const void* x;              // [k][n] binary16
    void* y;                    // [m][n] binary16
    const void* apk;            // weight operands [chunk][2][64][8] binary16
    const float* bias;          // [row_tiles * 64]
    const int32_t* tile_off;    // [row_tiles + 1], multiples of 16
    const int32_t* tile_cols;   // compact lists
    int32_t m, n, row_tiles, col_tiles, items, per_xcd, relu;
    // a batch of products with the same weights (the images of a 1x1 convolution): item = (image, column tile, row tile)
    int64_t x_stride, y_stride;  // elements between the x (y) matrices of consecutive images
};

constexpr int kK4Stages = 4;
constexpr int kK4RowPitch = 1024 + 64;                                   // bytes between staged rows of x: an odd multiple of 64,
                                                                          // so the four rows one transposing read touches use different banks
constexpr int kK4StageBytes = kBlockChunk * kK4RowPitch + 2 * 1024;      // 16 rows of x + two weight operands
constexpr int kK4CornerPitch = 256 + 16;                                 // epilogue: [32 rows][128 columns] binary16 per wavefront
constexpr int kK4LdsBytes = kK4Stages * kK4StageBytes;
static_assert(4 * 32 * kK4CornerPitch <= kK4LdsBytes, "the epilogue reuses the ring");

typedef __fp16 k4_hh4 __attribute__((__vector_size__(4 * sizeof(__fp16))));
typedef _Float16 k4_h2 __attribute__((ext_vector_type(2)));
typedef _Float16 k4_h4 __attribute__((ext_vector_type(4)));
typedef _Float16 k4_h8 __attribute__((ext_vector_type(8)));
typedef float k4_f2 __attribute__((ext_vector_type(2)));
typedef float k4_f16 __attribute__((ext_vector_type(16)));
typedef uint32_t k4_u4 __attribute__((ext_vector_type(4)));

template <typename P> __device__ __forceinline__ P* k4_uniform_ptr(P* p) {
    const uint64_t v = (uint64_t)(uintptr_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (P*)(uintptr_t)(((uint64_t)hi << 32) | lo);
}

// One direct load: every active lane fetches 16 bytes at base + off into LDS at lds_dst + 16 * lane.
// Inline assembly: the compiler cannot tell which stage an in-flight direct load fills and would make
// the next LDS read wait for all of them.
__device__ __forceinline__ void k4_dma16(uint32_t off, const void* base, uint32_t lds_dst) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(off), "s"(base), "s"(lds_dst) : "memory", "m0");
}

// s_waitcnt vmcnt(n) for a wave-uniform n in 0..15
__device__ __forceinline__ void k4_wait_vm(int n) {
    switch (n) {
#define PPC_K4_W(N) case N: asm volatile("s_waitcnt vmcnt(" #N ")" ::: "memory"); break;
        PPC_K4_W(1) PPC_K4_W(2) PPC_K4_W(3) PPC_K4_W(4) PPC_K4_W(5) PPC_K4_W(6) PPC_K4_W(7) PPC_K4_W(8) PPC_K4_W(9) PPC_K4_W(10)
        PPC_K4_W(11) PPC_K4_W(12) PPC_K4_W(13) PPC_K4_W(14) PPC_K4_W(15)
#undef PPC_K4_W
        default: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
    }
}

__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2))) void k4_block_gemm(const K4Args a) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char k4_smem[];
    constexpr int NS = kK4Stages, NT = 4;
    const int lane = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    // Consecutive workgroup ids land on different XCDs (id % 8): each XCD takes a contiguous range of
    // work items, ordered column tile first, so that the workgroups sharing an L2 read the same columns of x.
    const int item = (int)(blockIdx.x & 7u) * a.per_xcd + (int)(blockIdx.x >> 3);
    if (item >= a.items) return;
    const int per_image = a.row_tiles * a.col_tiles;
    const int img = item / per_image, in_image = item - img * per_image;
    const int ct = in_image / a.row_tiles, rt = in_image - ct * a.row_tiles;
    const int col0 = ct * kBlockColTile;
    const int e0 = __builtin_amdgcn_readfirstlane(a.tile_off[rt]), e1 = __builtin_amdgcn_readfirstlane(a.tile_off[rt + 1]);
    const int nch = (e1 - e0) / kBlockChunk;
    // the list is read through the constant address space: wave-uniform scalar loads, which do not count
    // against the direct loads in flight
    typedef const __attribute__((address_space(4))) int32_t* k4_const_i32;
    const k4_const_i32 list = (k4_const_i32)(uintptr_t)k4_uniform_ptr(a.tile_cols + e0);
    const unsigned char* wsrc = k4_uniform_ptr(static_cast<const unsigned char*>(a.apk) + (int64_t)(e0 / kBlockChunk) * 2048 + wave * 1024);
    const unsigned char* xsrc = k4_uniform_ptr(static_cast<const unsigned char*>(a.x) + ((int64_t)img * a.x_stride + col0) * 2);
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)k4_smem;
    const uint32_t lane16 = (uint32_t)lane * 16u;
    const bool piece_ok = col0 + lane * 8 < a.n;            // n is a multiple of 8: a 16-byte piece is inside a row or outside
    const uint32_t row_bytes = (uint32_t)a.n * 2u;          // x is smaller than 4 GB: byte offsets fit 32 bits
    const bool wload = wave < 2;                            // wavefronts 0 and 1 also fetch the two weight operands

    // chunks are issued in order, so the four list entries of the next chunk to issue are fetched one
    // issue ahead (the list is padded by a chunk at its very end)
    int rows[4];
    k4_const_i32 next_rows = list + wave;
    auto fetch_rows = [&]() {
#pragma unroll
        for (int i = 0; i < 4; ++i) rows[i] = next_rows[4 * i];
        next_rows += kBlockChunk;
    };
    auto issue = [&](int c, int stage) {
        const uint32_t st = lds0 + (uint32_t)(stage * kK4StageBytes);
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const uint32_t off = (uint32_t)rows[i] * row_bytes + lane16;
            if (piece_ok) k4_dma16(off, xsrc, st + (uint32_t)((wave + 4 * i) * kK4RowPitch));
        }
        if (wload) k4_dma16(lane16, wsrc + (int64_t)c * 2048, st + (uint32_t)(kBlockChunk * kK4RowPitch + wave * 1024));
        fetch_rows();
    };

    // accumulators: register i of tile (mt, nt) is row mt * 32 + (i / 4) * 8 + (lane / 32) * 4 + i % 4, column nt * 32 + lane % 32
    k4_f16 acc[2][NT];
    {
        const float* b = a.bias + rt * kBlockRowTile + (lane >> 5) * 4;
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float bv = b[mt * 32 + (i >> 2) * 8 + (i & 3)];
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) acc[mt][nt][i] = bv;
            }
    }

    // transposing read: inside a block of 16 lanes, lane 4 j + q reads four columns of list entry j; the
    // result hands lane i column i of entries 0..3.  Blocks 0, 1 take columns 0-15, 16-31 of entries
    // 0-7 (two reads: entries j and j + 4), blocks 2, 3 the same columns of entries 8-15.
    const int blk = lane >> 4, jj = (lane & 15) >> 2, qq = lane & 3;
    const uint32_t bbase = (uint32_t)((8 * (blk >> 1) + jj) * kK4RowPitch + (wave * 128 + 16 * (blk & 1) + 4 * qq) * 2);

    // Operand fragments live in two register sets: while the MFMAs of chunk c run from one, the
    // fragments of chunk c + 1 are read into the other, behind the one barrier per chunk that says
    // "chunk c + 1 has landed for every wavefront, and every wavefront has read chunk c out of LDS"
    // -- which also frees chunk c's stage for chunk c + 4.
    k4_h8 af[2][2], bf[2][NT];
    auto read_frags = [&](int stage, int set) {
        const uint32_t st = lds0 + (uint32_t)(stage * kK4StageBytes);
        const unsigned char* wst = k4_smem + stage * kK4StageBytes + kBlockChunk * kK4RowPitch + lane * 16;
        af[set][0] = *reinterpret_cast<const k4_h8*>(wst);
        af[set][1] = *reinterpret_cast<const k4_h8*>(wst + 1024);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const uint32_t ad = st + bbase + (uint32_t)(nt * 64);
            const k4_hh4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4f16(reinterpret_cast<__attribute__((address_space(3))) k4_hh4*>(ad));
            const k4_hh4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4f16(reinterpret_cast<__attribute__((address_space(3))) k4_hh4*>(ad + (uint32_t)(4 * kK4RowPitch)));
            bf[set][nt] = __builtin_shufflevector(__builtin_bit_cast(k4_h4, lo), __builtin_bit_cast(k4_h4, hi), 0, 1, 2, 3, 4, 5, 6, 7);
        }
    };
    // waits until this wavefront's direct loads of a chunk have landed, given how many younger chunks it has issued
    auto wait_chunk = [&](int younger) {
        if (younger >= 2) {
            if (wload) asm volatile("s_waitcnt vmcnt(10)" ::: "memory");
            else asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
        } else {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        }
    };
    auto step = [&](auto stage_tag, int c) {               // c % NS == S
        constexpr int S = decltype(stage_tag)::value;
        if (c + 1 < nch) {
            wait_chunk(nch - 2 - c);                       // chunks c + 2 and c + 3 may still be in flight
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // this wavefront's reads of chunk c have left LDS before anyone refills its stage
            __syncthreads();
            if (c + NS < nch) issue(c + NS, S);
            read_frags((S + 1) % NS, (S + 1) & 1);
        }
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) acc[mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[S & 1][mt], bf[S & 1][nt], acc[mt][nt], 0, 0, 0);
    };

    fetch_rows();
    if (nch > 0) {
#pragma unroll
        for (int c = 0; c < NS; ++c)
            if (c < nch) issue(c, c);
        k4_wait_vm((nch > NS ? NS - 1 : nch - 1) * (wload ? 5 : 4));
        __syncthreads();
        read_frags(0, 0);
#pragma unroll 1
        for (int c = 0; c < nch; c += NS) {
            step(std::integral_constant<int, 0>{}, c);
            if (c + 1 < nch) step(std::integral_constant<int, 1>{}, c + 1);
            if (c + 2 < nch) step(std::integral_constant<int, 2>{}, c + 2);
            if (c + 3 < nch) step(std::integral_constant<int, 3>{}, c + 3);
        }
    }
    __syncthreads();                           // the ring is free: its memory becomes the wavefronts' corners

    // ---- epilogue: ReLU, binary16, transpose through LDS, 16-byte stores in 256-byte runs ----
    unsigned char* corner = k4_smem + wave * 32 * kK4CornerPitch;
    const int p = lane & 31, kb = lane >> 5;
    const k4_h2 floor2 = a.relu ? k4_h2((_Float16)0.0f) : k4_h2((_Float16)-65504.0f);
    const int srow = lane >> 4, scol = (lane & 15) * 8;                  // store side: 16 lanes hold one row's 128 columns
    const int ycol = col0 + wave * 128 + scol;
    const bool col_ok = ycol < a.n;
    unsigned char* ybase = static_cast<unsigned char*>(a.y) + (int64_t)img * a.y_stride * 2;
#pragma unroll
    for (int mt = 0; mt < 2; ++mt) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int r = 0; r < 16; r += 2) {
                k4_f2 pr;
                pr.x = acc[mt][nt][r], pr.y = acc[mt][nt][r + 1];
                k4_h2 hv = __builtin_convertvector(pr, k4_h2);          // rows (row, row + 1) of this column, rounded to nearest even
                hv = __builtin_elementwise_max(hv, floor2);             // ReLU, or nothing (the floor is then the lowest finite value)
                const int row = (r >> 2) * 8 + kb * 4 + (r & 3);
                *reinterpret_cast<_Float16*>(corner + row * kK4CornerPitch + (nt * 32 + p) * 2) = hv.x;
                *reinterpret_cast<_Float16*>(corner + (row + 1) * kK4CornerPitch + (nt * 32 + p) * 2) = hv.y;
            }
        // a wavefront's LDS operations execute in order: its own corner needs no barrier
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int row = j * 4 + srow;
            const k4_u4 v = *reinterpret_cast<const k4_u4*>(corner + row * kK4CornerPitch + scol * 2);
            const int yrow = rt * kBlockRowTile + mt * 32 + row;
            if (col_ok && yrow < a.m) *reinterpret_cast<k4_u4*>(ybase + ((int64_t)yrow * a.n + ycol) * 2) = v;
        }
    }
}

// Generic kernel: one lane per output element, walking the tile's compact list (any dtype, any n).
template <typename T>
__global__ __launch_bounds__(256) void k4_generic(const T* __restrict__ x, T* __restrict__ y, const float* __restrict__ wc,
                                                  const float* __restrict__ bias, const int32_t* __restrict__ tile_off,
                                                  const int32_t* __restrict__ tile_cols, const int32_t* __restrict__ tile_len, int m, int n, int relu) {
    const int t = (int)blockIdx.y, j = (int)(blockIdx.x * 64 + threadIdx.x);
    if (j >= n) return;
    const int e0 = tile_off[t], len = tile_len[t];
    for (int r = (int)threadIdx.y; r < kBlockRowTile; r += (int)blockDim.y) {
        const int row = t * kBlockRowTile + r;
        if (row >= m) break;
        float acc = bias[row];
        for (int i = 0; i < len; ++i) acc = __builtin_fmaf(wc[(int64_t)(e0 + i) * kBlockRowTile + r], (float)x[(int64_t)tile_cols[e0 + i] * n + j], acc);
        if (relu) acc = acc > 0.0f ? acc : 0.0f;
        y[(int64_t)row * n + j] = (T)acc;
    }
}

}  // namespace ppc

// Direct-load matrix-core kernel for 3x3, stride-1 pattern-pruned convolutions stored in binary16
// (gfx950): the fast case of the matrix-core path.
//
// As in the general matrix-core kernel, the pruned weights are a dense zero-filled matrix and the layer
// is an implicit GEMM on v_mfma_f32_32x32x16_f16 with the filters as rows, output pixels as columns and
// (tap, input channel) as the reduction index, 16 channels per step.  What differs is how the input,
// which lies channel-outermost in memory (NCHW), becomes the "B" operand, which wants 8 consecutive
// channels of one pixel per lane:
//   * Staging moves no data through registers.  Every wavefront instruction of
//     global_load_lds_dwordx4 copies 64 pieces of 16 bytes (8 pixels of one channel row) straight from
//     memory into LDS, where the tile keeps the memory's own layout, [channel][row][column].
//   * The transposition happens in the LDS read: ds_read_b64_tr_b16 hands each lane of a 16-lane
//     block the four channels of its own pixel (lanes 4j..4j+3 address the 16 pixels of channel j;
//     lane i receives element i of each of the four rows).  Two such reads make one operand.
//   * That read takes 8-byte-aligned addresses only, so an operand cannot be shifted by one pixel to
//     reach the left and right taps.  The shift is moved to the other side of the product: the three
//     tap columns accumulate into three separate sets of accumulators, all from the same unshifted
//     operand,   P_c[j] = sum over tap rows r and channels of  w[r][c] * x[row + r][j],
//     and the output is  y[o] = P_0[o] + P_1[o+1] + P_2[o+2]  (computed column j holds input column
//     o - 1 + j of the segment), which the epilogue forms with two whole-wavefront lane shifts (DPP) per
//     value.  An operand is read once per tap row and used for six MFMAs.
// A column tile of 32 lanes is cut into segments of 32 or 16 computed columns, each with one halo
// column at either end (30 or 14 outputs), so no shift ever crosses a segment.  Segments are staged
// from memory one by one, each from the (2-byte aligned) address of its own first halo column, which
// keeps every LDS piece aligned whatever the segment's position in the image.
//
// Columns outside the image are not zeroed in LDS: a column of the operand only ever reaches the same
// column of the accumulators, so the two places where such a column would leak into a stored output
// (input column -1 through P_0, input column W through P_2) are cleared in the accumulators instead.
// Rows outside the images (padding and the separator row between two images of the batch) are never
// loaded; their places in LDS are zeroed whenever a ring place is filled for a tile that has such rows.
//
// Time.  On this chip a SIMD's vector ALU and its matrix core do not run side by side (measured: a
// wavefront of FMAs and a wavefront of MFMAs on one SIMD take the sum of their times), so every vector
// instruction is time taken from the MFMAs, and the kernel is written to have few of them:
//   * workgroups are persistent and walk through their tiles; the steps (chunk after chunk, tile after
//     tile) are staged one or two ahead into a ring of LDS buffers, with the load instructions dealt out
//     between the MFMAs of the step before and awaited by count (loads return in order);
//   * what a lane fetches is worked out once per tile from per-lane constants kept in LDS, at the head
//     of the tile before, and parked in LDS until the ring gets there (registers are short: 192 of 256
//     are accumulators);
//   * the bias arrives by a direct load and enters as the C operand of a tile's first MFMAs;
//   * the epilogue turns the outputs round through LDS so that one store instruction writes 64-byte runs
//     of 16 filters: a store costs the same whether a lane carries 2 or 16 bytes.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "mfma3_geom.hpp"
#include "mfma_geom.hpp"

namespace ppc {

struct K3Args {
    const void* x;
    void* y;
    const void* wpk;            // weight fragments [fb][q][9][2][64][8] binary16
    const float* bias;          // [fb*64]
    int32_t n, c_in, c_out, h, w;
    int32_t po;                 // rows per image of the tall virtual image: h + 1
    int32_t vrows;              // (n - 1) * po + h
    int32_t tr, nseg;           // tile: rows x segments
    int32_t tiles_x, tiles_v, fb, q;
    int32_t work_items, blocks_per_xcd;
    int32_t chs, ppc, ppcp, nxi, xbuf_bytes;
    // floor(2^32 / d) + 1 for: pieces per channel with padding, pieces per staged row, segments per
    // tile row, rows per image (0 stands for d = 1)
    uint32_t magic_ppcp, magic_ppr, magic_nseg, magic_po;
    int32_t relu;
    int64_t x_elems;            // n * c_in * h * w
    // split reduction (SPLIT instantiations): each work item takes qs = q / ksplit consecutive chunks and stores
    // its partial sums, without bias or activation, as binary32 into slab ks of the workspace ([ksplit][n][c_out][h][w])
    int32_t out_h, out_w;       // size of y per image and filter (h / 2 x w / 2 with the fused pool, else h x w)
    int32_t ksplit, qs;
    float* ws;
    int64_t slab_elems;         // n * c_out * h * w
};

typedef __fp16 k3_hh4 __attribute__((__vector_size__(4 * sizeof(__fp16))));
typedef _Float16 k3_h2 __attribute__((ext_vector_type(2)));
typedef _Float16 k3_h4 __attribute__((ext_vector_type(4)));
typedef _Float16 k3_h8 __attribute__((ext_vector_type(8)));
typedef float k3_f2 __attribute__((ext_vector_type(2)));
typedef float k3_f16 __attribute__((ext_vector_type(16)));
typedef uint32_t k3_u3 __attribute__((ext_vector_type(3)));
typedef uint32_t k3_u4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) unsigned char* k3_lds_ptr;
typedef uint32_t __attribute__((may_alias)) k3_u32_alias;

// n / d for n < 65536 and 1 <= d < 65536 with magic = floor(2^32 / d) + 1 (0 stands for d = 1)
__device__ __forceinline__ int k3_div(int n, uint32_t magic) { return magic ? (int)__umulhi((uint32_t)n, magic) : n; }

template <typename P> __device__ __forceinline__ P* k3_uniform_ptr(P* p) {
    const uint64_t v = (uint64_t)(uintptr_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (P*)(uintptr_t)(((uint64_t)hi << 32) | lo);
}

// One direct load: every active lane fetches 16 (or 4) bytes at base + off into LDS at lds_dst + 16 (4) * lane.
// Inline assembly rather than the compiler builtin: the compiler cannot tell which buffer an
// in-flight direct load fills and would make the first LDS read after it wait for all of them.
__device__ __forceinline__ void k3_dma16(uint32_t off, const void* base, uint32_t lds_dst) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(off), "s"(base), "s"(lds_dst) : "memory", "m0");
}
__device__ __forceinline__ void k3_dma4(uint32_t off, const void* base, uint32_t lds_dst) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1" ::"v"(off), "s"(base), "s"(lds_dst) : "memory", "m0");
}

// A staged piece that reaches outside the tensor (the halo column in front of the very first row, the
// columns behind the very last one): eight guarded element loads, zeros outside.  Rare; kept out of line.
__device__ __attribute__((noinline)) void k3_edge_piece(const uint16_t* x, int64_t e0, int64_t n_elems, unsigned char* lds_dst) {
    uint32_t v[4];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
        const int64_t idx = e0 + e;
        const uint32_t bits = (idx >= 0 && idx < n_elems) ? (uint32_t)x[idx] : 0u;
        v[e >> 1] = (e & 1) ? (v[e >> 1] | (bits << 16)) : bits;
    }
    k3_u4 v4;
    v4.x = v[0], v4.y = v[1], v4.z = v[2], v4.w = v[3];
    *reinterpret_cast<k3_u4*>(lds_dst) = v4;
}

// s_waitcnt vmcnt(n) for a wave-uniform n (0..31; anything else waits for everything)
__device__ __forceinline__ void k3_wait_vm(int n) {
    switch (n) {
#define PPC_K3_W(N) case N: asm volatile("s_waitcnt vmcnt(" #N ")" ::: "memory"); break;
        PPC_K3_W(1) PPC_K3_W(2) PPC_K3_W(3) PPC_K3_W(4) PPC_K3_W(5) PPC_K3_W(6) PPC_K3_W(7) PPC_K3_W(8) PPC_K3_W(9) PPC_K3_W(10)
        PPC_K3_W(11) PPC_K3_W(12) PPC_K3_W(13) PPC_K3_W(14) PPC_K3_W(15) PPC_K3_W(16) PPC_K3_W(17) PPC_K3_W(18) PPC_K3_W(19) PPC_K3_W(20)
        PPC_K3_W(21) PPC_K3_W(22) PPC_K3_W(23) PPC_K3_W(24) PPC_K3_W(25) PPC_K3_W(26) PPC_K3_W(27) PPC_K3_W(28) PPC_K3_W(29) PPC_K3_W(30) PPC_K3_W(31)
#undef PPC_K3_W
        default: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
    }
}

// lane i <- lane i + 1 over the whole wavefront (the last lane receives 0)
__device__ __forceinline__ float k3_shl1(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x130, 0xf, 0xf, true));
}

template <int SW, int WAVES, bool SPLIT, bool POOL>
__global__ __launch_bounds__(64 * WAVES) __attribute__((amdgpu_waves_per_eu(2, 2)))
void k3_mfma(const K3Args a) {
    constexpr int NT = kK3ColTiles, UPT = 32 / SW, SEGB = SW * 2, PPS = SEGB / 16, VALID = SW - 2;
    constexpr int MAXX = k3_max_x_units(WAVES);
    constexpr int NS = k3_stages(WAVES);             // ring of staged steps
    constexpr int NWU = 18, WU = (NWU + WAVES - 1) / WAVES;
    constexpr int NL = 64 * WAVES;                   // lanes of the workgroup
    static_assert(WU + MAXX <= 9, "one staging slot per tap");
    extern __shared__ __align__(16) unsigned char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // Workgroups are persistent: the grid holds as many as are resident at once, and each walks through
    // its share of the work items (filter block fastest, then tile column, then tile row).  Block ids go
    // round-robin to the 8 XCDs, so XCD i gets the contiguous item range [i * blocks_per_xcd, ...) and
    // its workgroups take the items of that range in turn: at any moment an XCD works on neighbouring
    // tiles, which share input rows, and its L2 sees them together.
    const int xcd = (int)(blockIdx.x % 8u), slot = (int)(blockIdx.x / 8u), gslots = (int)(gridDim.x / 8u);
    const int first_item = xcd * a.blocks_per_xcd;
    const int left = a.work_items - first_item, avail = left < a.blocks_per_xcd ? left : a.blocks_per_xcd;
    const int my_n = avail > slot ? (avail - slot + gslots - 1) / gslots : 0;
    if (my_n == 0) return;

    const int hw = a.h * a.w;
    const uint32_t lds0 = (uint32_t)(uintptr_t)(k3_lds_ptr)smem;
    const int xb_bytes = a.xbuf_bytes;
    const int rowb = a.nseg * SEGB;                 // LDS bytes per staged row of one channel
    const _Float16* __restrict__ xin = static_cast<const _Float16*>(a.x);
    // LDS behind the ring: per wavefront 64 bias values and a [32 filters][32 columns] binary16 tile for
    // the epilogue; per lane the parked staging set of the next tile and the lane's staging constants
    const int corner0 = NS * (xb_bytes + kK3WeightBytes);
    float* bias_lds = reinterpret_cast<float*>(smem + corner0) + wave * kMfmaFilters;
    unsigned char* tb = smem + corner0 + WAVES * kMfmaFilters * 4 + wave * 2048;
    uint32_t* park = reinterpret_cast<uint32_t*>(smem + corner0 + WAVES * (kMfmaFilters * 4 + 2048)) + tid;   // [MAXX + 1][NL]
    uint32_t* lconst = park + (MAXX + 1) * NL;                                                                  // [2 * MAXX][NL]

    // ---- staging: which piece each lane fetches in each of this wavefront's instructions ----
    // Instruction `it` fills LDS bytes [1024 it, 1024 it + 1024) of a ring place; piece g = 64 it + lane is
    // piece g % ppcp of channel g / ppcp.  What does not depend on the tile is worked out here, once:
    // the piece's element offset from (channel 0, image 0, row 0, the tile's first output column), and its
    // staged row and first column relative to the tile (bit 31: no place of the tile, padding).
    const int nx = wave < a.nxi ? (a.nxi - wave + WAVES - 1) / WAVES : 0;
    const int nwu = (NWU - wave + WAVES - 1) / WAVES;                     // weight instructions of this wavefront per step
#pragma unroll
    for (int k = 0; k < MAXX; ++k) {
        const int g = (wave + WAVES * k) * 64 + lane;
        const int ch = k3_div(g, a.magic_ppcp), pr = g - ch * a.ppcp;
        const int srow = k3_div(pr, a.magic_ppr), rem = pr - srow * (a.nseg * PPS);
        const int seg = rem / PPS, piece = rem - seg * PPS;
        const int colrel = seg * VALID - 1 + piece * 8;                   // first column of the piece, from the tile's first output column
        const bool place = k < nx && ch < kMfmaChunk && pr < a.ppc;
        lconst[(2 * k) * NL] = (uint32_t)(ch * hw + colrel);
        lconst[(2 * k + 1) * NL] = place ? (uint32_t)(srow | ((colrel + 1) << 8)) : 0x80000000u;
    }

    // tile coordinates of a work item (wave-uniform)
    auto decode = [&](int item, int& fbi_o, int& ks_o, int& ox0_o, int& v0_o) {
        fbi_o = item % a.fb;
        item /= a.fb;
        ks_o = 0;
        if constexpr (SPLIT) {
            ks_o = item % a.ksplit;
            item /= a.ksplit;
        }
        const int tx = item % a.tiles_x, tv = item / a.tiles_x;
        ox0_o = tx * a.nseg * VALID;
        v0_o = tv * a.tr;
    };

    // Per tile: the offset of each of the lane's pieces and what is to be done with it.
    uint32_t xoff[MAXX];                            // byte offset of the lane's k-th piece from (first element of the chunk's channel 0) - 16
    uint32_t cls = 0u;                              // bit k: fetch; 4+k: zero instead (outside the images); 8+k / 12+k: the piece
                                                    // reaches below / beyond the tensor in the first / last chunk
    bool any_hole = false, any_edge = false;        // wave-uniform
    int fbi_s = 0, ks_s = 0;                        // filter block and reduction share of the tile being staged
    const int QN = SPLIT ? a.qs : a.q;              // chunks per work item
    const int last_chunk_elems = (int)(a.x_elems - (int64_t)(a.q - 1) * kMfmaChunk * hw);   // the tensor has fewer than 2^31 elements
    // The set of the workgroup's next tile is worked out at the head of a tile, while the accumulators are
    // not yet in use, and parked in this lane's own words of LDS until the ring gets there.
    auto setup_tile = [&](int item) {
        int ox0, v0, fbi_n, ks_n;
        decode(item, fbi_n, ks_n, ox0, v0);
        const int u0 = v0 - 1;                                            // virtual input row of staged row 0
        const int img0 = (u0 + a.po) / a.po - 1, iy0 = u0 - img0 * a.po;  // u0 = -1 belongs to "image -1"
        const int img_hw = a.c_in * hw;
        uint32_t cls_n = 0u;
#pragma unroll
        for (int k = 0; k < MAXX; ++k) {
            const int cbase = (int)lconst[(2 * k) * NL], crow = (int)lconst[(2 * k + 1) * NL];
            const int t = iy0 + (crow & 255), di = k3_div(t, a.magic_po);
            const int img = img0 + di, iy = t - di * a.po;
            const bool place = crow >= 0;
            const bool ok = place && img >= 0 && img < a.n && iy < a.h && ox0 + ((crow >> 8) & 0xFFFF) - 1 < a.w;
            // the piece that holds input column -1 of a row starts 2 bytes before that row, and offsets must
            // not be negative: they count from 16 bytes before the chunk's first element
            const int e0 = img * img_hw + iy * a.w + ox0 + cbase;        // first element, relative to the chunk (-1 at the earliest)
            uint32_t xo = 16u;                                            // padding lanes fetch the chunk's first bytes (in bounds, never read)
            if (ok) {
                xo = 16u + 2u * (uint32_t)e0;
                cls_n |= 1u << k;
                if (e0 < 0) cls_n |= 256u << k;
                if (e0 + 8 > last_chunk_elems) cls_n |= 4096u << k;
            } else if (place) {
                cls_n |= 16u << k;
            }
            park[k * NL] = xo;
        }
        park[MAXX * NL] = cls_n;
    };
    auto take_tile = [&](int item) {                // the parked set becomes the staged tile
#pragma unroll
        for (int k = 0; k < MAXX; ++k) xoff[k] = park[k * NL];
        cls = park[MAXX * NL];
        any_hole = __builtin_amdgcn_ballot_w64((cls & 0xF0u) != 0u) != 0;
        any_edge = __builtin_amdgcn_ballot_w64((cls & 0xFF00u) != 0u) != 0;
        fbi_s = item % a.fb;
        ks_s = SPLIT ? (item / a.fb) % a.ksplit : 0;
    };

    // The loads of one step (chunk qi of the staged tile, into ring place `buf`) are WU weight instructions
    // and up to MAXX input instructions per wavefront, plus the tile's bias values with its first chunk:
    // nine "slots", issued one per tap of an earlier step, so that the address unit works through them
    // while the matrix cores run.  Nothing here waits.
    struct Step {
        const unsigned char* wbase;
        const unsigned char* xbase;
        const float* bbase;
        uint32_t ldsw, ldsx, edge_bits;
        int64_t chunk_elem0;
        int buf;
        int count;                                  // load instructions this wavefront issues for the step
        bool on;
        bool plain;                                 // every lane of every input instruction fetches (no place outside the images, no piece outside the tensor)
        bool bias;                                  // the tile's first chunk: the bias values come along
    };
    const uint32_t lane16 = (uint32_t)(lane * 16);
    auto begin_step = [&](int ql, int buf) {         // ql: chunk within the work item
        Step st;
        st.on = true;
        st.buf = buf;
        const int qi = SPLIT ? ks_s * a.qs + ql : ql; // chunk of the layer
        st.wbase = k3_uniform_ptr(static_cast<const unsigned char*>(a.wpk) + ((int64_t)fbi_s * a.q + qi) * kK3WeightBytes + wave * 1024);
        st.ldsw = lds0 + (uint32_t)(NS * xb_bytes + buf * kK3WeightBytes + wave * 1024);
        st.chunk_elem0 = (int64_t)qi * kMfmaChunk * hw;
        st.xbase = k3_uniform_ptr(reinterpret_cast<const unsigned char*>(xin + st.chunk_elem0) - 16);
        st.ldsx = lds0 + (uint32_t)(buf * xb_bytes + wave * 1024);
        st.bias = !SPLIT && qi == 0;
        st.bbase = k3_uniform_ptr(a.bias + fbi_s * kMfmaFilters);
        st.plain = !(any_edge || any_hole);
        st.edge_bits = 0u;
        st.count = nwu + nx + (st.bias ? 1 : 0);
        if (!st.plain) {
            // A piece may reach a few bytes outside the tensor at its two ends (the halo column of the very
            // first row, the columns past the very last row): those lanes assemble their piece from guarded
            // element loads instead.  Only the first and the last chunk can have such pieces.
            st.edge_bits = !any_edge ? 0u : ((qi == 0 ? (cls >> 8) & 15u : 0u) | (qi == a.q - 1 ? (cls >> 12) & 15u : 0u));
            // an instruction is issued if any lane takes part in it: count them the way issue_slot decides
            st.count = nwu + (st.bias ? 1 : 0);
#pragma unroll
            for (int k = 0; k < MAXX; ++k)
                if (k < nx && __builtin_amdgcn_ballot_w64(((cls >> k) & 1u) && !((st.edge_bits >> k) & 1u)) != 0) ++st.count;
        }
        return st;
    };
    auto issue_slot = [&](const Step& st, int j) {          // j = 0 .. 8, a compile-time constant at every call
        if (!st.on) return;
        if (j < WU) {
            if (wave + WAVES * j < NWU) k3_dma16(lane16, st.wbase + WAVES * j * 1024, st.ldsw + (uint32_t)(WAVES * j * 1024));
        } else if (j - WU < MAXX) {
            const int k = j - WU;
            if (k < nx) {
                if (st.plain) {
                    // almost every tile: all 64 lanes fetch
                    k3_dma16(xoff[k], st.xbase, st.ldsx + (uint32_t)(WAVES * k * 1024));
                } else {
                    // (the branch is on the wavefront's vote, so that the instruction count is what begin_step says)
                    const bool mine = ((cls >> k) & 1u) && !((st.edge_bits >> k) & 1u);
                    if (__builtin_amdgcn_ballot_w64(mine) != 0 && mine) k3_dma16(xoff[k], st.xbase, st.ldsx + (uint32_t)(WAVES * k * 1024));
                }
            }
        }
        // the last slot also brings this wavefront's copy of the tile's 64 bias values
        if (j == 8 && st.bias) k3_dma4(lane16 >> 2, st.bbase, lds0 + (uint32_t)(corner0 + wave * kMfmaFilters * 4));
    };
    auto finish_step = [&](const Step& st) {                 // the rare pieces that are not plain loads
        if (!st.on || st.plain) return;
#pragma unroll
        for (int k = 0; k < MAXX; ++k) {
            if (k < nx) {
                unsigned char* mine = smem + st.buf * xb_bytes + (wave + WAVES * k) * 1024 + lane * 16;
                if ((st.edge_bits >> k) & 1u)
                    k3_edge_piece(reinterpret_cast<const uint16_t*>(xin), st.chunk_elem0 + ((int64_t)(int32_t)(xoff[k] - 16u)) / 2, a.x_elems, mine);
                // a place outside the images would keep whatever the ring place's last tile left there
                if ((cls >> (4 + k)) & 1u) *reinterpret_cast<k3_u4*>(mine) = k3_u4(0u);
            }
        }
    };

    // ---- per-lane operand address: lanes 4j..4j+3 of a 16-lane block address channel j, pixels 4q..4q+3 ----
    const int blk = lane >> 4, jch = (lane >> 2) & 3, qd = lane & 3;
    uint32_t baddr[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int p0 = 16 * (blk & 1) + 4 * qd;
        const int ui = (wave * NT + nt) * UPT + p0 / SW;
        const int row = k3_div(ui, a.magic_nseg), seg = ui - row * a.nseg;
        baddr[nt] = (uint32_t)((8 * (blk >> 1) + jch) * a.chs + row * rowb + seg * SEGB + (p0 % SW) * 2);
    }
    const bool wide_ok = (a.w & 1) == 0;             // rows start on 4-byte boundaries

    // ---- accumulators: three tap columns x two filter halves x NT column tiles ----
    k3_f16 acc[3][2][NT];
    // A computed column outside the image (input column -1 or w) must not reach an output: its P_0 (for
    // output 0) or P_2 (for output w - 1) is cleared before the columns are combined.  Rare and
    // wave-uniform, so a branch around in-place selects (the empty asm keeps it a branch).
    auto clear_outside = [&](int nt, bool fix, bool kill0, bool kill2) {
        if (fix) {
            asm volatile("" ::: "memory");
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    acc[0][mt][nt][r] = kill0 ? 0.0f : acc[0][mt][nt][r];
                    acc[2][mt][nt][r] = kill2 ? 0.0f : acc[2][mt][nt][r];
                }
        }
    };

    // Steps (chunk after chunk, tile after tile) are staged NS - 1 ahead of the step being multiplied.
    int ik = 0, iq = 0, ibuf = 0;                   // the next step to stage: tile, chunk, ring place
    int young = 0;                                  // load instructions issued after those of the step that is waited for next
    // An epilogue's stores are issued behind the loads of the next NS - 1 steps: the waits for those steps
    // may leave them in flight too.  Counted is a lower bound (the full-width store instructions).
    int stores_behind = 0, store_credit = 0;
    auto advance_issue = [&]() {
        ibuf = ibuf + 1 == NS ? 0 : ibuf + 1;
        if (++iq == QN) iq = 0, ++ik;
    };
    setup_tile(first_item + slot);
    take_tile(first_item + slot);
    // fill the pipeline with the first NS - 1 steps (all of the first tile: the launcher sees to it that a
    // tile has at least NS - 1 chunks)
#pragma unroll
    for (int d = 0; d < NS - 1; ++d) {
        const Step st0 = begin_step(iq, ibuf);
#pragma unroll
        for (int j = 0; j < 9; ++j) issue_slot(st0, j);
        finish_step(st0);
        if (d > 0) young += st0.count;
        advance_issue();
    }

    // The step to stage during a multiplication: NS - 1 after the one being multiplied.
    auto next_step = [&]() -> Step {
        Step st;
        st.on = false;
        if (ik < my_n) {
            if (iq == 0) take_tile(first_item + slot + ik * gslots);   // parked at the head of tile ik - 1
            st = begin_step(iq, ibuf);
            advance_issue();
        }
        young = NS > 2 ? (st.on ? st.count : 0) : 0;
        return st;
    };

    // One step: multiply the chunk in ring place sbuf, and deal out the loads of the step to stage between the taps.
    // That step's description (a hundred-odd scalar instructions of address arithmetic) is worked out behind the
    // first tap's MFMAs rather than ahead of them: the matrix cores start right after the barrier.
    // FIRST: the tile's first chunk, whose MFMAs start the accumulators (the centre column's from the bias).
    auto multiply = [&](auto first_tag, int sbuf, int setup_item) -> Step {
        constexpr bool FIRST = decltype(first_tag)::value;
        Step nxt;
        nxt.on = false;
        const uint32_t xb = lds0 + (uint32_t)(sbuf * xb_bytes);
        const unsigned char* wb = smem + NS * xb_bytes + sbuf * kK3WeightBytes + lane * 16;
        // Operand fragments are read one tap ahead into a second set of registers, so that the LDS latency
        // of tap t + 1 hides behind the four MFMAs of tap t; the input operand changes with the tap row only.
        k3_h8 af[2][2], bf[2][NT];
        auto read_a = [&](int set, int t) {
            af[set][0] = *reinterpret_cast<const k3_h8*>(wb + (t * 2 + 0) * 1024);
            af[set][1] = *reinterpret_cast<const k3_h8*>(wb + (t * 2 + 1) * 1024);
        };
        auto read_b = [&](int set, int r) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const uint32_t ad = xb + baddr[nt] + (uint32_t)(r * rowb);
                const k3_hh4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4f16(reinterpret_cast<__attribute__((address_space(3))) k3_hh4*>(ad));
                const k3_hh4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4f16(reinterpret_cast<__attribute__((address_space(3))) k3_hh4*>(ad + (uint32_t)(4 * a.chs)));
                const k3_h4 l4 = __builtin_bit_cast(k3_h4, lo), h4 = __builtin_bit_cast(k3_h4, hi);
                bf[set][nt] = __builtin_shufflevector(l4, h4, 0, 1, 2, 3, 4, 5, 6, 7);
            }
        };
        read_b(0, 0);
        read_a(0, 0);
        k3_f16 cb[2];                               // FIRST: the bias in accumulator order (an accumulator register holds one filter)
        if constexpr (FIRST && !SPLIT) {
            const int kb = lane >> 5;
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const float4 b4 = *reinterpret_cast<const float4*>(bias_lds + mt * 32 + g * 8 + kb * 4);
                    cb[mt][g * 4 + 0] = b4.x, cb[mt][g * 4 + 1] = b4.y, cb[mt][g * 4 + 2] = b4.z, cb[mt][g * 4 + 3] = b4.w;
                }
        }
#pragma unroll
        for (int t = 0; t < 9; ++t) {
            const int r = t / 3, c = t % 3;
            if (t + 1 < 9) {
                read_a((t + 1) & 1, t + 1);
                if ((t + 1) % 3 == 0) read_b(((t + 1) / 3) & 1, (t + 1) / 3);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int mt = 0; mt < 2; ++mt) {
                    k3_f16 cin;
                    if (FIRST && r == 0) {
                        if (c == 1 && !SPLIT) cin = cb[mt];
                        else
#pragma unroll
                            for (int e = 0; e < 16; ++e) cin[e] = 0.0f;
                    } else {
                        cin = acc[c][mt][nt];
                    }
                    acc[c][mt][nt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[t & 1][mt], bf[r & 1][nt], cin, 0, 0, 0);
                }
            if (t == 0) nxt = next_step();
            if constexpr (WAVES == 8) {
                if (t == 1 && setup_item >= 0) setup_tile(setup_item);
            }
            issue_slot(nxt, t);
            __builtin_amdgcn_sched_barrier(0);
        }
        return nxt;
    };

    int sbuf = 0;                                   // ring place of the current step
    for (int kt = 0; kt < my_n; ++kt) {
        const int item_c = first_item + slot + kt * gslots;
        // The staging set of the next tile is worked out and parked in LDS before the ring gets there, which is during
        // chunk QN - (NS - 1) of this tile: behind the MFMAs of the second chunk when that is early enough (eight-wavefront
        // workgroups only: measured, it gains 2-3 % there and loses as much with four), else here, at the head of the tile.
        const bool setup_late = WAVES == 8 && QN - (NS - 1) >= 2;
        const int setup_next = kt + 1 < my_n ? item_c + gslots : -1;
        if (!setup_late && setup_next >= 0) setup_tile(setup_next);
        __builtin_amdgcn_sched_barrier(0);

        // ---- main loop over chunks of 16 channels ----
        for (int qi = 0; qi < QN; ++qi) {
            // This wavefront's loads of the current step have landed (and its zero fills and edge pieces are
            // written); after the barrier everyone's have, and everyone is done reading the ring place that
            // is filled next.  Loads return in order: all but the `young` most recent instructions are
            // awaited.
            k3_wait_vm(young + (store_credit > 0 ? stores_behind : 0));
            if (store_credit > 0) --store_credit;
            __syncthreads();
            const Step nxt = qi == 0 ? multiply(std::true_type{}, sbuf, -1) : multiply(std::false_type{}, sbuf, qi == 1 && setup_late ? setup_next : -1);
            finish_step(nxt);
            sbuf = sbuf + 1 == NS ? 0 : sbuf + 1;
        }

        // ---- epilogue: combine the three tap columns, ReLU, binary16, store ----
        // An accumulator register holds one filter for the 32 columns of a column tile (lanes 0-31; lanes
        // 32-63 hold the filter four further on).  Output o of a segment sits in lane o: its own P_0, the
        // next lane's P_1 (which carries the bias), the P_2 two lanes on.  Pairs of registers (two filters of
        // one column) are converted together and written as two 16-bit halves into this wavefront's
        // [32 filters][32 columns] corner of LDS; read back 16 bytes per lane, four lanes hold a filter's 32
        // columns and one store instruction writes 64-byte runs of 16 filters.
        // The lane's position is worked out again here, every time, instead of living in registers across
        // the main loop (the empty asm stops the compiler from hoisting it).
        int lane_e = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
        asm volatile("" : "+v"(lane_e));
        const int p = lane_e & 31, kb = lane_e >> 5;
        const int tb_w = kb * 4 * 64 + p * 2;                                 // + filter row * 64
        const int tb_r = lane_e * 16;                                         // filter lane / 4, columns 8 (lane % 4) ..
        int fbi, ks_c, ox0, v0;
        decode(item_c, fbi, ks_c, ox0, v0);
        const int oimg0 = v0 / a.po, oy0 = v0 - oimg0 * a.po;
        if constexpr (POOL) {
            // Fused 2x2 max-pool (stride 2).  The plan lays the tile out so that a wavefront's two column tiles are an
            // even row of the tall image and the row below it, same segments, same columns (segments per tile row =
            // segments per column tile), and gives every image an even number of rows in the tall image: the vertical
            // maximum is between a lane's own two accumulators, the horizontal one with the next lane.  Even lanes
            // of a segment then hold the pooled outputs, seven (or fifteen) consecutive binary16 values per segment.
            // A store instruction costs about the same however few lanes take part, so two filters share one: the even
            // lanes store the filter of register r, the odd lanes (handed the value by their even neighbour) the filter
            // of register r + 1 at the same pooled column.
            static_assert(!SPLIT && NT == 2, "the pooled epilogue pairs the two column tiles of a wavefront");
            _Float16* yb = static_cast<_Float16*>(a.y);
            const int ohw = a.out_h * a.out_w;
            const int ui = wave * NT * UPT + p / SW, col = p % SW;
            const int row = k3_div(ui, a.magic_nseg), seg = ui - row * a.nseg;
            const int ox = ox0 + seg * VALID + col;
            const bool kill0 = ox == 0, kill2 = ox == a.w + 1;
            const bool fix = __builtin_amdgcn_ballot_w64(kill0 || kill2) != 0;
            const int t = oy0 + row, di = k3_div(t, a.magic_po);
            const int img = oimg0 + di, oy = t - di * a.po;
            const int odd = col & 1;                                      // VALID and w are even: an even column and the next one are outputs together
            const bool ok = col - odd < VALID && ox - odd < a.w && v0 + row < a.vrows && oy < a.h;
            const int off = ((img * a.c_out + fbi * kMfmaFilters + kb * 4 + odd) * a.out_h + (oy >> 1)) * a.out_w + ((ox - odd) >> 1);
            const bool full = (fbi + 1) * kMfmaFilters <= a.c_out;
            stores_behind = 0;
            store_credit = NS - 1;
            if (full && __builtin_amdgcn_ballot_w64(ok) != 0) stores_behind += 16;
            const float floor1 = a.relu ? 0.0f : -65504.0f;
            clear_outside(0, fix, kill0, kill2);
            clear_outside(1, fix, kill0, kill2);
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int r = 0; r < 16; r += 2) {
                    float m[2];
#pragma unroll
                    for (int i = 0; i < 2; ++i) {
                        float v[2];
#pragma unroll
                        for (int nt = 0; nt < 2; ++nt)
                            v[nt] = acc[0][mt][nt][r + i] + k3_shl1(acc[1][mt][nt][r + i] + k3_shl1(acc[2][mt][nt][r + i]));
                        m[i] = __builtin_fmaxf(v[0], v[1]);
                        m[i] = __builtin_fmaxf(m[i], k3_shl1(m[i]));
                        m[i] = __builtin_fmaxf(m[i], floor1);
                    }
                    // lane i <- lane i - 1: an odd lane receives filter r + 1 of the pooled column of its even neighbour
                    const float up = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, m[1]), 0x138, 0xf, 0xf, true));
                    const float val = odd ? up : m[0];
                    const int f = mt * 32 + (r >> 2) * 8 + (r & 3);           // + odd: in `off`
                    if (ok && (full || fbi * kMfmaFilters + f + odd + kb * 4 < a.c_out)) yb[off + f * ohw] = (_Float16)val;
                }
            continue;
        }
        if constexpr (SPLIT) {
            // Partial sums of this item's chunks: the three tap columns combined as below, stored as binary32 into
            // the item's slab of the workspace, no bias, no activation (a second kernel adds the slabs up in
            // slab order).  A register holds one filter for 32 columns: lanes 0-31 write a 128-byte run of one
            // filter's row, lanes 32-63 the same columns of the filter four further on.  With an even image width two
            // registers share a store instruction of twice the width: the even lanes store columns (c, c + 1) of the
            // filter of register r, the odd lanes columns (c - 1, c) of the filter of register r + 1.
            float* wsb = k3_uniform_ptr(a.ws + (int64_t)ks_c * a.slab_elems);
            stores_behind = 0;
            store_credit = NS - 1;
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const int ui = (wave * NT + nt) * UPT + p / SW, col = p % SW;
                const int row = k3_div(ui, a.magic_nseg), seg = ui - row * a.nseg;
                const int ox = ox0 + seg * VALID + col;
                const bool kill0 = ox == 0, kill2 = ox == a.w + 1;
                const bool fix = __builtin_amdgcn_ballot_w64(kill0 || kill2) != 0;
                const int t = oy0 + row, di = k3_div(t, a.magic_po);
                const int img = oimg0 + di, oy = t - di * a.po;
                const bool ok = col < VALID && ox < a.w && v0 + row < a.vrows && oy < a.h;
                const int off = ((img * a.c_out + fbi * kMfmaFilters + kb * 4) * a.h + oy) * a.w + ox;   // + (filter - 4 kb) * h * w
                // a whole block of 64 filters inside the layer (wave-uniform): then every store instruction below has
                // an active lane as soon as one column of this tile is an output, and all of them are counted
                const bool full = (fbi + 1) * kMfmaFilters <= a.c_out;
                if (full && __builtin_amdgcn_ballot_w64(ok) != 0) stores_behind += wide_ok ? 16 : 32;
                clear_outside(nt, fix, kill0, kill2);
                if (wide_ok) {
                    const int odd = col & 1;                              // VALID and w are even: an even column and the next one are outputs together
                    const bool ok2 = col - odd < VALID && ox - odd < a.w && v0 + row < a.vrows && oy < a.h;
                    const int off2 = off + odd * (hw - 1);                // the odd lane: the next filter, one column back
#pragma unroll
                    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                        for (int r = 0; r < 16; r += 2) {
                            const float va = acc[0][mt][nt][r] + k3_shl1(acc[1][mt][nt][r] + k3_shl1(acc[2][mt][nt][r]));
                            const float vb = acc[0][mt][nt][r + 1] + k3_shl1(acc[1][mt][nt][r + 1] + k3_shl1(acc[2][mt][nt][r + 1]));
                            const float va_next = k3_shl1(va);            // lane i <- lane i + 1
                            const float vb_prev = __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, vb), 0x138, 0xf, 0xf, true));   // lane i <- lane i - 1
                            k3_f2 pair;
                            pair.x = odd ? vb_prev : va;
                            pair.y = odd ? vb : va_next;
                            const int f = mt * 32 + (r >> 2) * 8 + (r & 3);           // + odd (in off2) + 4 kb
                            if (ok2 && (full || fbi * kMfmaFilters + f + odd + kb * 4 < a.c_out)) *reinterpret_cast<k3_f2*>(wsb + off2 + f * hw) = pair;
                        }
                    continue;
                }
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float v = acc[0][mt][nt][r] + k3_shl1(acc[1][mt][nt][r] + k3_shl1(acc[2][mt][nt][r]));
                        const int f = mt * 32 + (r >> 2) * 8 + (r & 3);               // + 4 kb: the register's filter inside the block
                        if (ok && (full || fbi * kMfmaFilters + f + kb * 4 < a.c_out)) wsb[off + f * hw] = v;
                    }
            }
            continue;
        }
        unsigned char* ybase = static_cast<unsigned char*>(a.y);
        const uint32_t fstride = (uint32_t)(a.h * a.w * 2);              // bytes between filters
        const k3_h2 floor2 = a.relu ? k3_h2((_Float16)0.0f) : k3_h2((_Float16)-65504.0f);
        stores_behind = 0;
        store_credit = NS - 1;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            // accumulator side: this lane's computed column is input column ox - 1, outside the image for
            // ox = 0 (it would reach output 0 through P_0) and for ox = w + 1 (output w - 1 through P_2)
            bool kill0, kill2, fix;
            {
                const int ui = (wave * NT + nt) * UPT + p / SW, col = p % SW;
                const int row = k3_div(ui, a.magic_nseg), seg = ui - row * a.nseg;
                const int ox = ox0 + seg * VALID + col;
                kill0 = ox == 0;
                kill2 = ox == a.w + 1;
                fix = __builtin_amdgcn_ballot_w64(kill0 || kill2) != 0;
            }
            clear_outside(nt, fix, kill0, kill2);
            // store side: lane = 4 * filter + piece; the piece's 8 columns, how many of them are outputs.  The last
            // piece of a segment would hold 6 outputs and 2 halo columns: where the whole segment lies inside the image
            // it is moved back by those 2 columns and writes 8 outputs, 2 of them a second time with the same values,
            // so that one full-width store instruction serves every lane instead of a wide and a narrow one.
            const int sp = lane_e & 3, sf = lane_e >> 2;
            int nv, back;
            uint32_t off;
            {
                const int ui = (wave * NT + nt) * UPT + (8 * sp) / SW, col0 = (8 * sp) % SW;
                const int row = k3_div(ui, a.magic_nseg), seg = ui - row * a.nseg;
                const int t = oy0 + row, di = k3_div(t, a.magic_po);
                const int ox_seg = ox0 + seg * VALID;                     // the segment's first output column
                back = (col0 + 8 > VALID && a.w - ox_seg >= VALID) ? col0 + 8 - VALID : 0;
                const int col = col0 - back;
                const int img = oimg0 + di, oy = t - di * a.po, ox = ox_seg + col;
                int lim = a.w - ox;                                       // outputs left in the image row
                if (lim > VALID - col) lim = VALID - col;                 // ... and in the segment
                nv = (v0 + row < a.vrows && oy < a.h) ? (lim > 8 ? 8 : (lim < 0 ? 0 : lim)) : 0;
                off = (uint32_t)(((img * a.c_out + fbi * kMfmaFilters + sf) * a.h + oy) * a.w + ox) * 2u;
            }
#pragma unroll
            for (int mt = 0; mt < 2; ++mt) {
#pragma unroll
                for (int r = 0; r < 16; r += 2) {
                    k3_f2 pr;
#pragma unroll
                    for (int i = 0; i < 2; ++i)
                        pr[i] = acc[0][mt][nt][r + i] + k3_shl1(acc[1][mt][nt][r + i] + k3_shl1(acc[2][mt][nt][r + i]));
                    k3_h2 hv = __builtin_convertvector(pr, k3_h2);                // (filter, filter + 1) of this column, rounded to nearest even
                    hv = __builtin_elementwise_max(hv, floor2);                   // ReLU (or nothing: the floor is then the lowest finite value)
                    const int frow = (r >> 2) * 8 + (r & 3);                      // + kb * 4: the filter's row in the corner
                    *reinterpret_cast<_Float16*>(tb + tb_w + frow * 64) = hv.x;
                    *reinterpret_cast<_Float16*>(tb + tb_w + (frow + 1) * 64) = hv.y;
                }
                // the wavefront's own corner: LDS operations of one wavefront execute in order
#pragma unroll
                for (int j = 0; j < 2; ++j) {
                    // (4-byte aligned; the type may alias the binary16 values written above)
                    const k3_u32_alias* src = reinterpret_cast<const k3_u32_alias*>(tb + tb_r + j * 1024 - 2 * back);
                    k3_u4 w4;
                    w4.x = src[0], w4.y = src[1], w4.z = src[2], w4.w = src[3];
                    const int f = mt * 32 + j * 16 + sf;                  // filter inside the block
                    const bool fok = fbi * kMfmaFilters + f < a.c_out;
                    unsigned char* dst = ybase + (off + (uint32_t)(mt * 32 + j * 16) * fstride);
                    if (__builtin_amdgcn_ballot_w64(fok && wide_ok && nv == 8) != 0) ++stores_behind;
                    if (fok && nv > 0) {
                        if (wide_ok && nv == 8) {
                            *reinterpret_cast<k3_u4*>(dst) = w4;
                        } else if (wide_ok && nv == 6) {
                            k3_u3 w3;
                            w3.x = w4.x, w3.y = w4.y, w3.z = w4.z;
                            *reinterpret_cast<k3_u3*>(dst) = w3;
                        } else {
                            const uint32_t ws[4] = {w4.x, w4.y, w4.z, w4.w};
#pragma unroll
                            for (int e = 0; e < 8; ++e)
                                if (e < nv) *reinterpret_cast<uint16_t*>(dst + 2 * e) = (uint16_t)(ws[e >> 1] >> (16 * (e & 1)));
                        }
                    }
                }
            }
        }
    }
}

typedef void (*k3_launch_fn)(const K3Args& a, int blocks, int lds_bytes, hipStream_t stream);
// The instantiation for a segment width (32 or 16) and a workgroup size (4 or 8 wavefronts); nullptr otherwise.
k3_launch_fn k3_lookup(int sw, int waves, bool split, bool pool);
k3_launch_fn k3_lookup_split(int sw, int waves);
k3_launch_fn k3_lookup_pool(int sw, int waves);

}  // namespace ppc

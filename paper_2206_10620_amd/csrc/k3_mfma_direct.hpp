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
// loaded; their places in LDS are zeroed once per workgroup.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

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
    int32_t vrows;              // n * po - 1
    int32_t tr, nseg;           // tile: rows x segments
    int32_t tiles_x, tiles_v, fb, q;
    int32_t work_items, blocks_per_xcd;
    int32_t chs, ppc, ppcp, nxi, xbuf_bytes;
    // floor(2^32 / d) + 1 for: pieces per channel with padding, pieces per staged row, segments per
    // tile row, rows per image (0 stands for d = 1)
    uint32_t magic_ppcp, magic_ppr, magic_nseg, magic_po;
    int32_t relu;
    int64_t x_elems;            // n * c_in * h * w
};

typedef __fp16 k3_hh4 __attribute__((__vector_size__(4 * sizeof(__fp16))));
typedef _Float16 k3_h4 __attribute__((ext_vector_type(4)));
typedef _Float16 k3_h8 __attribute__((ext_vector_type(8)));
typedef float k3_f16 __attribute__((ext_vector_type(16)));
typedef uint32_t k3_u4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) unsigned char* k3_lds_ptr;

// n / d for n < 65536 and 1 <= d < 65536 with magic = floor(2^32 / d) + 1 (0 stands for d = 1)
__device__ __forceinline__ int k3_div(int n, uint32_t magic) { return magic ? (int)__umulhi((uint32_t)n, magic) : n; }

template <typename P> __device__ __forceinline__ P* k3_uniform_ptr(P* p) {
    const uint64_t v = (uint64_t)(uintptr_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (P*)(uintptr_t)(((uint64_t)hi << 32) | lo);
}

// One direct load: every active lane fetches 16 bytes at base + off into LDS at lds_dst + 16 * lane.
// Inline assembly rather than the compiler builtin: the compiler cannot tell which buffer an
// in-flight direct load fills and would make the first LDS read after it wait for all of them.
__device__ __forceinline__ void k3_dma16(uint32_t off, const void* base, uint32_t lds_dst) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(off), "s"(base), "s"(lds_dst) : "memory", "m0");
}

// lane i <- lane i + 1 over the whole wavefront (the last lane receives 0)
__device__ __forceinline__ float k3_shl1(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x130, 0xf, 0xf, true));
}

template <int SW>
__global__ __launch_bounds__(64 * kK3Waves) __attribute__((amdgpu_waves_per_eu(2, 2)))
void k3_mfma(const K3Args a) {
    constexpr int NT = kK3ColTiles, WAVES = kK3Waves, UPT = 32 / SW, SEGB = SW * 2, PPS = SEGB / 16, VALID = SW - 2;
    constexpr int MAXX = kK3MaxXUnits;
    constexpr int NWU = 18, WU = (NWU + WAVES - 1) / WAVES;
    extern __shared__ __align__(16) unsigned char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // block -> work item, XCD-aware: consecutive block ids go round-robin to the 8 XCDs, so each XCD
    // gets a contiguous range of items (filter block fastest, then tile column, then tile row) and
    // workgroups that read the same or neighbouring input tiles share an L2.
    int item = (int)(blockIdx.x % 8u) * a.blocks_per_xcd + (int)(blockIdx.x / 8u);
    if (item >= a.work_items) return;
    const int fbi = item % a.fb;
    item /= a.fb;
    const int tx = item % a.tiles_x;
    const int tv = item / a.tiles_x;
    const int ox0 = tx * a.nseg * VALID;            // first output column of the tile
    const int v0 = tv * a.tr;                       // first virtual output row
    const int u0 = v0 - 1;                          // virtual input row held by staged row 0
    const int hw = a.h * a.w;
    // image and row inside it of staged row 0 (u0 = -1 belongs to "image -1")
    const int img0 = (u0 + a.po) / a.po - 1, iy0 = u0 - img0 * a.po;
    const int oimg0 = v0 / a.po, oy0 = v0 - oimg0 * a.po;

    const uint32_t lds0 = (uint32_t)(uintptr_t)(k3_lds_ptr)smem;
    const int xb_bytes = a.xbuf_bytes;
    const int rowb = a.nseg * SEGB;                 // LDS bytes per staged row of one channel
    const _Float16* __restrict__ xin = static_cast<const _Float16*>(a.x);

    // ---- staging set-up: which piece each lane fetches in each of this wavefront's instructions ----
    // Instruction `it` fills LDS bytes [1024 it, 1024 it + 1024) of a buffer; piece g = 64 it + lane is
    // piece g % ppcp of channel g / ppcp.  xoff = byte offset of the piece from (chunk base - 16 bytes):
    // the piece that holds input column -1 of a row starts 2 bytes before that row.
    uint32_t xoff[MAXX];
    uint32_t okmask = 0u;                           // bit k: the lane fetches a piece in its k-th instruction
    const int nx = wave < a.nxi ? (a.nxi - wave + WAVES - 1) / WAVES : 0;
#pragma unroll
    for (int k = 0; k < MAXX; ++k) {
        xoff[k] = 16u;
        if (k < nx) {
            const int g = (wave + WAVES * k) * 64 + lane;
            const int ch = k3_div(g, a.magic_ppcp), pr = g - ch * a.ppcp;
            const int srow = k3_div(pr, a.magic_ppr), rem = pr - srow * (a.nseg * PPS);
            const int seg = rem / PPS, piece = rem - seg * PPS;
            const int t = iy0 + srow, di = k3_div(t, a.magic_po);
            const int img = img0 + di, iy = t - di * a.po;
            const int col = ox0 + seg * VALID - 1 + piece * 8;       // input column of the piece's first pixel
            const bool ok = ch < kMfmaChunk && pr < a.ppc && img >= 0 && img < a.n && iy < a.h && col < a.w;
            if (ok) {
                xoff[k] = (uint32_t)(16 + 2 * (((img * a.c_in + ch) * a.h + iy) * a.w + col));
                okmask |= 1u << k;
            } else {
                // a place no load ever writes: zero it in both buffers, once
                *reinterpret_cast<k3_u4*>(smem + (wave + WAVES * k) * 1024 + lane * 16) = k3_u4(0u);
                *reinterpret_cast<k3_u4*>(smem + xb_bytes + (wave + WAVES * k) * 1024 + lane * 16) = k3_u4(0u);
            }
        }
    }

    // Start the loads of chunk qi into buffer `buf`.  Nothing here waits.
    auto issue = [&](int qi, int buf) {
        const int64_t chunk_elem0 = (int64_t)qi * kMfmaChunk * hw;
        const unsigned char* xbase = k3_uniform_ptr(reinterpret_cast<const unsigned char*>(xin + chunk_elem0) - 16);
        const uint32_t ldsx = lds0 + (uint32_t)(buf * xb_bytes);
#pragma unroll
        for (int k = 0; k < MAXX; ++k) {
            if (k < nx) {
                const bool ok = (okmask >> k) & 1u;
                // A piece may reach a few bytes outside the tensor at its two ends (the halo column of the
                // very first row, the columns past the very last row): those lanes assemble their piece
                // from guarded element loads instead.
                const int64_t e0 = chunk_elem0 + ((int64_t)xoff[k] - 16) / 2;
                const bool edge = ok && (e0 < 0 || e0 + 8 > a.x_elems);
                if (ok && !edge) k3_dma16(xoff[k], xbase, ldsx + (uint32_t)((wave + WAVES * k) * 1024));
                if (__builtin_amdgcn_ballot_w64(edge) != 0) {
                    if (edge) {
                        k3_h8 v;
#pragma unroll
                        for (int e = 0; e < 8; ++e) {
                            const int64_t idx = e0 + e;
                            v[e] = (idx >= 0 && idx < a.x_elems) ? xin[idx] : (_Float16)0.0f;
                        }
                        *reinterpret_cast<k3_h8*>(smem + buf * xb_bytes + (wave + WAVES * k) * 1024 + lane * 16) = v;
                    }
                }
            }
        }
        const unsigned char* wbase = k3_uniform_ptr(static_cast<const unsigned char*>(a.wpk) + ((int64_t)fbi * a.q + qi) * kK3WeightBytes);
        const uint32_t ldsw = lds0 + (uint32_t)(2 * xb_bytes + buf * kK3WeightBytes);
#pragma unroll
        for (int k = 0; k < WU; ++k) {
            const int unit = wave + WAVES * k;
            if (unit < NWU) k3_dma16((uint32_t)(unit * 1024 + lane * 16), wbase, ldsw + (uint32_t)(unit * 1024));
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

    // ---- accumulators: three tap columns x two filter halves x NT column tiles ----
    // The bias starts out in the centre column's set (lane halves hold filters 4 apart).
    const int p = lane & 31, kb = lane >> 5;
    k3_f16 acc[3][2][NT];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const float bz = a.bias[fbi * kMfmaFilters + mt * 32 + (r >> 2) * 8 + kb * 4 + (r & 3)];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                acc[0][mt][nt][r] = 0.0f;
                acc[1][mt][nt][r] = bz;
                acc[2][mt][nt][r] = 0.0f;
            }
        }

    // ---- main loop over chunks of 16 channels ----
    issue(0, 0);
    for (int qi = 0; qi < a.q; ++qi) {
        // this wavefront's loads of chunk qi have landed (and its zero fills and edge pieces are written);
        // after the barrier everyone's have, and everyone is done reading the other buffer
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (qi + 1 < a.q) issue(qi + 1, (qi + 1) & 1);

        const uint32_t xb = lds0 + (uint32_t)((qi & 1) * xb_bytes);
        const unsigned char* wb = smem + 2 * xb_bytes + (qi & 1) * kK3WeightBytes + lane * 16;
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            k3_h8 bf[NT];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const uint32_t ad = xb + baddr[nt] + (uint32_t)(r * rowb);
                const k3_hh4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4f16(reinterpret_cast<__attribute__((address_space(3))) k3_hh4*>(ad));
                const k3_hh4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4f16(reinterpret_cast<__attribute__((address_space(3))) k3_hh4*>(ad + (uint32_t)(4 * a.chs)));
                const k3_h4 l4 = __builtin_bit_cast(k3_h4, lo), h4 = __builtin_bit_cast(k3_h4, hi);
                bf[nt] = __builtin_shufflevector(l4, h4, 0, 1, 2, 3, 4, 5, 6, 7);
            }
#pragma unroll
            for (int c = 0; c < 3; ++c) {
                const k3_h8 af0 = *reinterpret_cast<const k3_h8*>(wb + ((r * 3 + c) * 2 + 0) * 1024);
                const k3_h8 af1 = *reinterpret_cast<const k3_h8*>(wb + ((r * 3 + c) * 2 + 1) * 1024);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    acc[c][0][nt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af0, bf[nt], acc[c][0][nt], 0, 0, 0);
                    acc[c][1][nt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af1, bf[nt], acc[c][1][nt], 0, 0, 0);
                }
            }
        }
    }

    // ---- epilogue: combine the three tap columns, ReLU, binary16, store ----
    // An accumulator register holds one filter for the 32 columns of a column tile (lanes 0-31; lanes
    // 32-63 hold the filter four further on).  Output o of a segment sits in lane o: its own P_0, the
    // next lane's P_1, the P_2 two lanes on.
    _Float16* __restrict__ yout = static_cast<_Float16*>(a.y);
    const int64_t fstride = (int64_t)a.h * a.w * 2;              // bytes between filters
    unsigned char* ybase = reinterpret_cast<unsigned char*>(yout);
    const bool whole_block = (fbi + 1) * kMfmaFilters <= a.c_out;
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int ui = (wave * NT + nt) * UPT + p / SW, col = p % SW;
        const int row = k3_div(ui, a.magic_nseg), seg = ui - row * a.nseg;
        const int t = oy0 + row, di = k3_div(t, a.magic_po);
        const int img = oimg0 + di, oy = t - di * a.po, ox = ox0 + seg * VALID + col;
        const bool valid = col < VALID && ox < a.w && v0 + row < a.vrows && oy < a.h;
        // this lane's computed column is input column ox - 1: outside the image for ox = 0 (it would
        // reach output 0 through P_0) and for ox = w + 1 (output w - 1 through P_2)
        const bool kill0 = ox == 0, kill2 = ox == a.w + 1;
        const bool fix = __builtin_amdgcn_ballot_w64(kill0 || kill2) != 0;
        const uint32_t off = (uint32_t)(((img * a.c_out + fbi * kMfmaFilters + kb * 4) * a.h + oy) * a.w + ox) * 2u;
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                float p0 = acc[0][mt][nt][r], p1 = acc[1][mt][nt][r], p2 = acc[2][mt][nt][r];
                if (fix) {
                    p0 = kill0 ? 0.0f : p0;
                    p2 = kill2 ? 0.0f : p2;
                }
                float v = p0 + k3_shl1(p1 + k3_shl1(p2));
                if (a.relu) v = v > 0.0f ? v : 0.0f;
                const int fl = mt * 32 + (r >> 2) * 8 + (r & 3);             // the lower lanes' filter inside the block
                if (valid && (whole_block || fbi * kMfmaFilters + fl + kb * 4 < a.c_out))
                    *reinterpret_cast<_Float16*>(ybase + fl * fstride + off) = (_Float16)v;
            }
    }
}

typedef void (*k3_launch_fn)(const K3Args& a, int blocks, int lds_bytes, hipStream_t stream);
// The instantiation for a segment width (32 or 16); nullptr otherwise.
k3_launch_fn k3_lookup(int sw);

}  // namespace ppc

// Matrix-core kernel for pattern-pruned convolutions stored in binary16 (gfx950).
//
// The measured alternative to pattern-specialised vector code: the pruned weights are written
// out as a dense, zero-filled [c_out][K*K*c_in] matrix and the layer is computed as an implicit
// GEMM on the MFMA units (v_mfma_f32_32x32x16_f16, fp32 accumulation).  A 4-of-9 pattern at 28-40 %
// connectivity keeps 12-18 % of the weights, so the dense product does 5.6-8 times the
// multiply-accumulates of the sparse one -- at more than 30 times the rate of the vector ALUs.
// It takes any pattern table, kernel size (1, 3, 5, 7) and stride (1, 2), and folds bias, ReLU and
// an optional 2x2 max-pool into its epilogue.
//
// Mapping.  A workgroup is four or eight wavefronts and computes 64 filters (two 32-row MFMA tiles)
// for a TR x TC tile of output pixels of the batch laid out as one tall virtual image; each
// wavefront owns NTW 32-pixel column tiles of it for all 64 filters (2 x NTW accumulator tiles of 16
// registers).  The reduction runs over chunks of 16 input channels; per chunk the input tile
// (with its halo) and the chunk's weight fragments are staged in LDS, double buffered, one barrier
// per chunk:
//   * input: NCHW in memory, but the MFMA "B" operand wants, per lane, 8 consecutive reduction
//     indices of one pixel.  The tile is therefore staged channel-innermost ([pixel][16 channels],
//     48 bytes per pixel: the 16 bytes of padding spread consecutive pixels over the banks), so that
//     a lane's operand is one 128-bit read at (its pixel + the tap's offset).  The transposition
//     happens on the way in: a lane loads two adjacent pixels of two channels (one aligned 32-bit
//     word per channel), swaps halves in registers and writes one 32-bit word per pixel.
//   * weights: stored by the plan as the "A" operand fragments themselves (1 KB each: 64 lanes x
//     8 halves), copied to LDS and read back with one 128-bit read per lane.
// The epilogue adds the bias, applies ReLU, rounds to binary16 and passes the tile through LDS so
// that the stores to the NCHW output are whole 16-byte groups along a row (and so that the 2x2
// max-pool, when fused, finds its four inputs).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mfma_geom.hpp"

namespace ppc {

struct K2Args {
    const void* x;
    void* y;
    const void* wpk;            // weight fragments [fb][q][K*K][2][64][8] binary16
    const float* bias;          // [fb*64]
    int32_t n, c_in, c_out, h, w;
    int32_t ho, wo;             // the convolution's output size
    int32_t out_h, out_w;       // size of y per image (pooled if pool)
    int32_t po;                 // virtual rows per image
    int32_t vrows;              // rows of the tall virtual output image: (n-1)*po + ho
    int32_t tr, tc;             // tile
    int32_t trp, twpa;          // staged input rows per tile; staged columns per row (even: whole pairs)
    int32_t tiles_x, tiles_v;   // ceil(wo / tc), ceil(vrows / tr)
    int32_t fb, q;
    int32_t work_items, blocks_per_xcd;
    int32_t xbuf_bytes, out_pitch, gw;
    int32_t bias_off;           // byte offset in dynamic LDS of the workgroup's 64 bias values
    int32_t stride_;            // the layer's stride (the kernel's S)
    // floor(2^32 / d) + 1 for the divisors of the index arithmetic (0 stands for d = 1): staged pairs per
    // row, virtual input rows per image, tile columns, virtual output rows per image, store groups per
    // tile row, tile rows (the last two of the pooled tile when a pool is fused)
    uint32_t magic_ppr, magic_pi, magic_tc, magic_po, magic_gpr, magic_srows;
    int32_t relu, pool;
};

typedef _Float16 k2_h8 __attribute__((ext_vector_type(8)));
typedef _Float16 k2_h4 __attribute__((ext_vector_type(4)));
typedef _Float16 k2_h2 __attribute__((ext_vector_type(2)));
typedef float k2_f16 __attribute__((ext_vector_type(16)));
typedef uint32_t k2_u4 __attribute__((ext_vector_type(4)));

// n / d for n < 65536 and 1 <= d < 65536 with magic = floor(2^32 / d) + 1 (0 stands for d = 1)
__device__ __forceinline__ int k2_div(int n, uint32_t magic) { return magic ? (int)__umulhi((uint32_t)n, magic) : n; }

// Input staging.  The staged tile is addressed in pairs of horizontally adjacent pixels that start
// on an even input column, so that (for even image widths) a pair of one channel is one aligned
// 32-bit word in memory.  One wavefront instruction covers 16 consecutive pairs of a tile row for
// 4 channel pairs (lane = 16 * channel pair + pair): 64 contiguous bytes per channel from memory, and,
// on the LDS side, 64 different banks: a staged pixel is 12 banks long, so 16 consecutive pixels
// start on the 16 different multiples of 4 and the 4 channel pairs fill the banks in between.  Each
// lane holds two pixels; lanes 0-7 of every 16 write their first pixel in the first store and the
// others their second, which gives both stores one pixel of every residue mod 16.
// A wavefront's units: channel-pair group (wave & 1) of the chunk, pair groups (wave >> 1) + (WAVES/2) * i.
//
// Everything that does not change from chunk to chunk is worked out once: the byte offset of each
// pair from the chunk's first channel (so that a load is "scalar base + 32-bit lane offset" with no
// address arithmetic), the two LDS addresses, the byte selectors of the two half-swaps.  Tiles that
// lie inside the images and chunks of 16 whole channels -- almost all -- take a path with no
// per-lane tests at all.
template <int WAVES, bool PAIRS, int MAXI>
struct K2Stager {
    static constexpr int kMaxI = MAXI;
    static constexpr int CS = kMfmaPixelBytes;
    uint32_t voff[kMaxI];           // byte offset of the pair's first pixel from channel 0 of the chunk (a valid place even if the pair is outside the images)
    uint32_t voff1[PAIRS ? 1 : kMaxI];   // odd image widths: the second pixel's, separately
    uint32_t r0[kMaxI], r1[kMaxI];  // even and odd channel of the lane's channel pair: (pixel 0, pixel 1) each
    uint32_t inside, inside1;       // bit i: the pair (odd widths: its first / second pixel) of unit i lies inside the images
    int ni;                         // units of this wavefront
    int chan;                       // first channel of the lane's pair inside a chunk
    int dst_a, dst_b;               // LDS byte offsets, inside a buffer, of the pixel written first / second in unit 0
    uint32_t sel_a, sel_b;          // v_perm selectors that build the word written first / second
    bool all_inside;                // wave-uniform: no unit of this wavefront touches a place outside the images

    __device__ __forceinline__ void setup(const K2Args& a, int wave, int lane, int img0, int iy0, int ixa, int hw) {
        const int ppr = a.twpa >> 1, npairs = a.trp * ppr;
        const int npg = (npairs + 15) >> 4;
        const int pg0 = wave >> 1;
        ni = pg0 < npg ? (npg - pg0 + WAVES / 2 - 1) / (WAVES / 2) : 0;
        const int pp = lane & 15, cpi = lane >> 4;
        chan = ((wave & 1) * 4 + cpi) * 2;
        const bool swap = (lane & 8) != 0;
        const int first = (pg0 * 16 + pp) * 2 * CS + chan * 2;
        dst_a = first + (swap ? CS : 0);
        dst_b = first + (swap ? 0 : CS);
        sel_a = swap ? 0x07060302u : 0x05040100u;      // pixel 1 / pixel 0 of (even channel, odd channel)
        sel_b = swap ? 0x05040100u : 0x07060302u;
        const uint32_t chan_bytes = (uint32_t)(chan < a.c_in ? chan : 0) * (uint32_t)hw * 2u;
        inside = inside1 = 0u;
        bool ok_all = true;
#pragma unroll
        for (int i = 0; i < kMaxI; ++i) {
            voff[i] = chan_bytes;
            if constexpr (!PAIRS) voff1[i] = chan_bytes;
            if (i < ni) {
                const int ps = (pg0 + (WAVES / 2) * i) * 16 + pp;
                const int row = k2_div(ps, a.magic_ppr), pc = ps - row * ppr;
                const int t = iy0 + row;                               // rows below the first staged row's image start
                const int di = k2_div(t, a.magic_pi);
                const int img = img0 + di, iy = t - di * (a.po * a.stride_), ix = ixa + 2 * pc;
                const bool row_ok = ps < npairs && img >= 0 && img < a.n && iy < a.h;
                const uint32_t base = (uint32_t)((img * a.c_in * a.h + iy) * a.w + ix) * 2u + chan_bytes;
                const bool ok0 = row_ok && ix >= 0 && ix < a.w;
                if (ok0) {
                    voff[i] = base;
                    inside |= 1u << i;
                }
                if constexpr (!PAIRS) {
                    const bool ok1 = row_ok && ix + 1 >= 0 && ix + 1 < a.w;
                    if (ok1) {
                        voff1[i] = base + 2u;
                        inside1 |= 1u << i;
                    }
                    ok_all = ok_all && (ok1 || ps >= npairs);
                }
                ok_all = ok_all && (ok0 || ps >= npairs);
            }
        }
        all_inside = __builtin_amdgcn_ballot_w64(!ok_all) == 0;
    }
    // issue the loads of chunk q (nothing here waits for them)
    __device__ __forceinline__ void load(const K2Args& a, const _Float16* __restrict__ xin, int q, int hw) {
        // a chunk that reaches past the last channel: lanes of absent channels read channel 0 of the
        // chunk instead (their values are dropped when stored)
        const unsigned char* base0 = reinterpret_cast<const unsigned char*>(xin + (int64_t)q * kMfmaChunk * hw);
        const int left = a.c_in - q * kMfmaChunk;
        if (left >= kMfmaChunk) {
            const unsigned char* base1 = base0 + 2 * (int64_t)hw;
#pragma unroll
            for (int i = 0; i < kMaxI; ++i) {
                if (i < ni) {
                    if constexpr (PAIRS) {
                        r0[i] = *reinterpret_cast<const uint32_t*>(base0 + voff[i]);
                        r1[i] = *reinterpret_cast<const uint32_t*>(base1 + voff[i]);
                    } else {
                        const uint32_t a0 = *reinterpret_cast<const uint16_t*>(base0 + voff[i]), a1 = *reinterpret_cast<const uint16_t*>(base0 + voff1[i]);
                        const uint32_t b0 = *reinterpret_cast<const uint16_t*>(base1 + voff[i]), b1 = *reinterpret_cast<const uint16_t*>(base1 + voff1[i]);
                        r0[i] = a0 | (a1 << 16);
                        r1[i] = b0 | (b1 << 16);
                    }
                }
            }
        } else {
            const uint32_t back = chan < left ? 0u : (uint32_t)(chan < a.c_in ? chan : 0) * (uint32_t)hw * 2u;
            const uint32_t fwd = chan + 1 < left ? 2u * (uint32_t)hw : 0u;
#pragma unroll
            for (int i = 0; i < kMaxI; ++i) {
                if (i < ni) {
                    if constexpr (PAIRS) {
                        r0[i] = *reinterpret_cast<const uint32_t*>(base0 + (voff[i] - back));
                        r1[i] = *reinterpret_cast<const uint32_t*>(base0 + (voff[i] - back + fwd));
                    } else {
                        const uint32_t a0 = *reinterpret_cast<const uint16_t*>(base0 + (voff[i] - back)), a1 = *reinterpret_cast<const uint16_t*>(base0 + (voff1[i] - back));
                        const uint32_t b0 = *reinterpret_cast<const uint16_t*>(base0 + (voff[i] - back + fwd)), b1 = *reinterpret_cast<const uint16_t*>(base0 + (voff1[i] - back + fwd));
                        r0[i] = a0 | (a1 << 16);
                        r1[i] = b0 | (b1 << 16);
                    }
                }
            }
        }
    }
    // transpose in registers and write chunk q's words into the buffer at xb
    __device__ __forceinline__ void store(const K2Args& a, unsigned char* xb, int q) {
        const int left = a.c_in - q * kMfmaChunk;
        if (all_inside && left >= kMfmaChunk) {
#pragma unroll
            for (int i = 0; i < kMaxI; ++i) {
                if (i < ni) {
                    const int step = i * (WAVES / 2) * 16 * 2 * CS;
                    *reinterpret_cast<uint32_t*>(xb + dst_a + step) = __builtin_amdgcn_perm(r1[i], r0[i], sel_a);
                    *reinterpret_cast<uint32_t*>(xb + dst_b + step) = __builtin_amdgcn_perm(r1[i], r0[i], sel_b);
                }
            }
        } else {
            const bool has0 = chan < left, has1 = chan + 1 < left;
#pragma unroll
            for (int i = 0; i < kMaxI; ++i) {
                if (i < ni) {
                    uint32_t e = r0[i], o = r1[i];
                    if constexpr (PAIRS) {
                        if (!((inside >> i) & 1u)) e = o = 0u;
                    } else {
                        if (!((inside >> i) & 1u)) {
                            e &= 0xFFFF0000u;
                            o &= 0xFFFF0000u;
                        }
                        if (!((inside1 >> i) & 1u)) {
                            e &= 0x0000FFFFu;
                            o &= 0x0000FFFFu;
                        }
                    }
                    if (!has0) e = 0u;
                    if (!has1) o = 0u;
                    const int step = i * (WAVES / 2) * 16 * 2 * CS;
                    *reinterpret_cast<uint32_t*>(xb + dst_a + step) = __builtin_amdgcn_perm(o, e, sel_a);
                    *reinterpret_cast<uint32_t*>(xb + dst_b + step) = __builtin_amdgcn_perm(o, e, sel_b);
                }
            }
        }
    }
};

// Four-wavefront workgroups with two column tiles per wavefront are meant to run two to a compute unit:
// they are asked to fit 256 vector registers.
template <int KS, int S, int NTW, int WAVES, bool PAIRS>
__global__ __launch_bounds__(64 * WAVES) __attribute__((amdgpu_waves_per_eu(NTW == 2 ? 2 : 1)))
void k2_mfma(const K2Args a) {
    constexpr int KK = KS * KS;
    constexpr int UPQ = KS <= 3 ? 1 : KS;           // weight units per channel chunk
    constexpr int TPU = KK / UPQ;                   // taps per unit
    constexpr int NFU = TPU * 2;                    // weight fragments per unit
    constexpr int MAXF = (NFU + WAVES - 1) / WAVES; // fragments a wavefront copies per unit
    constexpr int CS = kMfmaPixelBytes;
    constexpr int PAD = KS / 2;
    constexpr int NT = 64 * WAVES;
    extern __shared__ __align__(16) unsigned char smem[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // block -> work item, XCD-aware: consecutive block ids go round-robin to the 8 XCDs, so each XCD
    // gets a contiguous range of items; items are ordered filter block fastest, then tile column, then
    // tile row, so workgroups that read the same input tile or neighbouring ones share an L2.
    int item = (int)(blockIdx.x % 8u) * a.blocks_per_xcd + (int)(blockIdx.x / 8u);
    if (item >= a.work_items) return;
    const int fbi = item % a.fb;
    item /= a.fb;
    const int tx = item % a.tiles_x;
    const int tv = item / a.tiles_x;
    const int ox0 = tx * a.tc;
    const int v0 = tv * a.tr;                       // first virtual output row of the tile
    const int u0 = v0 * S - PAD;                    // virtual input row held by staged row 0
    const int ix0 = ox0 * S - PAD;                  // input column of the tile's first tap
    const int ixa = ix0 & ~1;                       // staged column 0: the even column at or before it
    const int pi = a.po * S;                        // virtual input rows per image
    const int hw = a.h * a.w;
    // image and row inside it of staged row 0 and of the tile's first output row (wave-uniform: the
    // divisions are scalar code, once per workgroup; everything per lane divides by multiplication)
    const int img0 = (u0 + pi) / pi - 1, iy0 = u0 - img0 * pi;
    const int oimg0 = v0 / a.po, oy0 = v0 - oimg0 * a.po;

    unsigned char* xbuf0 = smem;
    unsigned char* wbuf0 = smem + 2 * a.xbuf_bytes;
    constexpr int wbuf_bytes = NFU * 1024;

    K2Stager<WAVES, PAIRS, mfma_max_units(WAVES, NTW)> st;
    st.setup(a, wave, lane, img0, iy0, ixa, hw);
    const _Float16* __restrict__ xin = static_cast<const _Float16*>(a.x);
    const k2_u4* __restrict__ wsrc = reinterpret_cast<const k2_u4*>(a.wpk) + (size_t)fbi * a.q * KK * 2 * 64;

    // ---- per-lane operand addresses: pixel slot of lane p in column tile nt ----
    const int p = lane & 31, kb = lane >> 5;
    int bbase[NTW];
#pragma unroll
    for (int nt = 0; nt < NTW; ++nt) {
        int slot = (wave * NTW + nt) * 32 + p;
        if (slot >= a.tr * a.tc) slot = 0;          // idle lanes read a valid place; their results are dropped
        const int vr = k2_div(slot, a.magic_tc), px = slot - vr * a.tc;
        bbase[nt] = ((vr * S) * a.twpa + px * S + (ix0 - ixa)) * CS + kb * 16;
    }

    k2_f16 acc[2][NTW];
#pragma unroll
    for (int mt = 0; mt < 2; ++mt)
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mt][nt][r] = 0.0f;

    k2_u4 wr[MAXF];
    auto load_w = [&](int unit) {
        const k2_u4* src = wsrc + (size_t)unit * NFU * 64 + lane;
#pragma unroll
        for (int f = 0; f < MAXF; ++f)
            if (wave + WAVES * f < NFU) wr[f] = src[(wave + WAVES * f) * 64];
    };
    auto store_w = [&](int buf) {
        unsigned char* dst = wbuf0 + buf * wbuf_bytes + lane * 16;
#pragma unroll
        for (int f = 0; f < MAXF; ++f)
            if (wave + WAVES * f < NFU) *reinterpret_cast<k2_u4*>(dst + (wave + WAVES * f) * 1024) = wr[f];
    };

    // the workgroup's bias values wait in LDS for the epilogue
    float* bias_lds = reinterpret_cast<float*>(smem + a.bias_off);
    if (tid < kMfmaFilters) bias_lds[tid] = a.bias[fbi * kMfmaFilters + tid];

    // ---- main loop over (chunk, unit) ----
    const int units = a.q * UPQ;
    st.load(a, xin, 0, hw);
    load_w(0);
    st.store(a, xbuf0, 0);
    store_w(0);
    // vmcnt(0), as the builtin so that the compiler's own wait-count bookkeeping sees it: every staging
    // load has been consumed by now, but the loads and their stores sit under separate (identical)
    // conditions, and along the path that takes the one and skips the other -- which never runs -- the
    // loads look outstanding; without this the compiler makes the next round of loads wait for one
    // another.
    __builtin_amdgcn_s_waitcnt(0x0F70);
    __syncthreads();
    for (int u = 0; u < units; ++u) {
        const int q = u / UPQ, ur = u - q * UPQ;
        const bool more = u + 1 < units;
        const bool next_x = more && ur == UPQ - 1;      // the next unit starts a new chunk
        if (next_x) st.load(a, xin, q + 1, hw);
        if (more) load_w(u + 1);

        const unsigned char* xb = xbuf0 + (q & 1) * a.xbuf_bytes;
        const unsigned char* wb = wbuf0 + (u & 1) * wbuf_bytes + lane * 16;
        // Operand fragments are read one tap ahead into a second set of registers, so that the LDS
        // latency of tap t+1 hides behind the eight (or four) MFMAs of tap t.
        k2_h8 af[2][2], bf[2][NTW];
        auto read_tap = [&](int set, int t) {
            const int r = UPQ == 1 ? t / KS : ur, c = UPQ == 1 ? t % KS : t;
            const int tapoff = (r * a.twpa + c) * CS;
            af[set][0] = *reinterpret_cast<const k2_h8*>(wb + (t * 2 + 0) * 1024);
            af[set][1] = *reinterpret_cast<const k2_h8*>(wb + (t * 2 + 1) * 1024);
#pragma unroll
            for (int nt = 0; nt < NTW; ++nt) bf[set][nt] = *reinterpret_cast<const k2_h8*>(xb + bbase[nt] + tapoff);
        };
        read_tap(0, 0);
#pragma unroll
        for (int t = 0; t < TPU; ++t) {
            if (t + 1 < TPU) read_tap((t + 1) & 1, t + 1);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int nt = 0; nt < NTW; ++nt) {
                acc[0][nt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[t & 1][0], bf[t & 1][nt], acc[0][nt], 0, 0, 0);
                acc[1][nt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[t & 1][1], bf[t & 1][nt], acc[1][nt], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
        if (next_x) st.store(a, xbuf0 + ((q + 1) & 1) * a.xbuf_bytes, q + 1);
        if (more) store_w((u + 1) & 1);
        __builtin_amdgcn_s_waitcnt(0x0F70);
        __syncthreads();
    }

    // ---- epilogue: bias, ReLU, binary16 ----
    _Float16* __restrict__ yout = static_cast<_Float16*>(a.y);
    if (!a.pool) {
        // Straight from the accumulators: an MFMA result register holds one filter for 32 consecutive
        // pixel slots (lanes 0-31; lanes 32-63 hold the filter four further on), so one store
        // instruction writes two runs of 64 bytes, and the neighbouring column tile of the same
        // wavefront completes the 128-byte lines a few instructions later.  The filter term of the
        // address is wave-uniform and goes into the scalar base; everything per lane (image, row,
        // column, the +4 filters of the upper lanes) is one 32-bit offset per column tile.
        const int64_t fstride = (int64_t)a.ho * a.wo * 2;        // bytes between filters
        unsigned char* ybase = reinterpret_cast<unsigned char*>(yout);
        const bool whole_block = (fbi + 1) * kMfmaFilters <= a.c_out;
#pragma unroll
        for (int nt = 0; nt < NTW; ++nt) {
            const int slot = (wave * NTW + nt) * 32 + p;
            const int vr = k2_div(slot, a.magic_tc), px = slot - vr * a.tc;
            const int t = oy0 + vr, di = k2_div(t, a.magic_po);
            const int img = oimg0 + di, oy = t - di * a.po, ox = ox0 + px;
            const bool valid = slot < a.tr * a.tc && img < a.n && oy < a.ho && ox < a.wo;
            const uint32_t off = (uint32_t)(((img * a.c_out + fbi * kMfmaFilters + kb * 4) * a.ho + oy) * a.wo + ox) * 2u;
            if (valid) {
#pragma unroll
                for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int fl = mt * 32 + (r >> 2) * 8 + (r & 3);     // the lower lanes' filter inside the block
                        float v = acc[mt][nt][r] + bias_lds[fl + kb * 4];
                        if (a.relu) v = v > 0.0f ? v : 0.0f;
                        if (whole_block || fbi * kMfmaFilters + fl + kb * 4 < a.c_out)
                            *reinterpret_cast<_Float16*>(ybase + fl * fstride + off) = (_Float16)v;
                    }
            }
        }
    } else {
        // With a fused 2x2 max-pool the tile goes through LDS as [filter][pixel slot], so that the four
        // inputs of a pooled pixel, which sit in different lanes and column tiles, meet.  Tile rows and
        // columns are even and tiles start on even rows and columns.
        _Float16* ot = reinterpret_cast<_Float16*>(smem);
        const int op = a.out_pitch;
#pragma unroll
        for (int mt = 0; mt < 2; ++mt)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int f = mt * 32 + (r >> 2) * 8 + kb * 4 + (r & 3);
                const float bz = bias_lds[f];
#pragma unroll
                for (int nt = 0; nt < NTW; ++nt) {
                    const int slot = (wave * NTW + nt) * 32 + p;
                    float v = acc[mt][nt][r] + bz;
                    if (a.relu) v = v > 0.0f ? v : 0.0f;
                    if (slot < op) ot[f * op + slot] = (_Float16)v;
                }
            }
        __syncthreads();
        const int gw = a.gw;
        const int ptc = a.tc / 2, prows = a.tr / 2;
        const int gpr = ptc / gw;
        const int total = kMfmaFilters * prows * gpr;
        for (int g = tid; g < total; g += NT) {
            const int rest = k2_div(g, a.magic_gpr), cg = g - rest * gpr;
            const int f = k2_div(rest, a.magic_srows), prow = rest - f * prows;
            const int co = fbi * kMfmaFilters + f;
            const int ox = ox0 + 2 * cg * gw;
            const int t = oy0 + 2 * prow, di = k2_div(t, a.magic_po);
            const int img = oimg0 + di, oy = t - di * a.po;
            if (co >= a.c_out || img >= a.n || oy >= a.ho || ox >= a.wo) continue;
            const _Float16* src = ot + f * op + (2 * prow) * a.tc + 2 * cg * gw;
            _Float16* dst = yout + (((int64_t)img * a.c_out + co) * a.out_h + (oy >> 1)) * a.out_w + (ox >> 1);
            for (int k = 0; k < gw; ++k) {
                const _Float16 m0 = src[2 * k] > src[2 * k + 1] ? src[2 * k] : src[2 * k + 1];
                const _Float16 m1 = src[a.tc + 2 * k] > src[a.tc + 2 * k + 1] ? src[a.tc + 2 * k] : src[a.tc + 2 * k + 1];
                dst[k] = m0 > m1 ? m0 : m1;
            }
        }
    }
}

typedef void (*k2_launch_fn)(const K2Args& a, int blocks, int threads, int lds_bytes, hipStream_t stream);
// The instantiation for (kernel size, stride, column tiles per wavefront, wavefronts per workgroup,
// aligned-pair staging); nullptr if not built.
k2_launch_fn k2_lookup(int ks, int stride, int ntw, int waves, bool pairs);

}  // namespace ppc

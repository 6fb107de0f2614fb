// Tiled, pattern-specialised kernel for the pattern-pruned 3x3 convolution on gfx950.
//
// Mapping (chosen for 64-wide wavefronts, not the thread-per-filter mapping the paper uses on
// mobile CPUs/GPUs in its filter-kernel-reorder figure of section 2.3.1):
//   * lanes own output pixels: a lane holds an R x 4 micro-tile of adjacent pixels for each of
//     the F filters of its wavefront (F*R*4 fp32 accumulators);
//   * a wavefront therefore sees every weight, pattern and loop bound as a wave-uniform value:
//     they live in scalar registers, are fetched with scalar loads from the packed weight
//     stream, and every sparsity-dependent branch is a scalar branch -- no lane divergence;
//   * a workgroup is WF x KS wavefronts that share one LDS-resident input tile (the tiling of
//     the input in section 2.3.1): WF of them work on different filter groups, KS of them split the input
//     channels of each chunk and are summed through LDS at the end in a fixed order.
//
// Input tiles reach LDS without passing through registers where the shape allows it: gfx950's
// direct global-to-LDS loads write 64 consecutive 16-byte (or 4-byte) slots per wavefront
// instruction, asynchronously, so the tile of the next channel chunk is in flight into a second
// buffer while the current chunk is consumed, at no cost in registers.
//
// Per input channel a lane reads its (R+2) x 6 input window from LDS once, with one 128-bit
// (fp32) or 64-bit (fp16) read for the four interior columns and one 64-bit read for the
// (left, right) halo pair per row, and reuses it from registers for every kernel of the
// wavefront's filters that keeps that channel.  The multiply-accumulates of one kernel are a
// straight-line block specialised on (filter slot, pattern): all register indices are static
// (a pattern fixes its data accesses when the code is generated: section 2.3.1 on load
// redundancy elimination).
//
// The batch is laid out as one tall virtual image: image n, row y is virtual row n*(H+1)+y and
// row y = H of every image is a shared zero row, so that tiles may straddle images.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "tile_geom.hpp"

namespace ppc {

struct K1Args {
    const void* x;
    void* y;
    const uint32_t* stream;     // weight-stream entries
    const int32_t* wave_off;    // [G*KS] first entry per (group, split)
    int32_t idle_off;           // first entry of a run of end-of-chunk entries, for wavefronts without a filter group
    const float* bias_pad;      // [G*F]
    const int32_t* chan_map;    // [filter blocks][chunks*cc] input channel at each place of each chunk
    const int32_t* perm_pad;    // [G*F] original filter index or -1
    int32_t n, c_in, c_out, h, w;
    int32_t vh;                 // virtual output rows: n*(h+1)-1
    int32_t mrows;              // micro-rows: ceil(vh / R)
    int32_t wg_per_strip;       // ceil(mrows*LW / 64)
    int32_t strips;             // ceil(w / (4*LW))
    int32_t nfb;                // filter blocks: ceil(G / WF)
    int32_t work_items;         // strips * wg_per_strip * nfb
    int32_t blocks_per_xcd;     // ceil(work_items / 8); the grid has 8 * blocks_per_xcd blocks
    int32_t groups;             // G
    int32_t wf, ks, cc, chunks;
    int32_t wf_recip;           // 65536 / wf + 1: (wave * wf_recip) >> 16 == wave / wf for wave < 16
    int32_t red_par;            // channel splits whose partial sums fit in LDS side by side (1 .. ks-1)
    int32_t vec;                // register staging: vector width in elements
    int32_t mode;               // 0: staging through registers; 1: direct-to-LDS loads, 16-byte slots; 2: 4-byte slots
    int32_t nbuf;               // direct modes: tile buffers in the ring (2..8)
    int32_t table_offset;       // direct modes: byte offset of the slot tables in dynamic LDS (after the tile buffers; multiple of 16)
    int32_t relu;
    // channel split across workgroups: slice s of split_wg takes chunks [s*chunks/split_wg, (s+1)*chunks/split_wg)
    int32_t split_wg;
    int32_t out_elems;          // n*c_out*h*w: elements of one partial-sum plane in ws
    float* ws;                  // [split_wg][n][c_out][h][w] partial sums (split_wg > 1)
    int32_t* counters;          // [work_items / split_wg] arrivals per output tile; zero between launches
};

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef const __attribute__((address_space(3))) unsigned char* lds_cbyte_ptr;   // a byte address in LDS

template <typename T, int N> struct VecOf;
template <> struct VecOf<float, 1> { typedef float type; };
template <> struct VecOf<float, 2> { typedef f32x2 type; };
template <> struct VecOf<float, 4> { typedef f32x4 type; };
template <> struct VecOf<_Float16, 1> { typedef _Float16 type; };
template <> struct VecOf<_Float16, 2> { typedef f16x2 type; };
template <> struct VecOf<_Float16, 4> { typedef f16x4 type; };
template <> struct VecOf<_Float16, 8> { typedef _Float16 type __attribute__((ext_vector_type(8))); };

template <typename T, int N> __device__ __forceinline__ T vec_elem(const typename VecOf<T, N>::type& v, int i) {
    if constexpr (N == 1) return v;
    else return v[i];
}

// A lane's input window for one channel: rows 0..R+1, columns -1..4, and the multiply-accumulate
// of one of its elements with a wave-uniform weight.  LDS holds, per tile row, the interior
// columns and, separately, one (left, right) pair of 32-bit words per micro-column: for fp32 the
// two neighbour elements themselves, for fp16 the words (x[-2], x[-1]) and (x[4], x[5]).
template <typename T, int R> struct Window;

// The four weights of a kernel as they sit in scalar registers: fp32 values, or for fp16 storage
// two words of two binary16 values each (w0 | w1 << 16, w2 | w3 << 16).
template <typename T> struct Weights;
template <> struct Weights<float> { float w[4]; };
template <> struct Weights<_Float16> { uint32_t pair[2]; };

template <int R> struct Window<float, R> {
    f32x4 mid[R + 2];    // columns 0..3
    f32x2 halo[R + 2];   // (column -1, column 4)
    __device__ __forceinline__ void clear() {
#pragma unroll
        for (int rr = 0; rr < R + 2; ++rr) {
            mid[rr] = f32x4(0);
            halo[rr] = f32x2(0);
        }
    }
    // pm, ph: LDS addresses of the lane's first interior element and first halo pair; strides in bytes
    __device__ __forceinline__ void load(lds_cbyte_ptr pm, lds_cbyte_ptr ph, int rs_bytes, int hrs_bytes) {
#pragma unroll
        for (int rr = 0; rr < R + 2; ++rr) {
            mid[rr] = *reinterpret_cast<const __attribute__((address_space(3))) f32x4*>(pm + rr * rs_bytes);
            halo[rr] = *reinterpret_cast<const __attribute__((address_space(3))) f32x2*>(ph + rr * hrs_bytes);
        }
    }
    template <int ROW, int COL, int J> __device__ __forceinline__ void fma(float& acc, const Weights<float>& wt) const {
        const float w = wt.w[J];
        if constexpr (COL < 0) acc = __builtin_fmaf(w, halo[ROW][0], acc);
        else if constexpr (COL > 3) acc = __builtin_fmaf(w, halo[ROW][1], acc);
        else acc = __builtin_fmaf(w, mid[ROW][COL], acc);
    }
};

// fp16 storage: the window stays packed, two halves per register, and every multiply-accumulate
// is one v_fma_mix_f32: fp16 weight from the low or high half of a scalar register, fp16 input
// from the low or high half of a vector register, both widened exactly, fp32 accumulator.  Written
// as inline assembly because the compiler otherwise unpacks halves that are used several times
// with extra conversion instructions.
template <int R> struct Window<_Float16, R> {
    uint32_t mid[R + 2][2];    // columns (0,1), (2,3)
    uint32_t halo[R + 2][2];   // (column -2, column -1), (column 4, column 5)
    __device__ __forceinline__ void clear() {
#pragma unroll
        for (int rr = 0; rr < R + 2; ++rr) mid[rr][0] = mid[rr][1] = halo[rr][0] = halo[rr][1] = 0u;
    }
    __device__ __forceinline__ void load(lds_cbyte_ptr pm, lds_cbyte_ptr ph, int rs_bytes, int hrs_bytes) {
        typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
#pragma unroll
        for (int rr = 0; rr < R + 2; ++rr) {
            const u32x2 m = *reinterpret_cast<const __attribute__((address_space(3))) u32x2*>(pm + rr * rs_bytes);
            const u32x2 h = *reinterpret_cast<const __attribute__((address_space(3))) u32x2*>(ph + rr * hrs_bytes);
            mid[rr][0] = m[0];
            mid[rr][1] = m[1];
            halo[rr][0] = h[0];
            halo[rr][1] = h[1];
        }
    }
    template <int ROW, int COL, int J> __device__ __forceinline__ void fma(float& acc, const Weights<_Float16>& wt) const {
        constexpr bool hi = (COL < 0) ? true : (COL > 3) ? false : (COL & 1) != 0;
        const uint32_t src = (COL < 0) ? halo[ROW][0] : (COL > 3) ? halo[ROW][1] : mid[ROW][(COL < 0 ? 0 : COL) >> 1];
        const uint32_t w = wt.pair[J >> 1];
        // op_sel_hi = 1: the operand is fp16; op_sel: which half of it
        if constexpr (hi && (J & 1))
            asm("v_fma_mix_f32 %0, %1, %2, %0 op_sel:[1,1,0] op_sel_hi:[1,1,0]" : "+v"(acc) : "s"(w), "v"(src));
        else if constexpr (hi)
            asm("v_fma_mix_f32 %0, %1, %2, %0 op_sel:[0,1,0] op_sel_hi:[1,1,0]" : "+v"(acc) : "s"(w), "v"(src));
        else if constexpr (J & 1)
            asm("v_fma_mix_f32 %0, %1, %2, %0 op_sel:[1,0,0] op_sel_hi:[1,1,0]" : "+v"(acc) : "s"(w), "v"(src));
        else
            asm("v_fma_mix_f32 %0, %1, %2, %0 op_sel_hi:[1,1,0]" : "+v"(acc) : "s"(w), "v"(src));
    }
};

// ---------------------------------------------------------------------------------------------
// Multiply-accumulate block of one kept kernel: filter slot FS, pattern slot PS (4 taps).
template <typename T, int R, int F, int FS, int RR, int TAP, int J>
__device__ __forceinline__ void mac_row(float (&acc)[F][R][4], const Window<T, R>& win, const Weights<T>& wt) {
    constexpr int dr = TAP / 3, dc = TAP % 3 - 1;
    win.template fma<RR + dr, 0 + dc, J>(acc[FS][RR][0], wt);
    win.template fma<RR + dr, 1 + dc, J>(acc[FS][RR][1], wt);
    win.template fma<RR + dr, 2 + dc, J>(acc[FS][RR][2], wt);
    win.template fma<RR + dr, 3 + dc, J>(acc[FS][RR][3], wt);
}

template <typename T, int R, int F, int FS, int TAP, int J, int RR = 0>
__device__ __forceinline__ void mac_tap(float (&acc)[F][R][4], const Window<T, R>& win, const Weights<T>& wt) {
    if constexpr (RR < R) {
        mac_row<T, R, F, FS, RR, TAP, J>(acc, win, wt);
        mac_tap<T, R, F, FS, TAP, J, RR + 1>(acc, win, wt);
    }
}

constexpr int nth_tap(uint32_t mask, int j) {
    for (int t = 0; t < 9; ++t)
        if ((mask >> t) & 1u) {
            if (j == 0) return t;
            --j;
        }
    return 0;
}

template <typename T, int R, int F, int FS, int PS>
__device__ __forceinline__ void mac_kernel(float (&acc)[F][R][4], const Window<T, R>& win, const Weights<T>& wt) {
    constexpr uint32_t mask = kBuiltinMasks[PS];
    mac_tap<T, R, F, FS, nth_tap(mask, 0), 0>(acc, win, wt);
    mac_tap<T, R, F, FS, nth_tap(mask, 1), 1>(acc, win, wt);
    mac_tap<T, R, F, FS, nth_tap(mask, 2), 2>(acc, win, wt);
    mac_tap<T, R, F, FS, nth_tap(mask, 3), 3>(acc, win, wt);
}

// Wave-uniform dispatch on code = filter slot * NP + pattern slot: a balanced tree of scalar
// compares down to the specialised block.  The tree is spelled with macros rather than a recursive
// template so that the end-of-chunk entry can be one more leaf of it (next to the last kernel
// code: the end code is larger than every kernel code) and leave the walker's loop from there;
// the kernels then pay no test of their own for it.  The expansion site provides: code, acc, win,
// wt, the constant kCopy that tells the two copies of the tree apart (the stream walker is
// unrolled twice), and the macros PPC_AT_BLOCK (statements at the head of a kernel block) and
// PPC_AT_END (statements of the end-of-chunk leaf).
// Distinct markers per block, before and after: without the first the optimiser hoists the blocks'
// common beginning back above the tree; without the second it merges the tails of blocks that
// differ only in their accumulator registers and pays for it with copies.
#define PPC_KERNEL_BLOCK(LO)                                                       \
    {                                                                              \
        asm volatile("; kernel block %0 copy %1" ::"n"(LO), "n"(kCopy));           \
        PPC_AT_BLOCK                                                               \
        mac_kernel<T, R, F, (LO) / NP, (LO) % NP>(acc, win, wt);                   \
        asm volatile("; end of block %0 copy %1" ::"n"(LO), "n"(kCopy));           \
    }
#define PPC_T1(LO)                                                                 \
    if constexpr ((LO) == F * NP - 1) {                                            \
        if (__builtin_expect(code == (uint32_t)(LO), 1)) PPC_KERNEL_BLOCK(LO) else { PPC_AT_END } \
    } else PPC_KERNEL_BLOCK(LO)
#define PPC_T2(LO) if (code < (uint32_t)((LO) + 1)) { PPC_T1(LO) } else { PPC_T1((LO) + 1) }
#define PPC_T4(LO) if (code < (uint32_t)((LO) + 2)) { PPC_T2(LO) } else { PPC_T2((LO) + 2) }
#define PPC_T8(LO) if (code < (uint32_t)((LO) + 4)) { PPC_T4(LO) } else { PPC_T4((LO) + 4) }
#define PPC_T16(LO) if (code < (uint32_t)((LO) + 8)) { PPC_T8(LO) } else { PPC_T8((LO) + 8) }
#define PPC_T32(LO) if (code < (uint32_t)((LO) + 16)) { PPC_T16(LO) } else { PPC_T16((LO) + 16) }
#define PPC_T64(LO) if (code < (uint32_t)((LO) + 32)) { PPC_T32(LO) } else { PPC_T32((LO) + 32) }
#define PPC_T128(LO) if (code < (uint32_t)((LO) + 64)) { PPC_T64(LO) } else { PPC_T64((LO) + 64) }
#define PPC_T256(LO) if (code < (uint32_t)((LO) + 128)) { PPC_T128(LO) } else { PPC_T128((LO) + 128) }
#define PPC_DISPATCH_TREE                                                          \
    static_assert(F * NP == 32 || F * NP == 64 || F * NP == 128 || F * NP == 256); \
    if constexpr (F * NP == 32) { PPC_T32(0) }                                     \
    else if constexpr (F * NP == 64) { PPC_T64(0) }                                \
    else if constexpr (F * NP == 128) { PPC_T128(0) }                              \
    else { PPC_T256(0) }

// One stream entry in scalar registers, fetched with a single scalar load.
//   fp32: 8 words {code, channel, -, -, w0, w1, w2, w3};   fp16: 4 words {code, w0|w1<<16, w2|w3<<16, channel}
template <typename T> struct Entry;
template <> struct Entry<float> {
    static constexpr int kWords = 8;
    typedef uint32_t vec_t __attribute__((ext_vector_type(8)));
    vec_t v;
    __device__ __forceinline__ uint32_t code() const { return v[0]; }
    __device__ __forceinline__ uint32_t channel() const { return v[1]; }
    __device__ __forceinline__ Weights<float> weights() const {
        // (element values are copied out first: a bit cast applied to a vector element expression
        // directly reads the wrong element with this compiler)
        const uint32_t u0 = v[4], u1 = v[5], u2 = v[6], u3 = v[7];
        return Weights<float>{{__builtin_bit_cast(float, u0), __builtin_bit_cast(float, u1), __builtin_bit_cast(float, u2),
                               __builtin_bit_cast(float, u3)}};
    }
};
template <> struct Entry<_Float16> {
    static constexpr int kWords = 4;
    typedef uint32_t vec_t __attribute__((ext_vector_type(4)));
    vec_t v;
    __device__ __forceinline__ uint32_t code() const { return v[0]; }
    __device__ __forceinline__ uint32_t channel() const { return v[3]; }
    __device__ __forceinline__ Weights<_Float16> weights() const { return Weights<_Float16>{{v[1], v[2]}}; }
};

// ---------------------------------------------------------------------------------------------
// LDS tile of one channel: [rows][TW] interior elements, then [rows][LW] halo pairs of two 32-bit
// words each.  Everything outside the images (padding rows, columns beyond W, the pairs of
// neighbours that do not exist) is zero: written as zeros by the register path, zeroed once per
// workgroup and never written again by the direct path.
//
// (1) Staging through registers, VEC elements per global load, for shapes whose rows are not
// aligned for the direct path.  Thread t takes vectors t, t + nthreads, ... of the chunk; two
// vectors are loaded before either is written and nothing looks at a loaded value until then,
// so both loads are in flight together.
template <typename T> struct StageRegs {
    uint32_t raw[2][4];   // up to 16 bytes per vector
    T edge[2];
};

template <typename T, int VEC, int LW, int R> struct Stager {
    static constexpr TileGeom tg = tile_geom(LW, R, (int)sizeof(T));
    static constexpr int TW = tg.tw, VPR = TW / VEC, CHS = tg.chs, HOFF = tg.hoff, HRS = tg.hrs;
    static constexpr int HP = HRS / LW;                      // elements per halo pair (2 for fp32, 4 for fp16)
    static constexpr int NB = VEC * (int)sizeof(T);
    static_assert(VPR >= 2, "a tile row must span at least two staging vectors");
    typedef typename VecOf<T, VEC>::type vec_t;

    // element index, inside a halo pair, of the left / right neighbour
    static constexpr int kLeft = HP == 2 ? 0 : 1, kRight = HP == 2 ? 1 : 2;

    static __device__ __forceinline__ void load(StageRegs<T>& sr, int u, int i, int total, const T* xc0,
                                                const int32_t* __restrict__ cmap, const int* rowtab, int trn,
                                                uint32_t trn_magic, int x0, int W, int hw) {
        const int row = i / VPR, v = i - row * VPR;              // VPR is a compile-time constant
        const int c = (int)__umulhi((uint32_t)row, trn_magic);   // row / trn (exact for row < 2^16)
        const int tr = row - c * trn;
        const int rb = i < total ? rowtab[tr] : -1;
        const int col = x0 + v * VEC;
        const uint32_t chan = (uint32_t)((i < total ? cmap[c] : 0) * hw);   // the channel staged at place c of the chunk
        const uint32_t goff = (rb >= 0 && col < W) ? chan + (uint32_t)(rb + col) : 0u;
        const vec_t val = *reinterpret_cast<const vec_t*>(xc0 + goff);
        __builtin_memcpy(&sr.raw[u][0], &val, NB);
        // the two elements just outside the strip are fetched by the first / last vector of a row
        const int ecol = v == 0 ? x0 - 1 : x0 + TW;
        const bool e_ok = rb >= 0 && (v == 0 || v == VPR - 1) && ecol >= 0 && ecol < W;
        sr.edge[u] = xc0[e_ok ? chan + (uint32_t)(rb + ecol) : 0u];
    }

    static __device__ __forceinline__ void store(const StageRegs<T>& sr, int u, int i, int total, T* tile,
                                                 const int* rowtab, int trn, uint32_t trn_magic, int x0, int W) {
        if (i >= total) return;
        const int row = i / VPR, v = i - row * VPR;
        const int c = (int)__umulhi((uint32_t)row, trn_magic);
        const int tr = row - c * trn;
        const bool in_img = rowtab[tr] >= 0;
        T* tc = tile + c * CHS;
        vec_t val;
        __builtin_memcpy(&val, &sr.raw[u][0], NB);
        if (!(in_img && x0 + v * VEC < W)) val = vec_t(0);
        *reinterpret_cast<vec_t*>(tc + tr * TW + v * VEC) = val;
        T* hrow = tc + HOFF + tr * HRS;
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            const int sc = v * VEC + k;                                       // column inside the strip
            const T e = vec_elem<T, VEC>(val, k);
            if ((sc & 3) == 0 && sc >= 4) hrow[(sc / 4 - 1) * HP + kRight] = e;     // right neighbour of the micro-column before
            if ((sc & 3) == 3 && sc + 1 < TW) hrow[(sc / 4 + 1) * HP + kLeft] = e;  // left neighbour of the next one
        }
        const int ecol = v == 0 ? x0 - 1 : x0 + TW;
        const T edge = (in_img && ecol >= 0 && ecol < W) ? sr.edge[u] : T(0);
        if (v == 0) hrow[kLeft] = edge;
        if (v == VPR - 1) hrow[(LW - 1) * HP + kRight] = edge;
    }

    static __device__ __forceinline__ void stage(const T* x, const int32_t* cmap, T* tile, const int* rowtab, int ccn, int trn,
                                                 uint32_t trn_magic, int x0, int W, int hw, int tid, int nthreads) {
        // Everything derived from the thread index is the same for every chunk; recomputing it is a
        // few integer instructions, keeping it live across the multiply-accumulate loop would cost
        // a dozen registers.  The empty asm makes the index opaque so that it is recomputed.
        asm volatile("" : "+v"(tid));
        const int total = ccn * trn * VPR;
        const T* xc0 = x;
        StageRegs<T> sr;
        for (int i0 = tid; i0 < total; i0 += 2 * nthreads) {
            load(sr, 0, i0, total, xc0, cmap, rowtab, trn, trn_magic, x0, W, hw);
            load(sr, 1, i0 + nthreads, total, xc0, cmap, rowtab, trn, trn_magic, x0, W, hw);
            store(sr, 0, i0, total, tile, rowtab, trn, trn_magic, x0, W);
            store(sr, 1, i0 + nthreads, total, tile, rowtab, trn, trn_magic, x0, W);
        }
    }
};

#define PPC_STAGE_DISPATCH(VECVAR, CALL)                                        \
    switch (VECVAR) {                                                           \
        case 8:                                                                 \
            if constexpr (sizeof(T) == 2 && LW % 2 == 0 && LW >= 4) { Stager<T, 8, LW, R>::CALL; } \
            break;                                                              \
        case 4: Stager<T, 4, LW, R>::CALL; break;                               \
        case 2: Stager<T, 2, LW, R>::CALL; break;                               \
        default: Stager<T, 1, LW, R>::CALL; break;                              \
    }

// A wave-uniform pointer, in scalar registers whatever the compiler thought of its provenance.
template <typename P> __device__ __forceinline__ P* uniform_ptr(P* p) {
    const uint64_t v = (uint64_t)(uintptr_t)p;
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v), hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return (P*)(uintptr_t)(((uint64_t)hi << 32) | lo);
}

// (2) Direct staging.  One wavefront instruction moves 64 slots of SLOT bytes from per-lane
// global addresses to 64 consecutive slots of LDS, asynchronously (counted by vmcnt).  The
// interior of a channel tile is ROWS*TW*sizeof(T)/SLOT slots, its halo area ROWS*LW*2 four-byte
// slots: NI + NH instructions per channel.  Which global element a lane fetches for instruction
// `it` of that sequence is the same for every channel and chunk, so it is tabulated once per
// workgroup as a byte offset from the channel's first element in use.  Two codes mark lanes that
// load nothing: kZeroSlot for a place that is read but lies outside the images (it is zeroed
// once per buffer, before the first load, and never written again), kNoSlot for a place nobody
// reads (rows the tile does not use, or past the end of its area).
//
// Buffers form a ring of NB; the loads of up to NB-1 chunks are in flight while one chunk is
// consumed.  Loads of one wavefront complete in order, so "chunk q has landed" is "at most as
// many loads outstanding as this wavefront has issued for later chunks" -- which needs the exact
// number of load instructions per chunk: an instruction without a single valid lane is skipped by
// a wave-uniform test, and every other one is issued unconditionally.
template <typename T, int SLOT, int LW, int R> struct DirectStager {
    static constexpr TileGeom tg = tile_geom(LW, R, (int)sizeof(T));
    static constexpr int TW = tg.tw, CHS = tg.chs, HOFF = tg.hoff, HRS = tg.hrs, ROWS = tg.rows;
    static constexpr int ES = SLOT / (int)sizeof(T);                  // elements per interior slot
    static constexpr int SPR = TW / ES;                               // interior slots per tile row
    static constexpr bool kUsable = TW % ES == 0;                     // (fp16, LW = 7 has 56-byte rows: 4-byte slots only)
    static constexpr int HE = 4 / (int)sizeof(T);                     // elements per halo slot (one 32-bit word)
    static constexpr int NI = (ROWS * SPR + 63) / 64, NH = (ROWS * LW * 2 + 63) / 64, NPER = NI + NH;
    static constexpr uint32_t kNoSlot = 0xFFFFFFFFu, kZeroSlot = 0xFFFFFFFEu;   // anything below is a byte offset

    // How the NPER instructions of each of a chunk's channels are dealt to the wavefronts:
    // wavefront w issues instruction w % NPER (and, with fewer wavefronts than instructions,
    // every nwaves-th one after it) for the channels phase, phase + nphase, ...
    struct Deal {
        int it0, phase, nphase;
        int valid_its;      // how many of this wavefront's instructions have a valid lane
    };

    static __device__ __forceinline__ void build(uint32_t* table, const int* rowtab, int rb0, int trn, int x0, int W,
                                                 int tid, int nthreads) {
        for (int j = tid; j < NI * 64; j += nthreads) {
            const int tr = j / SPR, v = j - tr * SPR;
            uint32_t off = kNoSlot;
            if (tr < trn) {
                const int rb = rowtab[tr];
                const int col = x0 + v * ES;
                off = (rb >= 0 && col < W) ? (uint32_t)(rb - rb0 + col) * (uint32_t)sizeof(T) : kZeroSlot;
            }
            table[j] = off;
        }
        uint32_t* htab = table + NI * 64;
        for (int j = tid; j < NH * 64; j += nthreads) {
            const int tr = j / (2 * LW), rem = j - tr * (2 * LW);
            const int mc = rem >> 1, side = rem & 1;
            uint32_t off = kNoSlot;
            if (tr < trn) {
                const int rb = rowtab[tr];
                // the word that holds the neighbour: fp32 the element itself; fp16 the aligned pair
                // (x[-2], x[-1]) on the left, (x[4], x[5]) on the right
                const int need = x0 + 4 * mc + (side ? 4 : -1);            // column of the neighbour element
                const int first = side ? need : need - (HE - 1);           // first column of the word
                off = (rb >= 0 && need >= 0 && need < W) ? (uint32_t)(rb - rb0 + first) * (uint32_t)sizeof(T) : kZeroSlot;
            }
            htab[j] = off;
        }
    }

    static __device__ __forceinline__ void deal(Deal& d, const uint32_t* table, int wave, int nwaves, int lane) {
        d.nphase = nwaves / NPER > 0 ? nwaves / NPER : 1;
        d.it0 = wave % NPER;
        d.phase = wave / NPER;
        d.valid_its = 0;
        if (d.phase >= d.nphase) {
            d.it0 = NPER;          // spare wavefront: issues nothing
            return;
        }
        for (int it = d.it0; it < NPER; it += nwaves)
            if (__builtin_amdgcn_ballot_w64(table[it * 64 + lane] < kZeroSlot) != 0) ++d.valid_its;
    }
    // load instructions this wavefront issues for a chunk of ccn channels
    static __device__ __forceinline__ int loads_per_chunk(const Deal& d, int ccn) {
        const int nch = ccn > d.phase ? (ccn - d.phase + d.nphase - 1) / d.nphase : 0;
        return nch * d.valid_its;
    }

    static __device__ __forceinline__ void run_setup(const uint32_t* table, int wave, int nwaves, int lane, int cc,
                                                     int ccn_last, int& it0, int& phase, int& nphase, int& valid,
                                                     int& loads_full, int& loads_last) {
        Deal d;
        deal(d, table, wave, nwaves, lane);
        it0 = d.it0;
        phase = d.phase;
        nphase = d.nphase;
        valid = d.valid_its;
        loads_full = loads_per_chunk(d, cc);
        loads_last = loads_per_chunk(d, ccn_last);
    }

    // Zero the places marked kZeroSlot in every channel of every buffer (nbuf * cc channel tiles in a
    // row, CHS elements apart), with the instructions dealt to the wavefronts as the loads are.
    static __device__ __forceinline__ void zero_holes(const Deal& d, const uint32_t* table, unsigned char* tiles, int nchan,
                                                      int nwaves, int lane) {
        for (int it = d.it0; it < NPER; it += nwaves) {
            const bool hole = table[it * 64 + lane] == kZeroSlot;
            if (__builtin_amdgcn_ballot_w64(hole) == 0) continue;
            unsigned char* p = tiles + (it < NI ? (it * 64 + lane) * SLOT : HOFF * (int)sizeof(T) + ((it - NI) * 64 + lane) * 4);
            for (int c = d.phase; c < nchan; c += d.nphase) {
                unsigned char* pc = p + c * (CHS * (int)sizeof(T));
                if (!hole) continue;
                if (it < NI) {
                    if constexpr (SLOT == 16) *reinterpret_cast<f32x4*>(pc) = f32x4(0);
                    else *reinterpret_cast<uint32_t*>(pc) = 0u;
                } else {
                    *reinterpret_cast<uint32_t*>(pc) = 0u;
                }
            }
        }
    }

    // One direct load: lanes with a slot fetch SLOT bytes at base + off into LDS at lds_dst + lane*SLOT.
    // Inline assembly rather than the compiler builtin on purpose: the compiler cannot tell which
    // later LDS reads an in-flight direct load may alias and would wait for all of them before the
    // first read of another buffer, which is exactly the overlap this path exists for.
    template <int BYTES>
    static __device__ __forceinline__ void dma(uint32_t off, const void* base, uint32_t lds_dst) {
        if constexpr (BYTES == 16)
            asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(off), "s"(base), "s"(lds_dst) : "memory", "m0");
        else
            asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1" ::"v"(off), "s"(base), "s"(lds_dst) : "memory", "m0");
    }

    // Start the loads of channels [c0, c0+ccn) into the buffer at LDS byte address lds_buf.
    // xrow0: the first element in use of channel 0 (image base + first valid tile row).
    // cmap: the channels of this chunk, by place (wave-uniform reads from constant memory).
    static __device__ __forceinline__ void issue(const Deal& d, const T* __restrict__ xrow0, uint32_t lds_buf,
                                                 const uint32_t* table, const __attribute__((address_space(4))) int32_t* cmap,
                                                 int ccn, int hw, int nwaves) {
        // the lane id is worked out here, every time, instead of living in a register across the
        // multiply-accumulate loop (the empty asm stops the compiler from hoisting it)
        int lane = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
        asm volatile("" : "+v"(lane));
        for (int it = d.it0; it < NPER; it += nwaves) {               // wave-uniform; one pass unless NPER > nwaves
            const uint32_t off = table[it * 64 + lane];
            const bool ok = off < kZeroSlot;
            if (__builtin_amdgcn_ballot_w64(ok) == 0) continue;
            const uint32_t lds_it = lds_buf + (uint32_t)(it < NI ? it * 64 * SLOT : HOFF * (int)sizeof(T) + (it - NI) * 64 * 4);
            for (int c = d.phase; c < ccn; c += d.nphase) {
                const T* xc = uniform_ptr(xrow0 + (int64_t)cmap[c] * hw);
                const uint32_t dst = lds_it + (uint32_t)(c * CHS * (int)sizeof(T));
                if (ok) {
                    if (it < NI) dma<SLOT>(off, xc, dst);
                    else dma<4>(off, xc, dst);
                }
            }
        }
    }
};

#define PPC_DIRECT_DISPATCH(MODEVAR, CALL)                                      \
    if (MODEVAR == 1) {                                                         \
        typedef DirectStager<T, 16, LW, R> ST;                                  \
        if constexpr (ST::kUsable) { ST::CALL; }                                \
    } else {                                                                    \
        typedef DirectStager<T, 4, LW, R> ST;                                   \
        ST::CALL;                                                               \
    }

// Wait until at most n of this wavefront's vector-memory operations are outstanding (the count is
// an immediate of the instruction; the hardware counter has 6 bits).
__device__ __forceinline__ void wait_vmcnt_at_most(int n) {
#define PPC_W(N) case N: asm volatile("s_waitcnt vmcnt(" #N ")" ::: "memory"); break;
    switch (n) {
        PPC_W(0) PPC_W(1) PPC_W(2) PPC_W(3) PPC_W(4) PPC_W(5) PPC_W(6) PPC_W(7)
        PPC_W(8) PPC_W(9) PPC_W(10) PPC_W(11) PPC_W(12) PPC_W(13) PPC_W(14) PPC_W(15)
        PPC_W(16) PPC_W(17) PPC_W(18) PPC_W(19) PPC_W(20) PPC_W(21) PPC_W(22) PPC_W(23)
        PPC_W(24) PPC_W(25) PPC_W(26) PPC_W(27) PPC_W(28) PPC_W(29) PPC_W(30) PPC_W(31)
        PPC_W(32) PPC_W(33) PPC_W(34) PPC_W(35) PPC_W(36) PPC_W(37) PPC_W(38) PPC_W(39)
        PPC_W(40) PPC_W(41) PPC_W(42) PPC_W(43) PPC_W(44) PPC_W(45) PPC_W(46) PPC_W(47)
        PPC_W(48) PPC_W(49) PPC_W(50) PPC_W(51) PPC_W(52) PPC_W(53) PPC_W(54) PPC_W(55)
        PPC_W(56) PPC_W(57) PPC_W(58) PPC_W(59) PPC_W(60) PPC_W(61) PPC_W(62)
        default: break;     // 63 or more: the counter cannot exceed that, nothing to wait for
    }
#undef PPC_W
}

// Variants with at most 32 accumulators per lane are asked to fit 64 vector registers, i.e. 8
// resident wavefronts per SIMD: two 16-wavefront workgroups per CU, which is what hides the scalar
// dispatch and LDS latency of one behind the multiply-accumulates of the other.  (Staging through
// registers needs the registers itself and is left at 4.)
template <typename T, int NP, int R, int F, int LW, bool DIRECT>
__global__ __launch_bounds__(1024) __attribute__((amdgpu_waves_per_eu(DIRECT && F * R * 4 <= 32 ? 8 : 4)))
void k1_tiled(const K1Args a) {
    constexpr TileGeom tg = tile_geom(LW, R, (int)sizeof(T));
    constexpr int TW = tg.tw, RS = tg.rs, CHS = tg.chs, ROWS = tg.rows, HOFF = tg.hoff, HRS = tg.hrs;
    constexpr int HP = HRS / LW;                    // elements per halo pair
    extern __shared__ __align__(16) unsigned char smem_raw[];
    __shared__ int rowtab[ROWS];
    T* tile = reinterpret_cast<T*>(smem_raw);

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nwaves = a.wf * a.ks;
    const int ksi = (wave * a.wf_recip) >> 16, wfi = wave - ksi * a.wf;   // wave / wf, wave % wf (wave < 16)

    // Block -> work item.  Consecutive block ids are dealt round-robin to the 8 XCDs, each with
    // its own L2, so block id i is first turned into "slot i/8 of XCD i%8" and every XCD is given a
    // contiguous range of work items.  Work items are ordered channel share fastest, then filter
    // block, then strip, then row band: workgroups that read the same input tile (other filter
    // blocks), its edge columns (neighbouring strips) or add up one output tile (other shares) run
    // on the same XCD at about the same time and find those lines in its L2.
    const int per_xcd = a.blocks_per_xcd;
    int item = (int)(blockIdx.x % 8u) * per_xcd + (int)(blockIdx.x / 8u);
    if (item >= a.work_items) return;            // grid is rounded up to a multiple of 8
    int slice = 0, q0 = 0, q1 = a.chunks;        // which share of the channel chunks
    if (a.split_wg > 1) {
        slice = item % a.split_wg;
        item /= a.split_wg;
        q0 = slice * a.chunks / a.split_wg;      // (products stay far below 2^31)
        q1 = (slice + 1) * a.chunks / a.split_wg;
    }
    const int tile_id = item;                    // the output tile: (filter block, strip, row band)
    const int fb = item % a.nfb;
    item /= a.nfb;
    const int strip = item % a.strips;
    const int b = item / a.strips;
    const int g = fb * a.wf + wfi;
    const bool has_group = g < a.groups;
    const int x0 = strip * TW;

    const int m0 = b * 64;
    const int mr0 = m0 / LW;
    int mr1 = (m0 + 63) / LW + 1;
    if (mr1 > a.mrows) mr1 = a.mrows;
    const int trn = (mr1 - mr0) * R + 2;          // LDS tile rows in use (<= ROWS)
    const int u0 = mr0 * R - 1;                    // virtual input row held by tile row 0
    const int m = m0 + lane;
    const int mrow = m / LW, mcol = m - mrow * LW;
    const int lr = mrow - mr0;

    // virtual input row -> element offset of that row in channel 0 of its image, or -1 for a zero row
    for (int tr = threadIdx.x; tr < ROWS; tr += blockDim.x) {
        const int u = u0 + tr;
        int off = -1;
        if (tr < trn && u >= 0) {
            const int img = u / (a.h + 1), yy = u - img * (a.h + 1);
            if (yy < a.h && img < a.n) off = (img * a.c_in * a.h + yy) * a.w;
        }
        rowtab[tr] = off;
    }

    float acc[F][R][4];
#pragma unroll
    for (int f = 0; f < F; ++f)
#pragma unroll
        for (int rr = 0; rr < R; ++rr)
#pragma unroll
            for (int k = 0; k < 4; ++k) acc[f][rr][k] = 0.0f;

    // The lane's interior columns start lane_bytes into a channel tile, and its halo pair at
    // HOFF + that offset * HRS / RS (rows of pairs are HRS long where rows of pixels are RS long, and
    // a pair takes HP elements where a micro-column takes 4: the same ratio), so one register holds
    // the lane's place.
    static_assert(HRS * 4 == RS * HP && (RS % HRS == 0), "halo rows must scale with interior rows");
    const int lane_bytes = (lr * R * RS + 4 * mcol) * (int)sizeof(T);
    const int hw = a.h * a.w;
    const uint32_t trn_magic = 0xFFFFFFFFu / (uint32_t)trn + 1u;      // ceil(2^32 / trn), trn >= 3
    const T* __restrict__ xin = static_cast<const T*>(a.x);
    const int32_t* __restrict__ cmap = a.chan_map + (int64_t)fb * a.chunks * a.cc;   // this filter block's channel order

    // This wavefront's entry stream (constant address space: wave-uniform loads from it are scalar
    // loads).  Wavefronts beyond the last filter group walk a stream of end-of-chunk entries only.
    typedef const __attribute__((address_space(4))) typename Entry<T>::vec_t* stream_ptr_t;
    typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr_t;
    stream_ptr_t sp = (stream_ptr_t)(a.stream) + (has_group ? ((const_i32_ptr_t)a.wave_off)[(g * a.ks + ksi) * a.split_wg + slice] : a.idle_off);

    // Direct staging: ring of a.nbuf buffers of a.cc channels each; the loads of the next
    // a.nbuf - 1 chunks are in flight while a chunk is consumed.
    typedef __attribute__((address_space(3))) unsigned char* lds_byte_ptr;
    const uint32_t lds_tile = (uint32_t)(uintptr_t)(lds_byte_ptr)smem_raw;   // LDS byte address of buffer 0
    const int buf_elems = a.cc * CHS;
    const uint32_t* table = reinterpret_cast<const uint32_t*>(smem_raw + a.table_offset);
    const T* xrow0 = xin;
    int d_it0 = 0, d_phase = 0, d_nphase = 1, d_valid = 0, loads_full = 0, loads_last = 0;
#define PPC_DEAL(ST) typename ST::Deal{d_it0, d_phase, d_nphase, d_valid}
    const int ahead = a.nbuf - 1;
    if constexpr (DIRECT) {
        __syncthreads();          // rowtab written
        int rb0 = rowtab[0];
        if (rb0 < 0) rb0 = rowtab[1];
        if (rb0 < 0) rb0 = rowtab[2];          // two consecutive virtual rows are never both outside the images
        if (rb0 < 0) rb0 = 0;
        rb0 = __builtin_amdgcn_readfirstlane(rb0);
        xrow0 = xin + rb0;
        PPC_DIRECT_DISPATCH(a.mode, build(reinterpret_cast<uint32_t*>(smem_raw + a.table_offset), rowtab, rb0, trn, x0, a.w,
                                          threadIdx.x, blockDim.x))
        __syncthreads();
        const int ccn_last = a.c_in - (a.chunks - 1) * a.cc;
        PPC_DIRECT_DISPATCH(a.mode, run_setup(table, wave, nwaves, lane, a.cc, ccn_last, d_it0, d_phase, d_nphase,
                                                               d_valid, loads_full, loads_last))
        if (q1 != a.chunks) loads_last = loads_full;        // only the layer's last chunk can be short
        // zero, once, the places inside the tiles that lie outside the images: no load ever writes them
        PPC_DIRECT_DISPATCH(a.mode, zero_holes(PPC_DEAL(ST), table, smem_raw, a.nbuf * a.cc, nwaves, lane))
        for (int k = 0; k < ahead && q0 + k < q1; ++k) {
            const int c0 = (q0 + k) * a.cc;
            const int ccn = (a.c_in - c0 < a.cc) ? a.c_in - c0 : a.cc;
            PPC_DIRECT_DISPATCH(a.mode, issue(PPC_DEAL(ST), xrow0, lds_tile + (uint32_t)(k * buf_elems * (int)sizeof(T)), table,
                                              (const_i32_ptr_t)cmap + c0, ccn, hw, nwaves))
        }
    }

    // Make chunk q readable: returns the LDS address of the buffer that holds it.
    int ring = 0;                 // buffer that holds chunk q
    auto begin_chunk = [&](int q) -> lds_cbyte_ptr {
        int boff = 0;
        if constexpr (DIRECT) {
            // chunk q has landed once no more loads are outstanding than were issued for the chunks
            // after it (q+1 .. q+ahead-1, as far as they exist; all but the last chunk are full)
            int later = q1 - 1 - q;
            if (later > ahead - 1) later = ahead - 1;
            int allowed = later * loads_full;
            if (later > 0 && q + later == q1 - 1) allowed += loads_last - loads_full;
            wait_vmcnt_at_most(allowed);
            __syncthreads();      // everyone's loads of chunk q have landed; everyone is done with chunk q-1
            boff = ring * buf_elems;
            const int qn = q + ahead;            // goes into the buffer chunk q-1 was read from
            if (qn < q1) {
                const int cn0 = qn * a.cc;
                const int ccn1 = (a.c_in - cn0 < a.cc) ? a.c_in - cn0 : a.cc;
                const int slot = ring == 0 ? ahead : ring - 1;
                PPC_DIRECT_DISPATCH(a.mode, issue(PPC_DEAL(ST), xrow0, lds_tile + (uint32_t)(slot * buf_elems * (int)sizeof(T)), table,
                                                  (const_i32_ptr_t)cmap + cn0, ccn1, hw, nwaves))
            }
            ring = ring + 1 == a.nbuf ? 0 : ring + 1;
        } else {
            const int c0 = q * a.cc;
            const int ccn = (a.c_in - c0 < a.cc) ? a.c_in - c0 : a.cc;
            __syncthreads();      // previous chunk fully consumed (and rowtab written, first time round)
            PPC_STAGE_DISPATCH(a.vec, stage(xin, cmap + c0, tile, rowtab, ccn, trn, trn_magic, x0, a.w, hw, threadIdx.x, blockDim.x))
            __syncthreads();
        }
        return (lds_cbyte_ptr)smem_raw + boff * (int)sizeof(T);
    };

    // The stream walker.  Entries are fetched one ahead, so that the scalar-load latency hides behind
    // the previous kernel's multiply-accumulates, and alternately into two register sets, so that
    // no entry is ever copied: the loop body exists twice, once per set, and the two copies fetch
    // at fixed offsets from one pointer that moves once per pair.  An end-of-chunk entry leaves the
    // inner loop; the outer loop switches to the next chunk's tile and restarts the pairs at the
    // entry after it.
    // The window's LDS reads are left in flight across the dispatch tree and awaited at the head of
    // the kernel block; only then is the next entry's scalar load issued: LDS reads and scalar loads
    // share one counter, so a wait with that load outstanding would expose its latency too.
    // (0xC07F = lgkmcnt(0), vmcnt and expcnt unconstrained; the builtin, unlike inline assembly, is
    // visible to the compiler's own wait-count bookkeeping)
    Window<T, R> win;
    win.clear();
    Entry<T> ea, eb;
#define PPC_STEP(CUR, NXT, COPY)                                                                        \
    {                                                                                                   \
        constexpr int kCopy = COPY;                                                                     \
        const uint32_t chan = CUR.channel();                                                            \
        if (chan != kSameChannel) {                                                                     \
            const lds_cbyte_ptr pc = chunk_base + chan;                                                 \
            win.load(pc + lane_bytes, pc + HOFF * (int)sizeof(T) + lane_bytes / (RS / HRS),             \
                     RS * (int)sizeof(T), HRS * (int)sizeof(T));                                        \
        }                                                                                               \
        const uint32_t code = CUR.code();                                                               \
        const Weights<T> wt = CUR.weights();                                                            \
        PPC_DISPATCH_TREE                                                                               \
    }
#define PPC_AT_BLOCK                        \
    __builtin_amdgcn_s_waitcnt(0xC07F);     \
    NXT_ENTRY.v = sp[kCopy + 1];
#define PPC_AT_END          \
    sp += kCopy + 1;        \
    break;
    for (int q = q0; q < q1; ++q) {
        const lds_cbyte_ptr chunk_base = begin_chunk(q);
        ea.v = sp[0];
        for (;;) {
#define NXT_ENTRY eb
            PPC_STEP(ea, eb, 0)
#undef NXT_ENTRY
#define NXT_ENTRY ea
            PPC_STEP(eb, ea, 1)
#undef NXT_ENTRY
            sp += 2;
        }
    }
#undef PPC_AT_BLOCK
#undef PPC_AT_END
#undef PPC_STEP

    // The epilogue reads the kernel arguments again from the argument segment (through a pointer the
    // compiler cannot see through) instead of keeping a dozen of them in scalar registers across the
    // loop, where scalar registers are short and every spilled one costs a vector register.
    typedef const __attribute__((address_space(4))) K1Args* args_ptr_t;
    args_ptr_t ka = (args_ptr_t)__builtin_amdgcn_kernarg_segment_ptr();
    asm volatile("" : "+s"(ka));

    // What the lane needs after the loop (its place in the tile) is derived again from the thread
    // index rather than kept in registers across the loop; the empty asm keeps the compiler from
    // merging the two computations.
    int lane_e = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));   // lane id, without the thread index
    asm volatile("" : "+v"(lane_e));
    const int m_e = m0 + lane_e;
    const int mrow_e = m_e / LW, mcol_e = m_e - mrow_e * LW;

    // ---- sum the channel splits through LDS, in a fixed order (deterministic): as many splits at a
    // time as LDS has room for (red_par slabs of [wf][F*R*4][64] floats), added in split order ----
    if (ka->ks > 1) {
        float* red = reinterpret_cast<float*>(smem_raw);
        const int slab = ka->wf * (F * R * 4 * 64);
        for (int s0 = 1; s0 < ka->ks; s0 += ka->red_par) {
            __syncthreads();
            if (ksi >= s0 && ksi < s0 + ka->red_par) {
                float* mine = red + (ksi - s0) * slab;
#pragma unroll
                for (int f = 0; f < F; ++f)
#pragma unroll
                    for (int rr = 0; rr < R; ++rr)
#pragma unroll
                        for (int k = 0; k < 4; ++k)
                            mine[((wfi * F + f) * R * 4 + rr * 4 + k) * 64 + lane_e] = acc[f][rr][k];
            }
            __syncthreads();
            if (ksi == 0) {
                for (int s = s0; s < s0 + ka->red_par && s < ka->ks; ++s) {
                    const float* theirs = red + (s - s0) * slab;
#pragma unroll
                    for (int f = 0; f < F; ++f)
#pragma unroll
                        for (int rr = 0; rr < R; ++rr)
#pragma unroll
                            for (int k = 0; k < 4; ++k)
                                acc[f][rr][k] += theirs[((wfi * F + f) * R * 4 + rr * 4 + k) * 64 + lane_e];
                }
            }
        }
    }
    // Visit this lane's outputs: fn(f, rr, element offset of the four pixels in an [n][c_out][h][w]
    // array, original filter index, slot).  Only the wavefronts that hold sums have any.
    const int xcol = x0 + 4 * mcol_e;
    const bool owns = ksi == 0 && has_group && mrow_e < ka->mrows && xcol < ka->w;
    auto for_each_output = [&](auto&& fn) {
        if (!owns) return;
#pragma unroll
        for (int rr = 0; rr < R; ++rr) {
            const int v = mrow_e * R + rr;
            if (v >= ka->vh) continue;
            const int img = v / (ka->h + 1), yy = v - img * (ka->h + 1);
            if (yy >= ka->h) continue;
#pragma unroll
            for (int f = 0; f < F; ++f) {
                const int co = ka->perm_pad[g * F + f];
                if (co < 0) continue;
                fn(f, rr, (((int64_t)img * ka->c_out + co) * ka->h + yy) * ka->w + xcol, g * F + f);
            }
        }
    };
    const bool vec_store = (ka->w & 3) == 0;

    // ---- channel split across workgroups: publish this share's partial sums; the workgroup that
    // arrives last at the tile adds up all shares, in share order whoever it is, and finishes ----
    // The shares may run on different XCDs, whose L2 caches are not coherent with each other.  A
    // device-scope fence would write back and invalidate a whole L2 for every workgroup; instead
    // everything the workgroups exchange (partial sums, arrival counter) is moved with device-scope
    // relaxed atomic loads and stores, which go past the L2, and ordered by hand: the stores have
    // been acknowledged (vmcnt 0) before the arrival is counted, and the sums are read only after
    // the count has come back.
    if (ka->split_wg > 1) {
        __shared__ int arrived;
        float* __restrict__ mine = ka->ws + (int64_t)slice * ka->out_elems;
        for_each_output([&](int f, int rr, int64_t off, int) {
            if (vec_store) {      // the same kind of store, 16 bytes wide
                const f32x4 v = {acc[f][rr][0], acc[f][rr][1], acc[f][rr][2], acc[f][rr][3]};
                asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1" ::"v"(mine + off), "v"(v) : "memory");
            } else {
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    if (xcol + k < ka->w) __hip_atomic_store(mine + off + k, acc[f][rr][k], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        });
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (wave == 0 && lane_e == 0) arrived = __hip_atomic_fetch_add(ka->counters + tile_id, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        if (arrived != ka->split_wg - 1) return;
        if (wave == 0 && lane_e == 0) __hip_atomic_store(ka->counters + tile_id, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);   // for the next launch
        for_each_output([&](int f, int rr, int64_t off, int) {
            float sum[4] = {0.0f, 0.0f, 0.0f, 0.0f};
            for (int sh = 0; sh < ka->split_wg; ++sh) {
                if (sh == slice) {
#pragma unroll
                    for (int k = 0; k < 4; ++k) sum[k] += acc[f][rr][k];
                } else {
                    const float* theirs = ka->ws + (int64_t)sh * ka->out_elems + off;
                    if (vec_store) {
                        f32x4 t;
                        asm volatile("global_load_dwordx4 %0, %1, off sc0 sc1\n\ts_waitcnt vmcnt(0)" : "=v"(t) : "v"(theirs) : "memory");
#pragma unroll
                        for (int k = 0; k < 4; ++k) sum[k] += t[k];
                    } else {
#pragma unroll
                        for (int k = 0; k < 4; ++k)
                            if (xcol + k < ka->w) sum[k] += __hip_atomic_load(theirs + k, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                }
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) acc[f][rr][k] = sum[k];
        });
    }

    // ---- epilogue: bias, ReLU, store at the filter's original index ----
    T* __restrict__ yout = static_cast<T*>(ka->y);
    for_each_output([&](int f, int rr, int64_t off, int slot) {
        const float bz = ka->bias_pad[slot];
        float o[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            o[k] = acc[f][rr][k] + bz;
            if (ka->relu) o[k] = o[k] > 0.0f ? o[k] : 0.0f;
        }
        T* dst = yout + off;
        if (vec_store) {
            typename VecOf<T, 4>::type ov;
            ov[0] = (T)o[0];
            ov[1] = (T)o[1];
            ov[2] = (T)o[2];
            ov[3] = (T)o[3];
            *reinterpret_cast<typename VecOf<T, 4>::type*>(dst) = ov;
        } else {
#pragma unroll
            for (int k = 0; k < 4; ++k)
                if (xcol + k < ka->w) dst[k] = (T)o[k];
        }
    });
}

typedef void (*k1_launch_fn)(const K1Args& a, int blocks, int threads, int lds_bytes, hipStream_t stream);
// Look up the instantiation for (dtype, np, r, f, lw, staging path); nullptr if that combination is not built.
k1_launch_fn k1_lookup(int dtype, int np, int r, int f, int lw, bool direct);

}  // namespace ppc

// Tiled, pattern-specialised kernel for the pattern-pruned 3x3 convolution on gfx950.
//
// Mapping (chosen for 64-wide wavefronts, not the thread-per-filter mapping the paper uses on
// mobile CPUs/GPUs in its filter-kernel-reorder figure of section 2.3.1):
//   * lanes own output pixels: a lane holds an R x 4 micro-tile of adjacent pixels for each of
//     the F filters of its wavefront (F*R*4 fp32 accumulators);
//   * a wavefront therefore sees every weight, pattern and loop bound as a wave-uniform value:
//     they live in scalar registers, are fetched with scalar loads from the packed weight
//     stream, and every sparsity-dependent branch is a scalar branch -- no lane divergence;
//   * a workgroup is WF x KS wavefronts that share one LDS-resident input tile (the paper's
//     "input tiling"): WF of them work on different filter groups, KS of them split the input
//     channels of each chunk and are summed through LDS at the end in a fixed order.
//
// Per input channel a lane reads its (R+2) x 6 input window from LDS once, with one 128-bit
// (fp32) or 64-bit (fp16) read for the four interior columns and one read for the packed
// (left, right) halo pair per row, and reuses it from registers for every kernel of the
// wavefront's filters that keeps that channel.  The multiply-accumulates of one kernel are a
// straight-line block specialised on (filter slot, pattern): all register indices are static
// ("statically determined data access instructions", section 2.3.1, load redundancy
// elimination).
//
// The batch is laid out as one tall virtual image: image n, row y is virtual row n*(H+1)+y and
// row y = H of every image is a shared zero row, so that tiles may straddle images.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "plan.hpp"

namespace ppc {

struct K1Args {
    const void* x;
    void* y;
    const uint32_t* stream;     // weight-stream entries
    const int32_t* wave_off;    // [G*KS] first entry per (group, split)
    const float* bias_pad;      // [G*F]
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
    int32_t vec;                // staging vector width in elements
    int32_t relu;
};

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

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
// of one of its elements with a wave-uniform weight.
template <typename T, int R> struct Window;

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
    __device__ __forceinline__ void load(const float* pm, const float* ph, int rs) {
#pragma unroll
        for (int rr = 0; rr < R + 2; ++rr) {
            mid[rr] = *reinterpret_cast<const f32x4*>(pm + rr * rs);
            halo[rr] = *reinterpret_cast<const f32x2*>(ph + rr * rs);
        }
    }
    template <int ROW, int COL> __device__ __forceinline__ void fma(float& acc, float w) const {
        if constexpr (COL < 0) acc = __builtin_fmaf(w, halo[ROW][0], acc);
        else if constexpr (COL > 3) acc = __builtin_fmaf(w, halo[ROW][1], acc);
        else acc = __builtin_fmaf(w, mid[ROW][COL], acc);
    }
};

// fp16 storage: the window stays packed, two halves per register, and every multiply-accumulate
// is one v_fma_mix_f32 (fp16 input selected from the low or high half, fp32 weight from a scalar
// register, fp32 accumulator).  Written as inline assembly because the compiler otherwise
// unpacks halves that are used several times with extra conversion instructions.
template <int R> struct Window<_Float16, R> {
    uint32_t mid[R + 2][2];   // columns (0,1), (2,3)
    uint32_t halo[R + 2];     // (column -1, column 4)
    __device__ __forceinline__ void clear() {
#pragma unroll
        for (int rr = 0; rr < R + 2; ++rr) mid[rr][0] = mid[rr][1] = halo[rr] = 0u;
    }
    __device__ __forceinline__ void load(const _Float16* pm, const _Float16* ph, int rs) {
        typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
#pragma unroll
        for (int rr = 0; rr < R + 2; ++rr) {
            const u32x2 m = *reinterpret_cast<const u32x2*>(pm + rr * rs);
            mid[rr][0] = m[0];
            mid[rr][1] = m[1];
            halo[rr] = *reinterpret_cast<const uint32_t*>(ph + rr * rs);
        }
    }
    template <int ROW, int COL> __device__ __forceinline__ void fma(float& acc, float w) const {
        constexpr bool hi = (COL < 0) ? false : (COL > 3) ? true : (COL & 1) != 0;
        const uint32_t src = (COL < 0 || COL > 3) ? halo[ROW] : mid[ROW][(COL < 0 ? 0 : COL) >> 1];
        if constexpr (hi)
            asm("v_fma_mix_f32 %0, %1, %2, %0 op_sel:[0,1,0] op_sel_hi:[0,1,0]" : "+v"(acc) : "s"(w), "v"(src));
        else
            asm("v_fma_mix_f32 %0, %1, %2, %0 op_sel_hi:[0,1,0]" : "+v"(acc) : "s"(w), "v"(src));
    }
};

// ---------------------------------------------------------------------------------------------
// Multiply-accumulate block of one kept kernel: filter slot FS, pattern slot PS (4 taps).
template <typename T, int R, int F, int FS, int RR, int TAP>
__device__ __forceinline__ void mac_row(float (&acc)[F][R][4], const Window<T, R>& win, float wj) {
    constexpr int dr = TAP / 3, dc = TAP % 3 - 1;
    win.template fma<RR + dr, 0 + dc>(acc[FS][RR][0], wj);
    win.template fma<RR + dr, 1 + dc>(acc[FS][RR][1], wj);
    win.template fma<RR + dr, 2 + dc>(acc[FS][RR][2], wj);
    win.template fma<RR + dr, 3 + dc>(acc[FS][RR][3], wj);
}

template <typename T, int R, int F, int FS, int TAP, int RR = 0>
__device__ __forceinline__ void mac_tap(float (&acc)[F][R][4], const Window<T, R>& win, float wj) {
    if constexpr (RR < R) {
        mac_row<T, R, F, FS, RR, TAP>(acc, win, wj);
        mac_tap<T, R, F, FS, TAP, RR + 1>(acc, win, wj);
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
__device__ __forceinline__ void mac_kernel(float (&acc)[F][R][4], const Window<T, R>& win, const float (&wt)[4]) {
    constexpr uint32_t mask = kBuiltinMasks[PS];
    mac_tap<T, R, F, FS, nth_tap(mask, 0)>(acc, win, wt[0]);
    mac_tap<T, R, F, FS, nth_tap(mask, 1)>(acc, win, wt[1]);
    mac_tap<T, R, F, FS, nth_tap(mask, 2)>(acc, win, wt[2]);
    mac_tap<T, R, F, FS, nth_tap(mask, 3)>(acc, win, wt[3]);
}

// Wave-uniform dispatch on code = filter slot * NP + pattern slot: a balanced tree of scalar
// compares down to the specialised block.
template <typename T, int R, int F, int NP, int LO, int HI>
__device__ __forceinline__ void dispatch(int code, float (&acc)[F][R][4], const Window<T, R>& win, const float (&wt)[4]) {
    if constexpr (HI - LO == 1) {
        mac_kernel<T, R, F, LO / NP, LO % NP>(acc, win, wt);
        // A distinct marker per block: without it the optimiser merges the tails of blocks that
        // differ only in their accumulator registers and pays for it with register copies.
        asm volatile("; kernel block %0" ::"n"(LO));
    } else {
        constexpr int MID = (LO + HI) / 2;
        if (code < MID) dispatch<T, R, F, NP, LO, MID>(code, acc, win, wt);
        else dispatch<T, R, F, NP, MID, HI>(code, acc, win, wt);
    }
}

// ---------------------------------------------------------------------------------------------
// Staging of one channel chunk into LDS (zero-filled outside the images), VEC elements per
// global load.  The chunk is a list of ccn*trn tile rows of VPR vectors each; thread t takes
// vectors t, t + nthreads, ...  Interior columns go to [row][0..TW); an element that is some
// micro-tile's left or right neighbour is also written to that micro-tile's (left, right) halo
// pair, which sits behind the interior at [row][HOFF + 2*mcol].  The pair array has one dummy pair
// on each side so that these writes need no bounds test.
//
// Two vectors per thread are loaded before either is written, and nothing looks at a loaded
// value until then (out-of-image vectors read a valid dummy address and are zeroed when stored),
// so both loads are in flight together.
template <typename T> struct StageRegs {
    uint32_t raw[2][4];   // up to 16 bytes per vector
    T edge[2];
};

template <typename T, int VEC, int LW, int R> struct Stager {
    static constexpr TileGeom tg = tile_geom(LW, R, (int)sizeof(T));
    static constexpr int TW = tg.tw, VPR = TW / VEC, RS = tg.rs, CHS = tg.chs, HOFF = tg.hoff;
    static constexpr int NB = VEC * (int)sizeof(T);
    static_assert(VPR >= 2, "a tile row must span at least two staging vectors");
    typedef typename VecOf<T, VEC>::type vec_t;

    static __device__ __forceinline__ void load(StageRegs<T>& sr, int u, int i, int total, const T* xc0,
                                                const int* rowtab, int trn, uint32_t trn_magic, int x0, int W, int hw) {
        const int row = i / VPR, v = i - row * VPR;              // VPR is a compile-time constant
        const int c = (int)__umulhi((uint32_t)row, trn_magic);   // row / trn (exact for row < 2^16)
        const int tr = row - c * trn;
        const int rb = i < total ? rowtab[tr] : -1;
        const int col = x0 + v * VEC;
        const uint32_t chan = (uint32_t)(c * hw);
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
        T* trow = tile + c * CHS + tr * RS;
        vec_t val;
        __builtin_memcpy(&val, &sr.raw[u][0], NB);
        if (!(in_img && x0 + v * VEC < W)) val = vec_t(0);
        *reinterpret_cast<vec_t*>(trow + v * VEC) = val;
        T* hrow = trow + HOFF;
#pragma unroll
        for (int k = 0; k < VEC; ++k) {
            const int sc = v * VEC + k;
            const T e = vec_elem<T, VEC>(val, k);
            if (VEC >= 4) {                                   // which elements are neighbours is static
                if ((k & 3) == 0) hrow[2 * (sc / 4 - 1) + 1] = e;
                if ((k & 3) == 3) hrow[2 * (sc / 4 + 1)] = e;
            } else {
                if ((sc & 3) == 0) hrow[2 * (sc / 4 - 1) + 1] = e;
                if ((sc & 3) == 3) hrow[2 * (sc / 4 + 1)] = e;
            }
        }
        const int ecol = v == 0 ? x0 - 1 : x0 + TW;
        const T edge = (in_img && ecol >= 0 && ecol < W) ? sr.edge[u] : T(0);
        if (v == 0) hrow[0] = edge;
        if (v == VPR - 1) hrow[2 * (LW - 1) + 1] = edge;
    }

    static __device__ __forceinline__ void stage(const T* x, T* tile, const int* rowtab, int c0, int ccn, int trn,
                                                 uint32_t trn_magic, int x0, int W, int hw, int tid, int nthreads) {
        // Everything derived from the thread index is the same for every chunk; recomputing it is a
        // few integer instructions, keeping it live across the multiply-accumulate loop would cost
        // a dozen registers.  The empty asm makes the index opaque so that it is recomputed.
        asm volatile("" : "+v"(tid));
        const int total = ccn * trn * VPR;
        const T* xc0 = x + (int64_t)c0 * hw;
        StageRegs<T> sr;
        for (int i0 = tid; i0 < total; i0 += 2 * nthreads) {
            load(sr, 0, i0, total, xc0, rowtab, trn, trn_magic, x0, W, hw);
            load(sr, 1, i0 + nthreads, total, xc0, rowtab, trn, trn_magic, x0, W, hw);
            store(sr, 0, i0, total, tile, rowtab, trn, trn_magic, x0, W);
            store(sr, 1, i0 + nthreads, total, tile, rowtab, trn, trn_magic, x0, W);
        }
    }
};

// Run the staging routine with the vector width picked at launch time.
#define PPC_STAGE_DISPATCH(VECVAR, CALL)                                        \
    switch (VECVAR) {                                                           \
        case 8:                                                                 \
            if constexpr (sizeof(T) == 2 && LW % 2 == 0 && LW >= 4) { Stager<T, 8, LW, R>::CALL; } \
            break;                                                              \
        case 4: Stager<T, 4, LW, R>::CALL; break;                               \
        case 2: Stager<T, 2, LW, R>::CALL; break;                               \
        default: Stager<T, 1, LW, R>::CALL; break;                              \
    }

// Variants with at most 32 accumulators per lane are asked to fit 64 vector registers, i.e. 8
// resident wavefronts per SIMD: two 16-wavefront workgroups per CU, which is what hides the scalar
// dispatch and LDS latency of one behind the multiply-accumulates of the other.
template <typename T, int NP, int R, int F, int LW>
__global__ __launch_bounds__(1024) __attribute__((amdgpu_waves_per_eu(F * R * 4 <= 32 ? 8 : 4)))
void k1_tiled(const K1Args a) {
    constexpr TileGeom tg = tile_geom(LW, R, (int)sizeof(T));
    constexpr int TW = tg.tw, RS = tg.rs, CHS = tg.chs, ROWS = tg.rows, HOFF = tg.hoff;
    constexpr int EW = 8;                           // 32-bit words per stream entry
    extern __shared__ __align__(16) unsigned char smem_raw[];
    __shared__ int rowtab[ROWS];
    T* tile = reinterpret_cast<T*>(smem_raw);

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nwaves = a.wf * a.ks;
    const int wfi = wave % a.wf, ksi = wave / a.wf;

    // Block -> work item.  Consecutive block ids are dealt round-robin to the 8 XCDs, each with
    // its own L2, so block id i is first turned into "slot i/8 of XCD i%8" and every XCD is given a
    // contiguous range of work items.  Work items are ordered filter block fastest, then strip,
    // then row band: workgroups that read the same input tile (other filter blocks) or its
    // edge columns (neighbouring strips) run on the same XCD at about the same time and find
    // those lines in its L2.
    const int per_xcd = a.blocks_per_xcd;
    int item = (int)(blockIdx.x % 8u) * per_xcd + (int)(blockIdx.x / 8u);
    if (item >= a.work_items) return;            // grid is rounded up to a multiple of 8
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

    const T* lane_mid = tile + lr * R * RS + 4 * mcol;
    const T* lane_halo = tile + lr * R * RS + HOFF + 2 * mcol;
    const int hw = a.h * a.w;
    const uint32_t trn_magic = 0xFFFFFFFFu / (uint32_t)trn + 1u;      // ceil(2^32 / trn), trn >= 3
    const T* __restrict__ xin = static_cast<const T*>(a.x);

    // this wavefront's entry stream (constant address space: wave-uniform loads from it are scalar loads)
    typedef const __attribute__((address_space(4))) uint32_t* stream_ptr_t;
    typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr_t;
    stream_ptr_t sp = (stream_ptr_t)(a.stream) + (int64_t)(has_group ? ((const_i32_ptr_t)a.wave_off)[g * a.ks + ksi] : 0) * EW;
    // the next entry to execute, fetched one entry ahead so that the scalar-load latency hides
    // behind the previous kernel's multiply-accumulates
    uint32_t n_head = sp[0], n_w0 = sp[4], n_w1 = sp[5], n_w2 = sp[6], n_w3 = sp[7];

    for (int q = 0; q < a.chunks; ++q) {
        const int c0 = q * a.cc;
        const int ccn = (a.c_in - c0 < a.cc) ? a.c_in - c0 : a.cc;
        __syncthreads();          // previous chunk fully consumed (and rowtab written, first time round)
        PPC_STAGE_DISPATCH(a.vec, stage(xin, tile, rowtab, c0, ccn, trn, trn_magic, x0, a.w, hw, threadIdx.x, blockDim.x))
        __syncthreads();
        if (!has_group) continue;

        Window<T, R> win;
        win.clear();
        for (;;) {
            const uint32_t head = n_head;
            const float wt[4] = {__builtin_bit_cast(float, n_w0), __builtin_bit_cast(float, n_w1),
                                 __builtin_bit_cast(float, n_w2), __builtin_bit_cast(float, n_w3)};
            const bool at_end = (head & kFlagEnd) != 0;
            if (!at_end && (head & kFlagNewChannel)) {
                const int cl = (int)(head >> kChanShift);
                win.load(lane_mid + cl * CHS, lane_halo + cl * CHS, RS);
                // Wait for the window here, before the next entry's scalar load is issued: LDS reads
                // and scalar loads share one counter, so a wait placed later (inside the kernel
                // blocks) would also wait for that prefetch and expose its latency on every kernel.
                // (0xC07F = lgkmcnt(0), vmcnt and expcnt unconstrained; the builtin, unlike inline
                // assembly, is visible to the compiler's own wait-count bookkeeping)
                __builtin_amdgcn_s_waitcnt(0xC07F);
            }
            sp += EW;                 // the stream is padded by one entry past the last wavefront
            n_head = sp[0];
            n_w0 = sp[4];
            n_w1 = sp[5];
            n_w2 = sp[6];
            n_w3 = sp[7];
            if (at_end) break;
            dispatch<T, R, F, NP, 0, F * NP>((int)(head & kCodeMask), acc, win, wt);
        }
    }

    // ---- sum the channel splits through LDS, in a fixed order (deterministic) ----
    if (a.ks > 1) {
        float* red = reinterpret_cast<float*>(smem_raw);      // [wf][F*R*4][64]
        for (int s = 1; s < a.ks; ++s) {
            __syncthreads();
            if (ksi == s) {
#pragma unroll
                for (int f = 0; f < F; ++f)
#pragma unroll
                    for (int rr = 0; rr < R; ++rr)
#pragma unroll
                        for (int k = 0; k < 4; ++k)
                            red[((wfi * F + f) * R * 4 + rr * 4 + k) * 64 + lane] = acc[f][rr][k];
            }
            __syncthreads();
            if (ksi == 0) {
#pragma unroll
                for (int f = 0; f < F; ++f)
#pragma unroll
                    for (int rr = 0; rr < R; ++rr)
#pragma unroll
                        for (int k = 0; k < 4; ++k)
                            acc[f][rr][k] += red[((wfi * F + f) * R * 4 + rr * 4 + k) * 64 + lane];
            }
        }
    }
    if (ksi != 0 || !has_group || mrow >= a.mrows) return;

    // ---- epilogue: bias, ReLU, store at the filter's original index ----
    T* __restrict__ yout = static_cast<T*>(a.y);
    const int xcol = x0 + 4 * mcol;
    if (xcol >= a.w) return;
    const bool vec_store = (a.w & 3) == 0;
#pragma unroll
    for (int rr = 0; rr < R; ++rr) {
        const int v = mrow * R + rr;
        if (v >= a.vh) continue;
        const int img = v / (a.h + 1), yy = v - img * (a.h + 1);
        if (yy >= a.h) continue;
#pragma unroll
        for (int f = 0; f < F; ++f) {
            const int co = a.perm_pad[g * F + f];
            if (co < 0) continue;
            const float bz = a.bias_pad[g * F + f];
            float o[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                o[k] = acc[f][rr][k] + bz;
                if (a.relu) o[k] = o[k] > 0.0f ? o[k] : 0.0f;
            }
            T* dst = yout + (((int64_t)img * a.c_out + co) * a.h + yy) * a.w + xcol;
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
                    if (xcol + k < a.w) dst[k] = (T)o[k];
            }
        }
    }
}

// Dynamic LDS bytes a launch needs: the tile, or the split-channel exchange area if larger.
inline int k1_lds_bytes(int lw, int r, int f, int wf, int ks, int cc, int elem_bytes) {
    TileGeom tg = tile_geom(lw, r, elem_bytes);
    int tile = cc * tg.chs * elem_bytes;
    int red = ks > 1 ? wf * f * r * 4 * 64 * 4 : 0;
    return tile > red ? tile : red;
}

typedef void (*k1_launch_fn)(const K1Args& a, int blocks, int threads, int lds_bytes, hipStream_t stream);
// Look up the instantiation for (dtype, np, r, f, lw); nullptr if that combination is not built.
k1_launch_fn k1_lookup(int dtype, int np, int r, int f, int lw);

}  // namespace ppc

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

// A lane's input window for one channel: rows 0..R+1, columns -1..4.
template <typename T, int R> struct Window {
    typename VecOf<T, 4>::type mid[R + 2];    // columns 0..3
    typename VecOf<T, 2>::type halo[R + 2];   // (column -1, column 4)
    template <int ROW, int COL> __device__ __forceinline__ float get() const {
        if constexpr (COL < 0) return (float)halo[ROW][0];
        else if constexpr (COL > 3) return (float)halo[ROW][1];
        else return (float)mid[ROW][COL];
    }
};

// ---------------------------------------------------------------------------------------------
// Multiply-accumulate block of one kept kernel: filter slot FS, pattern slot PS (4 taps).
template <typename T, int R, int F, int FS, int RR, int TAP>
__device__ __forceinline__ void mac_row(float (&acc)[F][R][4], const Window<T, R>& win, float wj) {
    constexpr int dr = TAP / 3, dc = TAP % 3 - 1;
    acc[FS][RR][0] = __builtin_fmaf(wj, win.template get<RR + dr, 0 + dc>(), acc[FS][RR][0]);
    acc[FS][RR][1] = __builtin_fmaf(wj, win.template get<RR + dr, 1 + dc>(), acc[FS][RR][1]);
    acc[FS][RR][2] = __builtin_fmaf(wj, win.template get<RR + dr, 2 + dc>(), acc[FS][RR][2]);
    acc[FS][RR][3] = __builtin_fmaf(wj, win.template get<RR + dr, 3 + dc>(), acc[FS][RR][3]);
}

template <typename T, int R, int F, int FS, int TAP>
__device__ __forceinline__ void mac_tap(float (&acc)[F][R][4], const Window<T, R>& win, float wj) {
    static_assert(R == 1 || R == 2, "rows per lane");
    mac_row<T, R, F, FS, 0, TAP>(acc, win, wj);
    if constexpr (R > 1) mac_row<T, R, F, FS, 1, TAP>(acc, win, wj);
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
// Stage the rows of one channel chunk into LDS (zero-filled outside the images), VEC elements
// per global load.  Interior columns go to [row][0..TW), and the elements that are some
// micro-tile's left/right neighbour are also written to that micro-tile's halo pair.
template <typename T, int VEC, int LW, int R>
__device__ __forceinline__ void stage_chunk(const T* __restrict__ x, T* tile, const int* rowtab, int c0, int ccn,
                                            int trn, int x0, int W, int64_t hw, int wave, int nwaves, int lane) {
    constexpr TileGeom tg = tile_geom(LW, R, (int)sizeof(T));
    constexpr int TW = tg.tw, VPR = TW / VEC, RS = tg.rs, CHS = tg.chs;
    constexpr int U = 2;
    typedef typename VecOf<T, VEC>::type vec_t;
    const int per_ch = trn * VPR;
    for (int c = wave; c < ccn; c += nwaves) {
        const T* xc = x + (int64_t)(c0 + c) * hw;
        T* tc = tile + c * CHS;
        for (int j0 = 0; j0 < per_ch; j0 += 64 * U) {
            vec_t reg[U];
            T edge_l[U], edge_r[U];
            int dst[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int j = j0 + u * 64 + lane;
                const int tr = j / VPR, v = j - tr * VPR;
                dst[u] = -1;
                reg[u] = vec_t(0);
                edge_l[u] = T(0);
                edge_r[u] = T(0);
                if (j < per_ch) {
                    dst[u] = tr * RS + v * VEC;
                    const int rb = rowtab[tr];
                    const int col = x0 + v * VEC;
                    if (rb >= 0) {
                        if (col < W) reg[u] = *reinterpret_cast<const vec_t*>(xc + (uint32_t)(rb + col));
                        if (v == 0 && x0 > 0) edge_l[u] = xc[(uint32_t)(rb + x0 - 1)];
                        if (v == VPR - 1 && x0 + TW < W) edge_r[u] = xc[(uint32_t)(rb + x0 + TW)];
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (dst[u] < 0) continue;
                const int j = j0 + u * 64 + lane;
                const int tr = j / VPR, v = j - tr * VPR;
                *reinterpret_cast<vec_t*>(tc + dst[u]) = reg[u];
                T* hrow = tc + tr * RS + TW;
#pragma unroll
                for (int i = 0; i < VEC; ++i) {
                    const int sc = v * VEC + i;
                    const T e = vec_elem<T, VEC>(reg[u], i);
                    if ((sc & 3) == 0 && sc >= 4) hrow[2 * (sc / 4 - 1) + 1] = e;
                    if ((sc & 3) == 3 && sc + 1 < TW) hrow[2 * (sc / 4 + 1)] = e;
                }
                if (v == 0) hrow[0] = edge_l[u];
                if (v == VPR - 1) hrow[2 * (LW - 1) + 1] = edge_r[u];
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
template <typename T, int NP, int R, int F, int LW>
__global__ __launch_bounds__(1024) void k1_tiled(const K1Args a) {
    constexpr TileGeom tg = tile_geom(LW, R, (int)sizeof(T));
    constexpr int TW = tg.tw, RS = tg.rs, CHS = tg.chs, ROWS = tg.rows;
    constexpr int EW = 8;                           // 32-bit words per stream entry
    extern __shared__ __align__(16) unsigned char smem_raw[];
    __shared__ int rowtab[ROWS];
    T* tile = reinterpret_cast<T*>(smem_raw);

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nwaves = a.wf * a.ks;
    const int wfi = wave % a.wf, ksi = wave / a.wf;

    // block -> (filter block [slowest: heavy filter groups are dispatched first], strip, range of micro-tiles)
    int bid = blockIdx.x;
    const int per_fb = a.strips * a.wg_per_strip;
    const int fb = bid / per_fb;
    bid -= fb * per_fb;
    const int strip = bid / a.wg_per_strip;
    const int b = bid - strip * a.wg_per_strip;
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
    const T* lane_halo = tile + lr * R * RS + TW + 2 * mcol;
    const int64_t hw = (int64_t)a.h * a.w;
    const T* __restrict__ xin = static_cast<const T*>(a.x);

    // this wavefront's entry stream
    // (constant address space: wave-uniform loads from it are scalar loads)
    typedef const __attribute__((address_space(4))) u32x4* stream_ptr_t;
    typedef const __attribute__((address_space(4))) int32_t* const_i32_ptr_t;
    const stream_ptr_t ent_base = (stream_ptr_t)(a.stream);
    int e = has_group ? ((const_i32_ptr_t)a.wave_off)[g * a.ks + ksi] : 0;
    u32x4 hd = ent_base[(int64_t)e * (EW / 4)];
    u32x4 wq = ent_base[(int64_t)e * (EW / 4) + 1];

    for (int q = 0; q < a.chunks; ++q) {
        const int c0 = q * a.cc;
        const int ccn = (a.c_in - c0 < a.cc) ? a.c_in - c0 : a.cc;
        __syncthreads();          // previous chunk fully consumed (and rowtab written, first time round)
        switch (a.vec) {
            case 8:
                if constexpr (sizeof(T) == 2 && LW % 2 == 0)
                    stage_chunk<T, 8, LW, R>(xin, tile, rowtab, c0, ccn, trn, x0, a.w, hw, wave, nwaves, lane);
                break;
            case 4: stage_chunk<T, 4, LW, R>(xin, tile, rowtab, c0, ccn, trn, x0, a.w, hw, wave, nwaves, lane); break;
            case 2: stage_chunk<T, 2, LW, R>(xin, tile, rowtab, c0, ccn, trn, x0, a.w, hw, wave, nwaves, lane); break;
            default: stage_chunk<T, 1, LW, R>(xin, tile, rowtab, c0, ccn, trn, x0, a.w, hw, wave, nwaves, lane); break;
        }
        __syncthreads();
        if (!has_group) continue;

        Window<T, R> win;
#pragma unroll
        for (int rr = 0; rr < R + 2; ++rr) {
            win.mid[rr] = typename VecOf<T, 4>::type(0);
            win.halo[rr] = typename VecOf<T, 2>::type(0);
        }
        for (;;) {
            const uint32_t head = __builtin_amdgcn_readfirstlane(hd[0]);
            float wt[4];
            wt[0] = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(wq[0]));
            wt[1] = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(wq[1]));
            wt[2] = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(wq[2]));
            wt[3] = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(wq[3]));
            const bool at_end = (head & kFlagEnd) != 0;
            if (!at_end && (head & kFlagNewChannel)) {
                const int cl = (int)(head >> kChanShift);
                const T* pm = lane_mid + cl * CHS;
                const T* ph = lane_halo + cl * CHS;
#pragma unroll
                for (int rr = 0; rr < R + 2; ++rr) {
                    win.mid[rr] = *reinterpret_cast<const typename VecOf<T, 4>::type*>(pm + rr * RS);
                    win.halo[rr] = *reinterpret_cast<const typename VecOf<T, 2>::type*>(ph + rr * RS);
                }
                // Wait for the window here, before the next entry's scalar load is issued: LDS reads
                // and scalar loads share one counter, so a wait placed later (inside the kernel
                // blocks) would also wait for that prefetch and expose its latency on every kernel.
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            }
            // prefetch the next entry (the stream is padded by one entry past the last wavefront)
            ++e;
            hd = ent_base[(int64_t)e * (EW / 4)];
            wq = ent_base[(int64_t)e * (EW / 4) + 1];
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

// Dynamic LDS bytes a launch needs.
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

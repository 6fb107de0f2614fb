// Deep reuse (paper, section 2.3.2): kernels and C ABI (include/pp_deep_reuse.h).
//
// Four launches per pass:
//   reuse_clear     representatives <- "none"
//   reuse_hash      one lane per neuron vector, segments fastest (a wavefront reads one contiguous stretch of x),
//                   hyperplanes in LDS; signature bits are signs of binary32 fused multiply-add chains; the
//                   lowest row of every cluster is elected with integer minimum atomics
//   reuse_products  P[s][g][:] = x[rep(s,g)][segment s] . W[segment s][:]
//   reuse_gather    y[i][:] = act(bias + sum_s P[s][sig(i,s)][:])
// Integer work (signatures, representatives) is deterministic; the float sums run in a fixed order.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <climits>
#include <cstdint>
#include <new>
#include <vector>

#include "pp_deep_reuse.h"

namespace {

constexpr int kMaxSeg = 32;

typedef const __attribute__((address_space(4))) float* const_f32;

__global__ __launch_bounds__(256) void reuse_clear(int32_t* rep, int count) {
    const int e = (int)(blockIdx.x * 256 + threadIdx.x);
    if (e < count) rep[e] = INT_MAX;
}

// One lane per neuron vector, segments fastest: consecutive lanes read consecutive runs of L floats of x, so a
// wavefront reads one contiguous stretch of memory (a lane per row, with the hyperplanes as wave-uniform scalar
// operands, was measured ten times slower: its loads are a cache line apart).  The hyperplanes of all segments
// sit in LDS, loaded once per workgroup, which then walks the neuron vectors with the stride of the grid; the
// segment pitch is H * L + 1 floats, so lanes on different segments use different banks.  A lane's signature
// bits are the signs of H chains of fused multiply-adds in ascending l.  The representative of a cluster is
// the lowest row: one integer minimum atomic per lane, skipped when the table already holds a row at least as
// low (the table only ever decreases, so a stale read can cost an atomic, never a wrong result).
template <int L>
__global__ __launch_bounds__(256) void reuse_hash(const float* __restrict__ x, const float* __restrict__ hyper, uint16_t* __restrict__ sig,
                                                  int32_t* __restrict__ rep, int n, int k, int hash_bits) {
    extern __shared__ __attribute__((aligned(16))) unsigned char reuse_smem[];
    float* hp = reinterpret_cast<float*>(reuse_smem);
    const int S = k / L, G = 1 << hash_bits, pitch = hash_bits * L + 1;
    for (int e = (int)threadIdx.x; e < S * hash_bits * L; e += 256) {
        const int s = e / (hash_bits * L);
        hp[s * pitch + (e - s * hash_bits * L)] = hyper[e];
    }
    __syncthreads();
    // a lane takes the same segment of RPL consecutive rows, so that every hyperplane value it reads from LDS serves RPL
    // neuron vectors; consecutive lanes take consecutive segments, so each of its loads is part of one contiguous row
    constexpr int RPL = 4;
    const uint32_t groups = (uint32_t)((n + RPL - 1) / RPL), total = groups * (uint32_t)S;      // below 2^31: n * k is
    for (uint32_t e = blockIdx.x * 256u + threadIdx.x; e < total; e += gridDim.x * 256u) {      // e = (i / RPL) * S + s
        const int i0 = (int)(e / (uint32_t)S) * RPL, s = (int)(e % (uint32_t)S);
        float xv[RPL][L];
#pragma unroll
        for (int j = 0; j < RPL; ++j) {
            const int i = i0 + j < n ? i0 + j : n - 1;                  // rows past the end repeat the last one (not stored)
            const float* src = x + (int64_t)i * k + s * L;
            if constexpr (L % 4 == 0) {
#pragma unroll
                for (int l = 0; l < L; l += 4) {
                    const float4 v = *reinterpret_cast<const float4*>(src + l);
                    xv[j][l] = v.x, xv[j][l + 1] = v.y, xv[j][l + 2] = v.z, xv[j][l + 3] = v.w;
                }
            } else {
#pragma unroll
                for (int l = 0; l < L; ++l) xv[j][l] = src[l];
            }
        }
        const float* h0 = hp + s * pitch;
        unsigned g[RPL];
#pragma unroll
        for (int j = 0; j < RPL; ++j) g[j] = 0;
        for (int h = 0; h < hash_bits; ++h) {
            float p[RPL];
#pragma unroll
            for (int j = 0; j < RPL; ++j) p[j] = 0.0f;
#pragma unroll
            for (int l = 0; l < L; ++l) {
                const float hv = h0[h * L + l];
#pragma unroll
                for (int j = 0; j < RPL; ++j) p[j] = __builtin_fmaf(xv[j][l], hv, p[j]);
            }
#pragma unroll
            for (int j = 0; j < RPL; ++j) g[j] |= (p[j] > 0.0f ? 1u : 0u) << h;
        }
#pragma unroll
        for (int j = 0; j < RPL; ++j) {
            const int i = i0 + j;
            if (i < n) {
                sig[(int64_t)i * S + s] = (uint16_t)g[j];
                int32_t* slot = rep + (int64_t)s * G + g[j];
                if (__builtin_nontemporal_load(slot) > i) atomicMin(slot, i);
            }
        }
    }
}

// grid (ceil(G * m / 256), S)
__global__ __launch_bounds__(256) void reuse_products(const float* __restrict__ x, const float* __restrict__ w, const int32_t* __restrict__ rep,
                                                      float* __restrict__ P, int k, int m, int L, int G) {
    const int s = (int)blockIdx.y, e = (int)(blockIdx.x * 256 + threadIdx.x);
    if (e >= G * m) return;
    const int g = e / m, c = e - g * m;
    const int r = rep[(int64_t)s * G + g];
    if (r == INT_MAX) return;                                       // an empty cluster: nobody reads its products
    float acc = 0.0f;
    for (int l = 0; l < L; ++l) acc = __builtin_fmaf(x[(int64_t)r * k + s * L + l], w[(int64_t)(s * L + l) * m + c], acc);
    P[((int64_t)s * G + g) * m + c] = acc;
}

// V output columns per lane (4 when m is a multiple of 4, else 1), columns fastest
template <int V>
__global__ __launch_bounds__(256) void reuse_gather(const uint16_t* __restrict__ sig, const float* __restrict__ P, const float* __restrict__ bias,
                                                    float* __restrict__ y, int n, int m, int S, int G, int relu) {
    const int mv = m / V;
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= (int64_t)n * mv) return;
    const int i = (int)(e / mv), c = (int)(e - (int64_t)i * mv) * V;
    float acc[V];
#pragma unroll
    for (int v = 0; v < V; ++v) acc[v] = bias[c + v];
    const uint16_t* srow = sig + (int64_t)i * S;
    for (int s = 0; s < S; ++s) {
        const float* p = P + ((int64_t)s * G + srow[s]) * m + c;
        if constexpr (V == 4) {
            const float4 v4 = *reinterpret_cast<const float4*>(p);
            acc[0] += v4.x, acc[1] += v4.y, acc[2] += v4.z, acc[3] += v4.w;
        } else {
            acc[0] += p[0];
        }
    }
#pragma unroll
    for (int v = 0; v < V; ++v)
        if (relu) acc[v] = acc[v] > 0.0f ? acc[v] : 0.0f;
    if constexpr (V == 4) {
        float4 o;
        o.x = acc[0], o.y = acc[1], o.z = acc[2], o.w = acc[3];
        *reinterpret_cast<float4*>(y + (int64_t)i * m + c) = o;
    } else {
        y[(int64_t)i * m + c] = acc[0];
    }
}

typedef void (*hash_fn)(const float*, const float*, uint16_t*, int32_t*, int, int, int);
template <int L> hash_fn pick_hash(int seg_len) {
    if constexpr (L == 0) return nullptr;
    else return seg_len == L ? reuse_hash<L> : pick_hash<L - 1>(seg_len);
}

}  // namespace

struct pp_reuse_plan {
    int k = 0, m = 0, L = 0, H = 0, n_max = 0;
    uint32_t flags = 0;
    bool on_device = false;
    float* d_w = nullptr;
    float* d_bias = nullptr;
    float* d_hyper = nullptr;
    uint16_t* d_sig = nullptr;
    int32_t* d_rep = nullptr;
    float* d_P = nullptr;
};

namespace {

void release(pp_reuse_plan_t* p) {
    void* bufs[] = {p->d_w, p->d_bias, p->d_hyper, p->d_sig, p->d_rep, p->d_P};
    for (void* b : bufs)
        if (b) (void)hipFree(b);
}

template <typename T>
bool put(T** dst, const void* src, size_t bytes) {
    void* p = nullptr;
    if (hipMalloc(&p, bytes + 16) != hipSuccess) return false;
    *dst = static_cast<T*>(p);
    if (hipMemset(p, 0, bytes + 16) != hipSuccess) return false;
    return !src || hipMemcpy(p, src, bytes, hipMemcpyHostToDevice) == hipSuccess;
}

}  // namespace

extern "C" {

pp_status_t pp_reuse_plan(const pp_reuse_desc_t* d, pp_reuse_plan_t** out_plan) {
    if (out_plan) *out_plan = nullptr;
    if (!d || !out_plan || !d->weights || !d->hyperplanes) return PP_ERR_NULL;
    if (d->k < 1 || d->m < 1 || d->n_max < 1 || d->seg_len < 1 || d->seg_len > kMaxSeg || d->k % d->seg_len != 0 || d->hash_bits < 1 ||
        d->hash_bits > 12)
        return PP_ERR_SHAPE;
    if ((int64_t)d->n_max * std::max(d->k, d->m) >= ((int64_t)1 << 31) || (int64_t)d->k * d->m >= ((int64_t)1 << 31)) return PP_ERR_SHAPE;
    if (d->flags & ~(uint32_t)(PP_FLAG_RELU | PP_FLAG_HOST_ONLY)) return PP_ERR_UNSUPPORTED;
    // the hash kernel keeps every segment's hyperplanes in LDS (H * L + 1 floats per segment)
    if ((int64_t)(d->k / d->seg_len) * (d->hash_bits * d->seg_len + 1) * 4 > 64 * 1024) return PP_ERR_UNSUPPORTED;
    pp_reuse_plan_t* p = new (std::nothrow) pp_reuse_plan_t();
    if (!p) return PP_ERR_ALLOC;
    p->k = d->k, p->m = d->m, p->L = d->seg_len, p->H = d->hash_bits, p->n_max = d->n_max, p->flags = d->flags;
    if (!(d->flags & PP_FLAG_HOST_ONLY)) {
        const int S = d->k / d->seg_len, G = 1 << d->hash_bits;
        std::vector<float> zero_bias;
        const float* bias = d->bias;
        if (!bias) {
            zero_bias.assign((size_t)d->m, 0.0f);
            bias = zero_bias.data();
        }
        bool ok = put(&p->d_w, d->weights, (size_t)d->k * d->m * 4) && put(&p->d_bias, bias, (size_t)d->m * 4) &&
                  put(&p->d_hyper, d->hyperplanes, (size_t)S * d->hash_bits * d->seg_len * 4) &&
                  put(&p->d_sig, nullptr, (size_t)S * d->n_max * 2) && put(&p->d_rep, nullptr, (size_t)S * G * 4) &&
                  put(&p->d_P, nullptr, (size_t)S * G * d->m * 4);
        if (!ok) {
            (void)hipGetLastError();
            release(p);
            delete p;
            return PP_ERR_DEVICE;
        }
        p->on_device = true;
    }
    *out_plan = p;
    return PP_OK;
}

pp_status_t pp_reuse_run(const pp_reuse_plan_t* p, const void* x_dev, void* y_dev, int32_t n, void* hip_stream) {
    if (!p || !x_dev || !y_dev) return PP_ERR_NULL;
    if (n < 1 || n > p->n_max) return PP_ERR_SHAPE;
    const uintptr_t xa = reinterpret_cast<uintptr_t>(x_dev), ya = reinterpret_cast<uintptr_t>(y_dev);
    if ((xa | ya) & 15u) return PP_ERR_ALIGN;
    const uintptr_t xe = xa + (uintptr_t)((int64_t)n * p->k * 4), ye = ya + (uintptr_t)((int64_t)n * p->m * 4);
    if (xa < ye && ya < xe) return PP_ERR_ALIGN;
    if (!p->on_device) return PP_ERR_UNSUPPORTED;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int S = p->k / p->L, G = 1 << p->H;
    const float* x = static_cast<const float*>(x_dev);
    float* y = static_cast<float*>(y_dev);
    const hash_fn hash = pick_hash<kMaxSeg>(p->L);
    if (!hash) return PP_ERR_UNSUPPORTED;
    (void)hipGetLastError();
    hipLaunchKernelGGL(reuse_clear, dim3((unsigned)((S * G + 255) / 256)), dim3(256), 0, stream, p->d_rep, S * G);
    const size_t lds = (size_t)S * (p->H * p->L + 1) * 4;
    const int64_t hash_blocks = std::min<int64_t>(((int64_t)((n + 3) / 4) * S + 255) / 256, 256 * 8);      // at most eight workgroups per compute unit
    hipLaunchKernelGGL(hash, dim3((unsigned)hash_blocks), dim3(256), lds, stream, x, p->d_hyper, p->d_sig, p->d_rep, n, p->k, p->H);
    hipLaunchKernelGGL(reuse_products, dim3((unsigned)((G * p->m + 255) / 256), (unsigned)S), dim3(256), 0, stream, x, p->d_w, p->d_rep, p->d_P, p->k,
                       p->m, p->L, G);
    const int relu = (p->flags & PP_FLAG_RELU) ? 1 : 0;
    if (p->m % 4 == 0) {
        const int64_t lanes = (int64_t)n * (p->m / 4);
        hipLaunchKernelGGL(reuse_gather<4>, dim3((unsigned)((lanes + 255) / 256)), dim3(256), 0, stream, p->d_sig, p->d_P, p->d_bias, y, n, p->m, S, G, relu);
    } else {
        const int64_t lanes = (int64_t)n * p->m;
        hipLaunchKernelGGL(reuse_gather<1>, dim3((unsigned)((lanes + 255) / 256)), dim3(256), 0, stream, p->d_sig, p->d_P, p->d_bias, y, n, p->m, S, G, relu);
    }
    return hipGetLastError() == hipSuccess ? PP_OK : PP_ERR_DEVICE;
}

pp_status_t pp_reuse_read_clusters(const pp_reuse_plan_t* p, int32_t n, uint16_t* sig_out, int32_t* rep_out) {
    if (!p) return PP_ERR_NULL;
    if (n < 1 || n > p->n_max) return PP_ERR_SHAPE;
    if (!p->on_device) return PP_ERR_UNSUPPORTED;
    if (hipDeviceSynchronize() != hipSuccess) return PP_ERR_DEVICE;
    const int S = p->k / p->L, G = 1 << p->H;
    try {
        if (sig_out) {
            if (hipMemcpy(sig_out, p->d_sig, (size_t)n * S * 2, hipMemcpyDeviceToHost) != hipSuccess) return PP_ERR_DEVICE;
        }
        if (rep_out) {
            if (hipMemcpy(rep_out, p->d_rep, (size_t)S * G * 4, hipMemcpyDeviceToHost) != hipSuccess) return PP_ERR_DEVICE;
            for (size_t e = 0; e < (size_t)S * G; ++e)
                if (rep_out[e] == INT_MAX) rep_out[e] = -1;
        }
    } catch (const std::bad_alloc&) {
        return PP_ERR_ALLOC;
    }
    return PP_OK;
}

pp_status_t pp_reuse_destroy(pp_reuse_plan_t* p) {
    if (!p) return PP_OK;
    release(p);
    delete p;
    return PP_OK;
}

}  // extern "C"

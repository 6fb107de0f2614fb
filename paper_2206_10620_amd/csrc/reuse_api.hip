// Deep reuse (paper, section 2.3.2): kernels and C ABI (include/pp_deep_reuse.h).
//
// Four launches per pass:
//   reuse_clear     representatives <- "none"
//   reuse_hash      one lane per row and segment: the L values go through LDS (read from memory in runs of L
//                   consecutive floats, then one row per lane), the hyperplanes are wave-uniform scalar loads;
//                   signature bits are signs of binary32 fused multiply-add chains; the lowest row of every
//                   cluster is elected with integer minimum atomics, first inside the workgroup's LDS table,
//                   then one global atomic per cluster the workgroup touched
//   reuse_products  P[s][g][:] = x[rep(s,g)][segment s] . W[segment s][:]
//   reuse_gather    y[i][:] = act(bias + sum_s P[s][sig(i,s)][:])
// Integer work (signatures, representatives) is deterministic; the float sums run in a fixed order.
#include <hip/hip_runtime.h>

#include <climits>
#include <cstdint>
#include <new>
#include <vector>

#include "pp_deep_reuse.h"

namespace {

constexpr int kRows = 256;          // rows per workgroup of reuse_hash
constexpr int kMaxSeg = 32;

typedef const __attribute__((address_space(4))) float* const_f32;

__global__ __launch_bounds__(256) void reuse_clear(int32_t* rep, int count) {
    const int e = (int)(blockIdx.x * 256 + threadIdx.x);
    if (e < count) rep[e] = INT_MAX;
}

template <int L>
__device__ __forceinline__ unsigned hash_row(const float* xv, const_f32 hp, int hash_bits) {
    unsigned g = 0;
    for (int h = 0; h < hash_bits; ++h) {
        float p = 0.0f;
#pragma unroll
        for (int l = 0; l < L; ++l) p = __builtin_fmaf(xv[l], hp[h * L + l], p);
        g |= (p > 0.0f ? 1u : 0u) << h;
    }
    return g;
}

// grid (ceil(n / 256)); dynamic LDS: 256 * (L + 1) floats + 2^H ints
template <int L>
__global__ __launch_bounds__(256) void reuse_hash(const float* __restrict__ x, const float* __restrict__ hyper, uint16_t* __restrict__ sig,
                                                  int32_t* __restrict__ rep, int n, int k, int hash_bits, int n_max) {
    extern __shared__ __attribute__((aligned(16))) unsigned char reuse_smem[];
    float* tile = reinterpret_cast<float*>(reuse_smem);                         // [256][L + 1]
    int32_t* table = reinterpret_cast<int32_t*>(tile + kRows * (L + 1));        // [2^H]
    const int t = (int)threadIdx.x, i0 = (int)blockIdx.x * kRows, i = i0 + t;
    const int S = k / L, G = 1 << hash_bits;
    const int rows_here = n - i0 < kRows ? n - i0 : kRows;
    const const_f32 hp_all = (const_f32)(uintptr_t)hyper;
    for (int s = 0; s < S; ++s) {
        for (int g = t; g < G; g += 256) table[g] = INT_MAX;
        for (int e = t; e < rows_here * L; e += 256) {
            const int row = e / L, l = e - row * L;
            tile[row * (L + 1) + l] = x[(int64_t)(i0 + row) * k + s * L + l];
        }
        __syncthreads();
        if (i < n) {
            float xv[L];
#pragma unroll
            for (int l = 0; l < L; ++l) xv[l] = tile[t * (L + 1) + l];
            const unsigned g = hash_row<L>(xv, hp_all + (int64_t)s * hash_bits * L, hash_bits);
            sig[(int64_t)s * n_max + i] = (uint16_t)g;
            atomicMin(&table[g], i);
        }
        __syncthreads();
        for (int g = t; g < G; g += 256) {
            const int v = table[g];
            if (v != INT_MAX) atomicMin(&rep[(int64_t)s * G + g], v);
        }
        __syncthreads();
    }
}

// grid (ceil(G * m / 256), S)
__global__ __launch_bounds__(256) void reuse_products(const float* __restrict__ x, const float* __restrict__ w, const int32_t* __restrict__ rep,
                                                      float* __restrict__ P, int k, int m, int L, int G) {
    const int s = (int)blockIdx.y, e = (int)(blockIdx.x * 256 + threadIdx.x);
    if (e >= G * m) return;
    const int g = e / m, c = e - g * m;
    const int r = rep[(int64_t)s * G + g];
    float acc = 0.0f;
    if (r != INT_MAX)
        for (int l = 0; l < L; ++l) acc = __builtin_fmaf(x[(int64_t)r * k + s * L + l], w[(int64_t)(s * L + l) * m + c], acc);
    P[((int64_t)s * G + g) * m + c] = acc;
}

// one lane per output element, columns fastest
__global__ __launch_bounds__(256) void reuse_gather(const uint16_t* __restrict__ sig, const float* __restrict__ P, const float* __restrict__ bias,
                                                    float* __restrict__ y, int n, int m, int S, int G, int n_max, int relu) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= (int64_t)n * m) return;
    const int i = (int)(e / m), c = (int)(e - (int64_t)i * m);
    float acc = bias[c];
    for (int s = 0; s < S; ++s) acc += P[((int64_t)s * G + sig[(int64_t)s * n_max + i]) * m + c];
    if (relu) acc = acc > 0.0f ? acc : 0.0f;
    y[e] = acc;
}

typedef void (*hash_fn)(const float*, const float*, uint16_t*, int32_t*, int, int, int, int);
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
    const size_t lds = (size_t)kRows * (p->L + 1) * 4 + (size_t)G * 4;
    hipLaunchKernelGGL(hash, dim3((unsigned)((n + kRows - 1) / kRows)), dim3(256), lds, stream, x, p->d_hyper, p->d_sig, p->d_rep, n, p->k, p->H, p->n_max);
    hipLaunchKernelGGL(reuse_products, dim3((unsigned)((G * p->m + 255) / 256), (unsigned)S), dim3(256), 0, stream, x, p->d_w, p->d_rep, p->d_P, p->k,
                       p->m, p->L, G);
    const int64_t outs = (int64_t)n * p->m;
    hipLaunchKernelGGL(reuse_gather, dim3((unsigned)((outs + 255) / 256)), dim3(256), 0, stream, p->d_sig, p->d_P, p->d_bias, y, n, p->m, S, G,
                       p->n_max, (p->flags & PP_FLAG_RELU) ? 1 : 0);
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
            std::vector<uint16_t> tmp((size_t)S * p->n_max);
            if (hipMemcpy(tmp.data(), p->d_sig, tmp.size() * 2, hipMemcpyDeviceToHost) != hipSuccess) return PP_ERR_DEVICE;
            for (int i = 0; i < n; ++i)
                for (int s = 0; s < S; ++s) sig_out[(size_t)i * S + s] = tmp[(size_t)s * p->n_max + i];
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

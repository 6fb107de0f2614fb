// C ABI of the library (declared in include/pp_conv.h): plan creation and upload, kernel
// selection and launch, the generic any-pattern kernel and the 2x2 max-pool helper.
#include <hip/hip_runtime.h>

#include <cstring>
#include <new>
#include <vector>

#include "k1_tiled.hpp"
#include "k2_mfma.hpp"
#include "k3_mfma_direct.hpp"
#include "block_plan.hpp"
#include "plan.hpp"
#include "pp_block_gemm.h"
#include "pp_conv.h"

namespace ppc {

k1_launch_fn k1_lookup_f32_p8_r1(int f, int lw, bool direct);
k1_launch_fn k1_lookup_f32_p8_r2(int f, int lw, bool direct);
k1_launch_fn k1_lookup_f32_p8_r4(int f, int lw, bool direct);
k1_launch_fn k1_lookup_f32_p16_r1(int f, int lw, bool direct);
k1_launch_fn k1_lookup_f32_p16_r2(int f, int lw, bool direct);
k1_launch_fn k1_lookup_f32_p16_r4(int f, int lw, bool direct);
k1_launch_fn k1_lookup_f16_p8_r1(int f, int lw, bool direct);
k1_launch_fn k1_lookup_f16_p8_r2(int f, int lw, bool direct);
k1_launch_fn k1_lookup_f16_p8_r4(int f, int lw, bool direct);
k1_launch_fn k1_lookup_f16_p16_r1(int f, int lw, bool direct);
k1_launch_fn k1_lookup_f16_p16_r2(int f, int lw, bool direct);
k1_launch_fn k1_lookup_f16_p16_r4(int f, int lw, bool direct);

k2_launch_fn k2_lookup_k1(int stride, int ntw, int waves, bool pairs);
k2_launch_fn k2_lookup_k3(int stride, int ntw, int waves, bool pairs);
k2_launch_fn k2_lookup_k5(int stride, int ntw, int waves, bool pairs);
k2_launch_fn k2_lookup_k7(int stride, int ntw, int waves, bool pairs);

k2_launch_fn k2_lookup(int ks, int stride, int ntw, int waves, bool pairs) {
    switch (ks) {
        case 1: return k2_lookup_k1(stride, ntw, waves, pairs);
        case 3: return k2_lookup_k3(stride, ntw, waves, pairs);
        case 5: return k2_lookup_k5(stride, ntw, waves, pairs);
        case 7: return k2_lookup_k7(stride, ntw, waves, pairs);
        default: return nullptr;
    }
}

k1_launch_fn k1_lookup(int dtype, int np, int r, int f, int lw, bool direct) {
#define PPC_PICK(DT, NP)                                   \
    switch (r) {                                           \
        case 1: return k1_lookup_##DT##_p##NP##_r1(f, lw, direct); \
        case 2: return k1_lookup_##DT##_p##NP##_r2(f, lw, direct); \
        case 4: return k1_lookup_##DT##_p##NP##_r4(f, lw, direct); \
        default: return nullptr;                           \
    }
    if (dtype == PP_F32) {
        if (np == 8) { PPC_PICK(f32, 8) }
        PPC_PICK(f32, 16)
    }
    if (np == 8) { PPC_PICK(f16, 8) }
    PPC_PICK(f16, 16)
#undef PPC_PICK
}

// ---------------------------------------------------------------------------------------------
// Generic kernel: any pattern table, kernel size, stride, with or without the fused 2x2 max-pool.
// One lane per stored output, one filter per blockIdx.y; walks the filter's reordered kernel list
// (same-pattern kernels consecutive) with wave-uniform indices and reads the input straight from
// global memory with bounds checks.  It is the correctness path for layers the fast kernels do not
// take, not a fast path.
struct K0Args {
    const void* x;
    void* y;
    const int32_t* filt_off;   // [c_out+1]
    const int32_t* kidx;       // [k_kept]
    const uint8_t* kpat;       // [k_kept]
    const float* w;            // [k_kept*taps] (binary16-rounded values for an fp16 plan)
    const int8_t* tap_dyx;     // [P*taps*2]
    const int32_t* perm;       // [c_out]
    const float* bias;         // [c_out] by original index
    int32_t n, c_in, c_out, h, w_, taps, relu;
    int32_t stride, ho, wo, out_h, out_w, pool;
};

template <typename T>
__global__ __launch_bounds__(256) void k0_generic(const K0Args a) {
    const int pos = blockIdx.y;
    const int64_t pix = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t ohw = (int64_t)a.out_h * a.out_w;
    if (pix >= (int64_t)a.n * ohw) return;
    const int img = (int)(pix / ohw);
    const int rem = (int)(pix - (int64_t)img * ohw);
    const int sy = rem / a.out_w, sx = rem - sy * a.out_w;      // stored output
    const int64_t hw = (int64_t)a.h * a.w_;
    const T* __restrict__ x = static_cast<const T*>(a.x);
    const int co = a.perm[pos];
    const int beg = a.filt_off[pos], end = a.filt_off[pos + 1];
    const int np = a.pool ? 2 : 1;
    float best = 0.0f;
    for (int py = 0; py < np; ++py)
        for (int px = 0; px < np; ++px) {
            const int oy = sy * np + py, ox = sx * np + px;     // the convolution's own output
            float acc = 0.0f;
            for (int e = beg; e < end; ++e) {
                const int ci = a.kidx[e];
                const int8_t* tp = a.tap_dyx + (int)a.kpat[e] * a.taps * 2;
                const float* wv = a.w + (int64_t)e * a.taps;
                const T* xc = x + ((int64_t)img * a.c_in + ci) * hw;
                for (int j = 0; j < a.taps; ++j) {
                    const int iy = oy * a.stride + tp[2 * j], ix = ox * a.stride + tp[2 * j + 1];
                    if (iy >= 0 && iy < a.h && ix >= 0 && ix < a.w_) acc = __builtin_fmaf(wv[j], (float)xc[iy * a.w_ + ix], acc);
                }
            }
            acc += a.bias[co];
            if (a.relu) acc = acc > 0.0f ? acc : 0.0f;
            const float v = (float)(T)acc;                      // pooling acts on stored values
            best = (py == 0 && px == 0) ? v : (v > best ? v : best);
        }
    static_cast<T*>(a.y)[((int64_t)img * a.c_out + co) * ohw + rem] = (T)best;
}

template <typename T>
__global__ __launch_bounds__(256) void maxpool2x2(const T* __restrict__ x, T* __restrict__ y, int64_t planes, int h, int w) {
    const int ho = h / 2, wo = w / 2;
    const int64_t total = planes * ho * wo;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256) {
        const int ox = (int)(i % wo);
        const int64_t t = i / wo;
        const int oy = (int)(t % ho);
        const int64_t p = t / ho;
        const T* s = x + (p * h + 2 * oy) * w + 2 * ox;
        const float a0 = (float)s[0], a1 = (float)s[1], a2 = (float)s[w], a3 = (float)s[w + 1];
        const float m0 = a0 > a1 ? a0 : a1, m1 = a2 > a3 ? a2 : a3;
        y[i] = (T)(m0 > m1 ? m0 : m1);
    }
}

__global__ __launch_bounds__(256) void fill_zero_i32(int32_t* p, int count) {
    const int i = (int)(blockIdx.x * 256 + threadIdx.x);
    if (i < count) p[i] = 0;
}

}  // namespace ppc

using namespace ppc;

// Device memory for pp_conv_run_static, the entry point that allocates nothing: the arrival counters
// (first kScratchCounterBytes) and the partial sums of a plan that splits channels across workgroups.
// Every GPU the library runs on holds its own copy at its own address until the process ends; in
// host code the array's name is only a handle for hipGetSymbolAddress, never a device address.
constexpr size_t kScratchBytes = (size_t)32 << 20;
constexpr size_t kScratchCounterBytes = (size_t)64 << 10;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};

// The address of `scratch` on the current device, looked up once per device.
hipError_t scratch_address(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}
}  // namespace

struct pp_conv_plan {
    HostPlan hp;
    bool on_device = false;
    // tiled kernel
    uint32_t* d_stream = nullptr;
    int32_t* d_wave_off = nullptr;
    int32_t* d_perm_pad = nullptr;
    int32_t* d_chan_map = nullptr;
    float* d_ws = nullptr;             // partial sums of a plan that splits channels across workgroups
    int32_t* d_counters = nullptr;     // arrivals per output tile (zero between launches)
    float* d_bias_pad = nullptr;
    k1_launch_fn launch = nullptr;
    // matrix-core kernel
    uint16_t* d_wpk = nullptr;
    float* d_bias_mfma = nullptr;
    k2_launch_fn launch2 = nullptr;
    k3_launch_fn launch3 = nullptr;
    k3_launch_fn launch3_split = nullptr;     // the same kernel storing partial sums of a share of the chunks
    float* d_ws3 = nullptr;                   // their workspace: [ksplit][n_hint][c_out][h][w] binary32
    pp_block_gemm_plan_t* pointwise = nullptr; // a 1x1 stride-1 layer in binary16 runs as a batch of matrix products (one per image)
    _Float16* d_xpad = nullptr;               // x with zero channels appended up to whole chunks of 16: [n_hint][cpad][h][w]
    // generic kernel
    int32_t* d_filt_off = nullptr;
    int32_t* d_kidx = nullptr;
    uint8_t* d_kpat = nullptr;
    float* d_w = nullptr;
    int8_t* d_tap = nullptr;
    int32_t* d_perm = nullptr;
    float* d_bias = nullptr;
};

namespace {

template <typename T>
bool upload(T** dst, const void* src, size_t bytes) {
    if (bytes == 0) bytes = 16;
    if (hipMalloc(reinterpret_cast<void**>(dst), bytes) != hipSuccess) {
        *dst = nullptr;
        return false;
    }
    if (src && hipMemcpy(*dst, src, bytes, hipMemcpyHostToDevice) != hipSuccess) return false;
    return true;
}

void free_device(pp_conv_plan_t* p) {
    void* bufs[] = {p->d_xpad, p->d_ws3, p->d_stream, p->d_wave_off, p->d_chan_map, p->d_ws, p->d_counters, p->d_perm_pad, p->d_bias_pad, p->d_wpk, p->d_bias_mfma, p->d_filt_off, p->d_kidx,
                    p->d_kpat,   p->d_w,        p->d_tap,      p->d_perm,     p->d_bias};
    for (void* b : bufs)
        if (b) (void)hipFree(b);
}

int staging_vec(int w, int tw, int elem_bytes) {
    int v = 16 / elem_bytes;
    while (v > 1 && (w % v != 0 || tw % v != 0 || tw / v < 2)) v /= 2;
    return v;
}

}  // namespace

extern "C" {

const char* pp_status_string(pp_status_t s) {
    switch (s) {
        case PP_OK: return "ok";
        case PP_ERR_NULL: return "null pointer";
        case PP_ERR_SHAPE: return "bad shape";
        case PP_ERR_PATTERN: return "bad pattern mask or id";
        case PP_ERR_UNSUPPORTED: return "unsupported request";
        case PP_ERR_ALLOC: return "host allocation failed";
        case PP_ERR_DEVICE: return "device error";
        case PP_ERR_ALIGN: return "misaligned or overlapping device buffers";
        case PP_ERR_SCRATCH: return "request exceeds the static scratch buffer";
    }
    return "unknown status";
}

// pp_conv_plan with tuning.autotune = 1: the execution parameters that section 2.3.1 leaves to tuning are
// decided by measurement.  A short list of candidates (the rules' own choice first, then the alternatives
// that have won on some layer: the other workgroup size and tile shapes of the matrix-core kernels, the
// other kernel, rows per lane and channel splits of the vector kernel) is planned, each plan is timed on
// scratch buffers of n_hint images on a stream of its own, and the fastest is kept.
static pp_status_t plan_autotuned(const pp_conv_desc_t* desc, pp_conv_plan_t** out_plan) {
    pp_conv_tuning_t base = *desc->tuning;
    base.autotune = 0;
    std::vector<pp_conv_tuning_t> cands;
    cands.push_back(base);
    auto add = [&](auto&& edit) {
        pp_conv_tuning_t t = base;
        edit(t);
        cands.push_back(t);
    };
    const bool f16 = desc->dtype == PP_F16;
    if (f16 && (base.variant == 0 || base.variant == 3)) {
        if (base.mfma_kind != 1) {
            for (int waves : {4, 8})
                for (int cols : {0, 60, 28})
                    if (!base.wg_waves && !base.tile_cols && !base.tile_rows)
                        add([&](pp_conv_tuning_t& t) { t.variant = 3, t.mfma_kind = 2, t.wg_waves = waves, t.tile_cols = cols; });
        }
        if (base.mfma_kind != 1 && !base.split_k)
            for (int k : {1, 2, 4})
                add([&](pp_conv_tuning_t& t) { t.variant = 3, t.mfma_kind = 2, t.split_k = k; });
        if (base.mfma_kind == 0) add([&](pp_conv_tuning_t& t) { t.variant = 3, t.mfma_kind = 1; });
    }
    if (base.variant == 0 || base.variant == 2) {
        if (f16 && base.variant == 0) add([&](pp_conv_tuning_t& t) { t.variant = 2; });
        if (!f16 || base.variant == 2)
            for (int r : {1, 2})
                for (int ks : {1, 2, 4})
                    if (!base.rows_per_lane && !base.split_c)
                        add([&](pp_conv_tuning_t& t) { t.variant = 2, t.rows_per_lane = r, t.split_c = ks; });
    }
    const int n = desc->n_hint > 0 ? desc->n_hint : 1;
    pp_conv_plan_t* best = nullptr;
    float best_ms = 0.0f;
    void *x = nullptr, *y = nullptr;
    hipStream_t stream = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    pp_status_t first_err = PP_ERR_UNSUPPORTED;
    bool device_ok = true;
    std::vector<pp_conv_tuning_t> timed;
    for (const pp_conv_tuning_t& t : cands) {
        pp_conv_desc_t d = *desc;
        d.tuning = &t;
        pp_conv_plan_t* p = nullptr;
        const pp_status_t st = pp_conv_plan(&d, &p);
        if (st != PP_OK) {
            if (&t == &cands[0]) first_err = st;
            if (st == PP_ERR_DEVICE || st == PP_ERR_ALLOC) {      // not a matter of the candidate
                first_err = st;
                device_ok = false;
                break;
            }
            continue;
        }
        bool seen = false;                                        // candidates that come to the same parameters are timed once
        for (const pp_conv_tuning_t& c : timed) seen = seen || std::memcmp(&c, &p->hp.chosen, sizeof c) == 0;
        if (seen) {
            pp_conv_destroy(p);
            continue;
        }
        timed.push_back(p->hp.chosen);
        if (!x) {
            const HostPlan& hp = p->hp;
            const size_t eb = hp.dtype == PP_F16 ? 2 : 4;
            const size_t xb = (size_t)n * hp.c_in * hp.h * hp.w * eb, yb = (size_t)n * hp.c_out * hp.out_h * hp.out_w * eb;
            device_ok = hipMalloc(&x, xb) == hipSuccess && hipMalloc(&y, yb) == hipSuccess &&
                        hipMemset(x, hp.dtype == PP_F16 ? 0x34 : 0x3c, xb) == hipSuccess &&     // finite values of moderate size in either type
                        hipStreamCreate(&stream) == hipSuccess && hipEventCreate(&e0) == hipSuccess && hipEventCreate(&e1) == hipSuccess;
            if (!device_ok) {
                pp_conv_destroy(p);
                first_err = PP_ERR_DEVICE;
                break;
            }
        }
        float ms = 1e30f;
        bool ok = true;
        for (int i = 0; i < 3 && ok; ++i) ok = pp_conv_run(p, x, y, n, stream) == PP_OK;
        for (int round = 0; round < 2 && ok; ++round) {
            ok = hipEventRecord(e0, stream) == hipSuccess;
            for (int i = 0; i < 10 && ok; ++i) ok = pp_conv_run(p, x, y, n, stream) == PP_OK;
            float r = 0.0f;
            ok = ok && hipEventRecord(e1, stream) == hipSuccess && hipEventSynchronize(e1) == hipSuccess &&
                 hipEventElapsedTime(&r, e0, e1) == hipSuccess;
            if (ok && r < ms) ms = r;
        }
        if (ok && (!best || ms < best_ms)) {
            if (best) pp_conv_destroy(best);
            best = p;
            best_ms = ms;
        } else {
            pp_conv_destroy(p);
        }
    }
    if (stream) (void)hipStreamSynchronize(stream);
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    if (stream) (void)hipStreamDestroy(stream);
    if (x) (void)hipFree(x);
    if (y) (void)hipFree(y);
    (void)hipGetLastError();
    if (!best) return first_err;
    best->hp.chosen.autotune = 1;
    *out_plan = best;
    return PP_OK;
}

pp_status_t pp_conv_plan(const pp_conv_desc_t* desc, pp_conv_plan_t** out_plan) {
    if (out_plan) *out_plan = nullptr;
    if (!desc || !out_plan) return PP_ERR_NULL;
    pp_status_t st = validate(*desc);
    if (st != PP_OK) return st;
    if (desc->tuning && desc->tuning->autotune != 0) {
        if (desc->tuning->autotune != 1) return PP_ERR_UNSUPPORTED;
        // a host-only plan has no device to measure on: the rules decide
        if (!(desc->flags & PP_FLAG_HOST_ONLY)) return plan_autotuned(desc, out_plan);
    }
    pp_conv_plan_t* p = new (std::nothrow) pp_conv_plan_t();
    if (!p) return PP_ERR_ALLOC;
    try {
        build_canonical(*desc, p->hp);
        st = build_layouts(*desc, p->hp);
    } catch (const std::bad_alloc&) {
        st = PP_ERR_ALLOC;
    }
    if (st != PP_OK) {
        delete p;
        return st;
    }
    HostPlan& hp = p->hp;
    if (hp.tiled) {
        p->launch = k1_lookup(hp.dtype, hp.tl.np, hp.tl.r, hp.tl.f, hp.tl.lw, hp.tl.mode != 0);
        if (!p->launch) {
            delete p;
            return PP_ERR_UNSUPPORTED;
        }
    } else if (hp.mfma) {
        if (hp.ml.direct) {
            p->launch3 = k3_lookup(hp.ml.g3.sw, hp.ml.g3.waves, false, hp.pool);
            if (hp.ml.ksplit > 1) p->launch3_split = k3_lookup(hp.ml.g3.sw, hp.ml.g3.waves, true, false);
        }
        else p->launch2 = k2_lookup(hp.ks, hp.stride, hp.ml.ntw, hp.ml.waves, hp.ml.pairs);
        if (!p->launch2 && !p->launch3) {
            delete p;
            return PP_ERR_UNSUPPORTED;
        }
    } else if (hp.c_out > 65535) {
        delete p;
        return PP_ERR_UNSUPPORTED;
    }
    // A 1x1, stride-1 layer is y_n = W x_n per image, with x_n = [c_in][h*w] as it lies in memory: the matrix-core
    // kernel of the block-pruned product runs it, connectivity pruning being its column pruning with 1 x 1 blocks.
    const int want_kind = desc->tuning ? desc->tuning->mfma_kind : 0;
    const bool pointwise_ok = hp.mfma && hp.ks == 1 && hp.stride == 1 && !hp.pool && hp.taps == 1 && (hp.h * hp.w) % 8 == 0 && !(desc->tuning && desc->tuning->split_k > 1);
    if (want_kind == 3 && !pointwise_ok) {
        delete p;
        return PP_ERR_UNSUPPORTED;
    }
    if (pointwise_ok && (want_kind == 0 || want_kind == 3)) {
        pp_block_gemm_desc_t bd{};
        bd.m = hp.c_out, bd.k = hp.c_in, bd.block_m = 1, bd.block_k = 1;
        bd.row_keep = nullptr;
        bd.col_keep = desc->conn_mask;          // [c_out][c_in]: block (co, ci) keeps its one column or not
        bd.weights = desc->weights;             // one weight per kernel: [c_out][c_in]
        bd.bias = desc->bias;
        bd.flags = desc->flags & (PP_FLAG_RELU | PP_FLAG_HOST_ONLY);
        bd.dtype = PP_F16;
        bd.variant = 2;
        const pp_status_t bst = pp_block_gemm_plan(&bd, &p->pointwise);
        if (bst != PP_OK) {
            delete p;
            return bst;
        }
        hp.chosen.mfma_kind = 3;
        hp.chosen.tile_rows = hp.chosen.tile_cols = hp.chosen.tiles_per_wave = 0;
        hp.chosen.wg_waves = 4;
        hp.chosen.split_k = 0;
    }
    if (desc->flags & PP_FLAG_HOST_ONLY) {
        *out_plan = p;
        return PP_OK;
    }
    bool ok = true;
    if (hp.tiled) {
        const TiledLayout& tl = hp.tl;
        ok = ok && upload(&p->d_stream, tl.stream.data(), tl.stream.size() * 4);
        ok = ok && upload(&p->d_wave_off, tl.wave_off.data(), tl.wave_off.size() * 4);
        ok = ok && upload(&p->d_perm_pad, tl.perm_pad.data(), tl.perm_pad.size() * 4);
        ok = ok && upload(&p->d_chan_map, tl.chan_map.data(), tl.chan_map.size() * 4);
        if (tl.sw > 1) {
            // workspace and arrival counters for batches of up to n_hint images
            const int nh = std::max(1, hp.n_hint), eb = hp.dtype == PP_F16 ? 2 : 4;
            const TileGeom tg = tile_geom(tl.lw, tl.r, eb);
            const int64_t mrows = ((int64_t)nh * (hp.h + 1) - 1 + tl.r - 1) / tl.r;
            const int64_t tiles = ((hp.w + tg.tw - 1) / tg.tw) * ((mrows * tl.lw + 63) / 64) * ((tl.groups + tl.wf - 1) / tl.wf);
            const int64_t ws_bytes = (int64_t)tl.sw * nh * hp.c_out * hp.h * hp.w * 4;
            ok = ok && hipMalloc(reinterpret_cast<void**>(&p->d_ws), (size_t)ws_bytes) == hipSuccess;
            ok = ok && hipMalloc(reinterpret_cast<void**>(&p->d_counters), (size_t)tiles * 4) == hipSuccess;
            ok = ok && hipMemset(p->d_counters, 0, (size_t)tiles * 4) == hipSuccess;
        }
        ok = ok && upload(&p->d_bias_pad, tl.bias_pad.data(), tl.bias_pad.size() * 4);
    } else if (hp.mfma) {
        ok = ok && upload(&p->d_wpk, hp.ml.wpk.data(), hp.ml.wpk.size() * 2);
        ok = ok && upload(&p->d_bias_mfma, hp.ml.bias_pad.data(), hp.ml.bias_pad.size() * 4);
        if (hp.ml.direct && hp.ml.cpad != hp.c_in)   // zero-padded copy of x (the padding is zeroed here, once)
            ok = ok && upload(&p->d_xpad, nullptr, (size_t)std::max(1, hp.n_hint) * hp.ml.cpad * hp.h * hp.w * 2) &&
                 hipMemset(p->d_xpad, 0, (size_t)std::max(1, hp.n_hint) * hp.ml.cpad * hp.h * hp.w * 2) == hipSuccess;
        if (hp.ml.direct && hp.ml.ksplit > 1)   // the shares' partial sums, for up to n_hint images
            ok = ok && upload(&p->d_ws3, nullptr, (size_t)hp.ml.ksplit * std::max(1, hp.n_hint) * hp.c_out * hp.h * hp.w * 4);
    } else {
        const Canonical& cn = hp.canon;
        std::vector<float> w = cn.wpacked;
        if (hp.dtype == PP_F16)
            for (float& v : w) v = f16_to_f32(f32_to_f16_rne(v));
        ok = ok && upload(&p->d_filt_off, hp.filt_off.data(), hp.filt_off.size() * 4);
        ok = ok && upload(&p->d_kidx, cn.kidx.data(), cn.kidx.size() * 4);
        ok = ok && upload(&p->d_kpat, cn.kpat.data(), cn.kpat.size());
        ok = ok && upload(&p->d_w, w.data(), w.size() * 4);
        ok = ok && upload(&p->d_tap, hp.tap_dyx.data(), hp.tap_dyx.size());
        ok = ok && upload(&p->d_perm, cn.perm.data(), cn.perm.size() * 4);
        ok = ok && upload(&p->d_bias, hp.bias.data(), hp.bias.size() * 4);
    }
    if (!ok) {
        free_device(p);
        delete p;
        (void)hipGetLastError();
        return PP_ERR_DEVICE;
    }
    {   // set-up is the place to look up this device's copy of the static scratch array
        void* unused = nullptr;
        if (scratch_address(&unused) != hipSuccess) (void)hipGetLastError();
    }
    p->on_device = true;
    *out_plan = p;
    return PP_OK;
}

// One launch of the tiled kernel on n images.
static pp_status_t launch_tiled(const pp_conv_plan_t* plan, const void* x_dev, void* y_dev, int32_t n, hipStream_t stream,
                                float* ws, int32_t* counters) {
    const HostPlan& hp = plan->hp;
    const int relu = (hp.flags & PP_FLAG_RELU) ? 1 : 0;
    const TiledLayout& tl = hp.tl;
    const int eb = hp.dtype == PP_F16 ? 2 : 4;
    const TileGeom tg = tile_geom(tl.lw, tl.r, eb);
    K1Args a{};
    a.x = x_dev;
    a.y = y_dev;
    a.stream = plan->d_stream;
    a.wave_off = plan->d_wave_off;
    a.idle_off = tl.idle_off;
    a.bias_pad = plan->d_bias_pad;
    a.perm_pad = plan->d_perm_pad;
    a.chan_map = plan->d_chan_map;
    a.n = n;
    a.c_in = hp.c_in;
    a.c_out = hp.c_out;
    a.h = hp.h;
    a.w = hp.w;
    a.vh = n * (hp.h + 1) - 1;
    a.mrows = (a.vh + tl.r - 1) / tl.r;
    a.wg_per_strip = (int)(((int64_t)a.mrows * tl.lw + 63) / 64);
    a.strips = (hp.w + tg.tw - 1) / tg.tw;
    a.groups = tl.groups;
    a.wf = tl.wf;
    a.wf_recip = 65536 / tl.wf + 1;
    a.ks = tl.ks;
    a.cc = tl.cc;
    a.chunks = tl.chunks;
    a.vec = staging_vec(hp.w, tg.tw, eb);
    a.mode = tl.mode;
    a.nbuf = tl.nbuf;
    a.table_offset = k1_lds_table_offset(tl.lw, tl.r, tl.cc, eb, tl.nbuf);
    a.relu = relu;
    const int nfb = (tl.groups + tl.wf - 1) / tl.wf;
    const int64_t items = (int64_t)a.strips * a.wg_per_strip * nfb * tl.sw;
    if (items >= ((int64_t)1 << 30)) return PP_ERR_SHAPE;
    a.split_wg = tl.sw;
    a.out_elems = (int32_t)((int64_t)n * hp.c_out * hp.h * hp.w);
    a.ws = ws;
    a.counters = counters;
    a.nfb = nfb;
    a.work_items = (int)items;
    a.blocks_per_xcd = (int)((items + 7) / 8);
    const int64_t blocks = (int64_t)a.blocks_per_xcd * 8;
    const int lds = (int)k1_lds_layout_bytes(tl.lw, tl.r, tl.f, tl.wf, tl.ks, tl.cc, eb, tl.mode, tl.nbuf);
    a.red_par = tl.ks > 1 ? std::max(1, std::min(tl.ks - 1, lds / (tl.wf * tl.f * tl.r * 4 * 64 * 4))) : 1;
    (void)hipGetLastError();          // an error left by the caller's earlier HIP work is not this launch's
    plan->launch(a, (int)blocks, 64 * tl.wf * tl.ks, lds, stream);
    return hipGetLastError() == hipSuccess ? PP_OK : PP_ERR_DEVICE;
}

// Argument checks shared by the run entry points; nothing here touches a device.
static pp_status_t check_run_args(const pp_conv_plan_t* plan, const void* x_dev, const void* y_dev, int32_t n) {
    if (!plan || !x_dev || !y_dev) return PP_ERR_NULL;
    const HostPlan& hp = plan->hp;
    if (n <= 0) return PP_ERR_SHAPE;
    const int64_t hw = (int64_t)hp.h * hp.w, ohw = (int64_t)hp.out_h * hp.out_w;
    if ((int64_t)n * hp.c_in * hw >= ((int64_t)1 << 31) || (int64_t)n * hp.c_out * hp.ho * hp.wo >= ((int64_t)1 << 31) ||
        (int64_t)n * (hp.h + 8) >= ((int64_t)1 << 30))
        return PP_ERR_SHAPE;
    // the kernels use 128-bit loads and stores: a misaligned or aliased buffer must become a status
    // code here, not a memory fault on the device
    const int64_t ebytes = hp.dtype == PP_F16 ? 2 : 4;
    const uintptr_t xa = reinterpret_cast<uintptr_t>(x_dev), ya = reinterpret_cast<uintptr_t>(y_dev);
    if ((xa | ya) & 15u) return PP_ERR_ALIGN;
    const uintptr_t xe = xa + (uintptr_t)((int64_t)n * hp.c_in * hw * ebytes), ye = ya + (uintptr_t)((int64_t)n * hp.c_out * ohw * ebytes);
    if (xa < ye && ya < xe) return PP_ERR_ALIGN;
    if (!plan->on_device) return PP_ERR_UNSUPPORTED;
    return PP_OK;
}

static pp_status_t launch_generic(const pp_conv_plan_t* plan, const void* x_dev, void* y_dev, int32_t n, hipStream_t stream) {
    const HostPlan& hp = plan->hp;
    const int64_t ohw = (int64_t)hp.out_h * hp.out_w;
    const int relu = (hp.flags & PP_FLAG_RELU) ? 1 : 0;
    K0Args a{x_dev, y_dev, plan->d_filt_off, plan->d_kidx, plan->d_kpat, plan->d_w, plan->d_tap, plan->d_perm,
             plan->d_bias, n, hp.c_in, hp.c_out, hp.h, hp.w, hp.taps, relu,
             hp.stride, hp.ho, hp.wo, hp.out_h, hp.out_w, hp.pool ? 1 : 0};
    const int64_t blocks = ((int64_t)n * ohw + 255) / 256;
    if (blocks >= ((int64_t)1 << 31)) return PP_ERR_SHAPE;
    dim3 grid((unsigned)blocks, (unsigned)hp.c_out);
    (void)hipGetLastError();
    if (hp.dtype == PP_F16) hipLaunchKernelGGL(k0_generic<_Float16>, grid, dim3(256), 0, stream, a);
    else hipLaunchKernelGGL(k0_generic<float>, grid, dim3(256), 0, stream, a);
    return hipGetLastError() == hipSuccess ? PP_OK : PP_ERR_DEVICE;
}

// One launch of the direct-load matrix-core kernel on n images.
// Adds the shares' partial sums in share order, then bias, activation and the rounding to binary16.
__global__ __launch_bounds__(256) void k3_sum_shares(const float* __restrict__ ws, const float* __restrict__ bias, _Float16* __restrict__ y, int ksplit,
                                                     int64_t slab_elems, int c_out, int hw, int relu) {
    const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= slab_elems) return;
    float acc = bias[(int)((e / hw) % c_out)];
    for (int k = 0; k < ksplit; ++k) acc += ws[(int64_t)k * slab_elems + e];
    if (relu) acc = acc > 0.0f ? acc : 0.0f;
    y[e] = (_Float16)acc;
}

// Copies the c_in channels of every image into the first c_in of cpad channels (the others were zeroed when the
// plan was made and are never written): 16 bytes per lane when an image plane is a multiple of 8 elements.
__global__ __launch_bounds__(256) void k3_pad_channels(const _Float16* __restrict__ x, _Float16* __restrict__ xp, int64_t total, int chw, int cpad_hw, int v) {
    const int64_t e = ((int64_t)blockIdx.x * 256 + threadIdx.x) * v;       // element of x; v = 8 or 1 elements per lane
    if (e >= total) return;
    const int64_t img = e / chw;
    const int64_t o = img * cpad_hw + (e - img * chw);
    if (v == 8) *reinterpret_cast<uint4*>(xp + o) = *reinterpret_cast<const uint4*>(x + e);
    else xp[o] = x[e];
}

static pp_status_t launch_mfma_direct(const pp_conv_plan_t* plan, const void* x_dev, void* y_dev, int32_t n, hipStream_t stream, bool may_split) {
    const HostPlan& hp = plan->hp;
    const MfmaLayout& ml = hp.ml;
    const K3Geom& g = ml.g3;
    const int cpad = ml.cpad;
    if (cpad != hp.c_in) {
        // the padded copy holds n_hint images: larger batches go through it a group at a time
        const int group = std::max(1, hp.n_hint);
        if (n > group) {
            for (int n0 = 0; n0 < n; n0 += group) {
                const pp_status_t st = launch_mfma_direct(plan, static_cast<const _Float16*>(x_dev) + (int64_t)n0 * hp.c_in * hp.h * hp.w,
                                                          static_cast<_Float16*>(y_dev) + (int64_t)n0 * hp.c_out * hp.out_h * hp.out_w, std::min(group, n - n0), stream, may_split);
                if (st != PP_OK) return st;
            }
            return PP_OK;
        }
        const int hw = hp.h * hp.w;
        const int64_t total = (int64_t)n * hp.c_in * hw;
        (void)hipGetLastError();
        const int v = hw % 8 == 0 ? 8 : 1;
        hipLaunchKernelGGL(k3_pad_channels, dim3((unsigned)((total / v + 255) / 256)), dim3(256), 0, stream, static_cast<const _Float16*>(x_dev), plan->d_xpad, total,
                           hp.c_in * hw, cpad * hw, v);
        if (hipGetLastError() != hipSuccess) return PP_ERR_DEVICE;
        x_dev = plan->d_xpad;
    }
    K3Args a{};
    a.x = x_dev;
    a.y = y_dev;
    a.wpk = plan->d_wpk;
    a.bias = plan->d_bias_mfma;
    a.n = n;
    a.c_in = cpad;
    a.c_out = hp.c_out;
    a.h = hp.h;
    a.w = hp.w;
    a.po = ml.po;
    a.vrows = (n - 1) * ml.po + hp.h;
    a.out_h = hp.out_h;
    a.out_w = hp.out_w;
    a.tr = g.tr;
    a.nseg = g.nseg;
    const int valid = g.sw - 2;
    a.tiles_x = (hp.w + g.nseg * valid - 1) / (g.nseg * valid);
    a.tiles_v = (a.vrows + g.tr - 1) / g.tr;
    a.fb = ml.fb;
    a.q = ml.q;
    // the reduction is split when the plan says so, its workspace is large enough and the caller allows it
    const bool split = may_split && ml.ksplit > 1 && plan->launch3_split && plan->d_ws3 && n <= std::max(1, hp.n_hint);
    a.ksplit = split ? ml.ksplit : 1;
    a.qs = ml.q / a.ksplit;
    a.ws = split ? plan->d_ws3 : nullptr;
    a.slab_elems = (int64_t)n * hp.c_out * hp.h * hp.w;
    const int64_t items = (int64_t)a.tiles_x * a.tiles_v * ml.fb * a.ksplit;
    // piece offsets are 32-bit byte offsets (+16) from a chunk's first element
    if (items >= ((int64_t)1 << 30) || (int64_t)n * cpad * hp.h * hp.w >= ((int64_t)1 << 31) - 16) return PP_ERR_SHAPE;
    a.work_items = (int)items;
    a.blocks_per_xcd = (int)((items + 7) / 8);
    a.chs = g.chs;
    a.ppc = g.ppc;
    a.ppcp = g.ppcp;
    a.nxi = g.nxi;
    a.xbuf_bytes = g.xbuf_bytes;
    auto magic = [](int d) -> uint32_t { return d <= 1 ? 0u : (uint32_t)((((uint64_t)1) << 32) / (uint64_t)d + 1u); };
    a.magic_ppcp = magic(g.ppcp);
    a.magic_ppr = magic(g.nseg * (g.segb / 16));
    a.magic_nseg = magic(g.nseg);
    a.magic_po = magic(ml.po);
    // the index arithmetic divides by multiplication, exact below 65536
    if (ml.po + g.trp >= 65536) return PP_ERR_SHAPE;
    if (a.qs < k3_stages(g.waves) - 1) return PP_ERR_UNSUPPORTED;      // the kernel's pipeline fill stays inside the first work item
    a.relu = (hp.flags & PP_FLAG_RELU) ? 1 : 0;
    a.x_elems = (int64_t)n * cpad * hp.h * hp.w;
    (void)hipGetLastError();
    // persistent workgroups: as many as are resident at once (16 wavefronts of this kernel per compute unit), fewer
    // if the layer has fewer tiles
    const int grid = std::min(a.blocks_per_xcd * 8, 256 * 8 / g.waves);
    if (!split) {
        plan->launch3(a, grid, g.lds_bytes, stream);
        return hipGetLastError() == hipSuccess ? PP_OK : PP_ERR_DEVICE;
    }
    plan->launch3_split(a, grid, g.lds_bytes, stream);
    if (hipGetLastError() != hipSuccess) return PP_ERR_DEVICE;
    hipLaunchKernelGGL(k3_sum_shares, dim3((unsigned)((a.slab_elems + 255) / 256)), dim3(256), 0, stream, plan->d_ws3, plan->d_bias_mfma,
                       static_cast<_Float16*>(y_dev), a.ksplit, a.slab_elems, hp.c_out, hp.h * hp.w, a.relu);
    return hipGetLastError() == hipSuccess ? PP_OK : PP_ERR_DEVICE;
}

// One launch of the matrix-core kernel on n images.
static pp_status_t launch_mfma(const pp_conv_plan_t* plan, const void* x_dev, void* y_dev, int32_t n, hipStream_t stream, bool may_split = true) {
    const HostPlan& hp = plan->hp;
    const MfmaLayout& ml = hp.ml;
    if (plan->pointwise)
        return pp_block_gemm_launch_batched(plan->pointwise, x_dev, y_dev, hp.h * hp.w, n, (int64_t)hp.c_in * hp.h * hp.w, (int64_t)hp.c_out * hp.h * hp.w, stream);
    if (ml.direct) return launch_mfma_direct(plan, x_dev, y_dev, n, stream, may_split);
    K2Args a{};
    a.x = x_dev;
    a.y = y_dev;
    a.wpk = plan->d_wpk;
    a.bias = plan->d_bias_mfma;
    a.n = n;
    a.c_in = hp.c_in;
    a.c_out = hp.c_out;
    a.h = hp.h;
    a.w = hp.w;
    a.ho = hp.ho;
    a.wo = hp.wo;
    a.out_h = hp.out_h;
    a.out_w = hp.out_w;
    a.po = ml.po;
    a.vrows = (n - 1) * ml.po + hp.ho;
    a.tr = ml.tr;
    a.tc = ml.tc;
    a.trp = ml.trp;
    a.twpa = ml.twpa;
    a.tiles_x = (hp.wo + ml.tc - 1) / ml.tc;
    a.tiles_v = (a.vrows + ml.tr - 1) / ml.tr;
    a.fb = ml.fb;
    a.q = ml.q;
    const int64_t items = (int64_t)a.tiles_x * a.tiles_v * ml.fb;
    if (items >= ((int64_t)1 << 30) || (int64_t)n * ml.po * hp.stride >= ((int64_t)1 << 30)) return PP_ERR_SHAPE;
    a.work_items = (int)items;
    a.blocks_per_xcd = (int)((items + 7) / 8);
    a.xbuf_bytes = ml.xbuf_bytes;
    a.out_pitch = ml.out_pitch;
    a.gw = ml.gw;
    a.bias_off = (int)ml.lds_bytes - kMfmaFilters * 4;
    a.stride_ = hp.stride;
    auto magic = [](int d) -> uint32_t { return d <= 1 ? 0u : (uint32_t)((((uint64_t)1) << 32) / (uint64_t)d + 1u); };
    const int store_cols = hp.pool ? ml.tc / 2 : ml.tc, store_rows = hp.pool ? ml.tr / 2 : ml.tr;
    a.magic_ppr = magic(ml.twpa / 2);
    a.magic_pi = magic(ml.po * hp.stride);
    a.magic_tc = magic(ml.tc);
    a.magic_po = magic(ml.po);
    a.magic_gpr = magic(store_cols / ml.gw);
    a.magic_srows = magic(store_rows);
    // the index arithmetic divides by multiplication, exact below 65536
    if (ml.po * hp.stride + ml.trp >= 65536 || ml.po + ml.tr >= 65536) return PP_ERR_SHAPE;
    a.relu = (hp.flags & PP_FLAG_RELU) ? 1 : 0;
    a.pool = hp.pool ? 1 : 0;
    (void)hipGetLastError();
    plan->launch2(a, a.blocks_per_xcd * 8, 64 * ml.waves, (int)ml.lds_bytes, stream);
    return hipGetLastError() == hipSuccess ? PP_OK : PP_ERR_DEVICE;
}

pp_status_t pp_conv_run(const pp_conv_plan_t* plan, const void* x_dev, void* y_dev, int32_t n, void* hip_stream) {
    const pp_status_t chk = check_run_args(plan, x_dev, y_dev, n);
    if (chk != PP_OK) return chk;
    const HostPlan& hp = plan->hp;
    const int64_t hw = (int64_t)hp.h * hp.w;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (hp.mfma) return launch_mfma(plan, x_dev, y_dev, n, stream);
    if (!hp.tiled) return launch_generic(plan, x_dev, y_dev, n, stream);
    // A plan that splits channels across workgroups owns a workspace for n_hint images: larger
    // batches go through it n_hint images at a time.
    const TiledLayout& tl = hp.tl;
    const int eb = hp.dtype == PP_F16 ? 2 : 4;
    const int step = tl.sw > 1 ? std::max(1, hp.n_hint) : n;
    for (int n0 = 0; n0 < n; n0 += step) {
        const int nb = std::min(step, n - n0);
        const pp_status_t st = launch_tiled(plan, static_cast<const char*>(x_dev) + (int64_t)n0 * hp.c_in * hw * eb,
                                            static_cast<char*>(y_dev) + (int64_t)n0 * hp.c_out * hw * eb, nb, stream,
                                            plan->d_ws, plan->d_counters);
        if (st != PP_OK) return st;
    }
    return PP_OK;
}

pp_status_t pp_conv_run_static(const pp_conv_plan_t* plan, const void* x_dev, void* y_dev, int32_t n, void* hip_stream) {
    const pp_status_t chk = check_run_args(plan, x_dev, y_dev, n);
    if (chk != PP_OK) return chk;
    const HostPlan& hp = plan->hp;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if (hp.mfma) return launch_mfma(plan, x_dev, y_dev, n, stream, false);      // no reduction split: that needs the plan's workspace
    if (!hp.tiled) return launch_generic(plan, x_dev, y_dev, n, stream);
    const TiledLayout& tl = hp.tl;
    if (tl.sw <= 1) return launch_tiled(plan, x_dev, y_dev, n, stream, nullptr, nullptr);
    // partial sums [sw][n][c_out][h][w] fp32 behind the arrival counters, one per output tile
    const int eb = hp.dtype == PP_F16 ? 2 : 4;
    const TileGeom tg = tile_geom(tl.lw, tl.r, eb);
    const int64_t mrows = ((int64_t)n * (hp.h + 1) - 1 + tl.r - 1) / tl.r;
    const int64_t tiles = ((hp.w + tg.tw - 1) / tg.tw) * ((mrows * tl.lw + 63) / 64) * ((tl.groups + tl.wf - 1) / tl.wf);
    const int64_t ws_bytes = (int64_t)tl.sw * n * hp.c_out * hp.h * hp.w * 4;
    if (tiles * 4 > (int64_t)kScratchCounterBytes || ws_bytes > (int64_t)(kScratchBytes - kScratchCounterBytes)) return PP_ERR_SCRATCH;
    void* base = nullptr;
    if (scratch_address(&base) != hipSuccess) {
        (void)hipGetLastError();
        return PP_ERR_DEVICE;
    }
    int32_t* counters = static_cast<int32_t*>(base);
    float* ws = reinterpret_cast<float*>(static_cast<unsigned char*>(base) + kScratchCounterBytes);
    // The array keeps whatever the last call left (a launch that did not complete leaves counts
    // behind): the counters of this call's tiles start at zero.  A kernel, not a memset, so that the
    // call can be recorded into a graph.
    (void)hipGetLastError();
    hipLaunchKernelGGL(fill_zero_i32, dim3((unsigned)((tiles + 255) / 256)), dim3(256), 0, stream, counters, (int)tiles);
    if (hipGetLastError() != hipSuccess) return PP_ERR_DEVICE;
    return launch_tiled(plan, x_dev, y_dev, n, stream, ws, counters);
}

pp_status_t pp_conv_destroy(pp_conv_plan_t* plan) {
    if (!plan) return PP_OK;
    if (plan->pointwise) (void)pp_block_gemm_destroy(plan->pointwise);
    free_device(plan);
    delete plan;
    return PP_OK;
}

pp_status_t pp_conv_plan_query(const pp_conv_plan_t* plan, pp_plan_info_t* out) {
    if (!plan || !out) return PP_ERR_NULL;
    const HostPlan& hp = plan->hp;
    out->c_out = hp.c_out;
    out->c_in = hp.c_in;
    out->num_patterns = hp.num_patterns;
    out->taps = hp.taps;
    out->out_h = hp.out_h;
    out->out_w = hp.out_w;
    out->k_kept = hp.canon.k_kept;
    out->perm = hp.canon.perm.data();
    out->kcount = hp.canon.kcount.data();
    out->pat_off = hp.canon.pat_off.data();
    out->kidx = hp.canon.kidx.data();
    out->kpat = hp.canon.kpat.data();
    out->wpacked = hp.canon.wpacked.data();
    out->chosen = hp.chosen;
    return PP_OK;
}

pp_status_t pp_conv_plan_unpack(const pp_conv_plan_t* plan, int32_t* kidx_out, uint8_t* kpat_out, float* w_out) {
    if (!plan || !kidx_out || !kpat_out || !w_out) return PP_ERR_NULL;
    try {
        return unpack_stream(plan->hp, kidx_out, kpat_out, w_out);
    } catch (const std::bad_alloc&) {
        return PP_ERR_ALLOC;
    }
}

pp_status_t pp_maxpool2x2_run(const void* x_dev, void* y_dev, int32_t n, int32_t c, int32_t h, int32_t w, int32_t dtype,
                              void* hip_stream) {
    if (!x_dev || !y_dev) return PP_ERR_NULL;
    if (n < 1 || c < 1 || h < 2 || w < 2 || (h & 1) || (w & 1)) return PP_ERR_SHAPE;
    if (dtype != PP_F32 && dtype != PP_F16) return PP_ERR_UNSUPPORTED;
    const int64_t planes = (int64_t)n * c;
    const int64_t total = planes * (h / 2) * (w / 2);
    int64_t blocks = (total + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    (void)hipGetLastError();
    if (dtype == PP_F16)
        hipLaunchKernelGGL(maxpool2x2<_Float16>, dim3((unsigned)blocks), dim3(256), 0, stream,
                           static_cast<const _Float16*>(x_dev), static_cast<_Float16*>(y_dev), planes, h, w);
    else
        hipLaunchKernelGGL(maxpool2x2<float>, dim3((unsigned)blocks), dim3(256), 0, stream,
                           static_cast<const float*>(x_dev), static_cast<float*>(y_dev), planes, h, w);
    return hipGetLastError() == hipSuccess ? PP_OK : PP_ERR_DEVICE;
}

}  // extern "C"

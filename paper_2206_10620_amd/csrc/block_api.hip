// C ABI of the block-pruned matrix product (include/pp_block_gemm.h): plan upload, launches.
#include <hip/hip_runtime.h>

#include <cstring>
#include <new>

#include "block_plan.hpp"
#include "k4_block_gemm.hpp"

struct pp_block_gemm_plan {
    ppc::BlockHostPlan hp;
    bool on_device = false;
    void* d_apk = nullptr;
    float* d_wc = nullptr;
    float* d_bias = nullptr;
    int32_t* d_tile_off = nullptr;
    int32_t* d_tile_cols = nullptr;
    int32_t* d_tile_len = nullptr;
};

namespace {

using namespace ppc;

template <typename T>
bool put(T** dst, const void* src, size_t bytes, size_t pad_bytes = 0) {
    void* p = nullptr;
    if (hipMalloc(&p, bytes + pad_bytes + 16) != hipSuccess) return false;
    *dst = static_cast<T*>(p);
    if (hipMemset(p, 0, bytes + pad_bytes + 16) != hipSuccess) return false;
    if (bytes && hipMemcpy(p, src, bytes, hipMemcpyHostToDevice) != hipSuccess) return false;
    return true;
}

void release(pp_block_gemm_plan_t* p) {
    void* bufs[] = {p->d_apk, p->d_wc, p->d_bias, p->d_tile_off, p->d_tile_cols, p->d_tile_len};
    for (void* b : bufs)
        if (b) (void)hipFree(b);
}

}  // namespace

pp_status_t pp_block_gemm_launch_batched(const pp_block_gemm_plan_t* plan, const void* x_dev, void* y_dev, int32_t n, int32_t batch, int64_t x_stride,
                                         int64_t y_stride, void* hip_stream) {
    if (!plan || !x_dev || !y_dev) return PP_ERR_NULL;
    const BlockHostPlan& hp = plan->hp;
    if (n < 1 || batch < 1 || (n % 8) != 0 || hp.dtype != PP_F16 || !plan->on_device) return PP_ERR_UNSUPPORTED;
    if ((int64_t)hp.k * n >= ((int64_t)1 << 31) || (int64_t)hp.m * n >= ((int64_t)1 << 31)) return PP_ERR_SHAPE;
    K4Args a;
    a.x = x_dev, a.y = y_dev, a.apk = plan->d_apk, a.bias = plan->d_bias;
    a.tile_off = plan->d_tile_off, a.tile_cols = plan->d_tile_cols;
    a.m = hp.m, a.n = n, a.row_tiles = hp.row_tiles;
    a.col_tiles = (n + kBlockColTile - 1) / kBlockColTile;
    const int64_t items = (int64_t)a.row_tiles * a.col_tiles * batch;
    if (items >= ((int64_t)1 << 28)) return PP_ERR_SHAPE;
    a.items = (int)items;
    a.per_xcd = (a.items + 7) / 8;
    a.relu = (hp.flags & PP_FLAG_RELU) ? 1 : 0;
    a.x_stride = x_stride, a.y_stride = y_stride;
    static const hipError_t lds_attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&k4_block_gemm), hipFuncAttributeMaxDynamicSharedMemorySize, kK4LdsBytes);
    (void)lds_attr;
    (void)hipGetLastError();
    hipLaunchKernelGGL(k4_block_gemm, dim3((unsigned)(a.per_xcd * 8)), dim3(256), kK4LdsBytes, static_cast<hipStream_t>(hip_stream), a);
    return hipGetLastError() == hipSuccess ? PP_OK : PP_ERR_DEVICE;
}

extern "C" {

pp_status_t pp_block_gemm_plan(const pp_block_gemm_desc_t* desc, pp_block_gemm_plan_t** out_plan) {
    if (out_plan) *out_plan = nullptr;
    if (!desc || !out_plan) return PP_ERR_NULL;
    pp_block_gemm_plan_t* p = nullptr;
    try {
        p = new pp_block_gemm_plan_t();
        const pp_status_t st = build_block_plan(*desc, p->hp);
        if (st != PP_OK) {
            delete p;
            return st;
        }
    } catch (const std::bad_alloc&) {
        delete p;
        return PP_ERR_ALLOC;
    }
    if (!(desc->flags & PP_FLAG_HOST_ONLY)) {
        const BlockHostPlan& hp = p->hp;
        bool ok = put(&p->d_wc, hp.wc.data(), hp.wc.size() * sizeof(float));
        ok = ok && put(&p->d_apk, hp.apk.data(), hp.apk.size() * sizeof(uint16_t));
        ok = ok && put(&p->d_bias, hp.bias.data(), hp.bias.size() * sizeof(float));
        ok = ok && put(&p->d_tile_off, hp.tile_off.data(), hp.tile_off.size() * sizeof(int32_t));
        ok = ok && put(&p->d_tile_cols, hp.tile_cols.data(), hp.tile_cols.size() * sizeof(int32_t), kBlockChunk * sizeof(int32_t));   // the kernel reads one chunk ahead
        ok = ok && put(&p->d_tile_len, hp.tile_len.data(), hp.tile_len.size() * sizeof(int32_t));
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

pp_status_t pp_block_gemm_run(const pp_block_gemm_plan_t* plan, const void* x_dev, void* y_dev, int32_t n, void* hip_stream) {
    if (!plan || !x_dev || !y_dev) return PP_ERR_NULL;
    const BlockHostPlan& hp = plan->hp;
    if (n < 1 || (int64_t)hp.k * n >= ((int64_t)1 << 31) || (int64_t)hp.m * n >= ((int64_t)1 << 31)) return PP_ERR_SHAPE;
    const int64_t eb = hp.dtype == PP_F16 ? 2 : 4;
    const uintptr_t xa = reinterpret_cast<uintptr_t>(x_dev), ya = reinterpret_cast<uintptr_t>(y_dev);
    if ((xa | ya) & 15u) return PP_ERR_ALIGN;
    const uintptr_t xe = xa + (uintptr_t)((int64_t)hp.k * n * eb), ye = ya + (uintptr_t)((int64_t)hp.m * n * eb);
    if (xa < ye && ya < xe) return PP_ERR_ALIGN;
    int variant = hp.variant;
    if (variant == 2 && (n % 8) != 0) {
        if (hp.forced) return PP_ERR_UNSUPPORTED;
        variant = 1;
    }
    if (!plan->on_device) return PP_ERR_UNSUPPORTED;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const int relu = (hp.flags & PP_FLAG_RELU) ? 1 : 0;
    (void)hipGetLastError();
    if (variant == 2) return pp_block_gemm_launch_batched(plan, x_dev, y_dev, n, 1, 0, 0, hip_stream);
    {
        const dim3 grid((unsigned)((n + 63) / 64), (unsigned)hp.row_tiles), block(64, 4);
        if (hp.row_tiles > 65535) return PP_ERR_SHAPE;
        if (hp.dtype == PP_F16)
            hipLaunchKernelGGL(k4_generic<_Float16>, grid, block, 0, stream, static_cast<const _Float16*>(x_dev), static_cast<_Float16*>(y_dev),
                               plan->d_wc, plan->d_bias, plan->d_tile_off, plan->d_tile_cols, plan->d_tile_len, hp.m, n, relu);
        else
            hipLaunchKernelGGL(k4_generic<float>, grid, block, 0, stream, static_cast<const float*>(x_dev), static_cast<float*>(y_dev), plan->d_wc,
                               plan->d_bias, plan->d_tile_off, plan->d_tile_cols, plan->d_tile_len, hp.m, n, relu);
    }
    return hipGetLastError() == hipSuccess ? PP_OK : PP_ERR_DEVICE;
}

pp_status_t pp_block_gemm_destroy(pp_block_gemm_plan_t* plan) {
    if (!plan) return PP_OK;
    release(plan);
    delete plan;
    return PP_OK;
}

pp_status_t pp_block_gemm_query(const pp_block_gemm_plan_t* plan, pp_block_gemm_info_t* out) {
    if (!plan || !out) return PP_ERR_NULL;
    const BlockHostPlan& hp = plan->hp;
    out->m = hp.m, out->k = hp.k, out->block_m = hp.bm, out->block_k = hp.bk;
    out->variant = hp.variant;
    out->row_tile = kBlockRowTile;
    out->row_tiles = hp.row_tiles;
    out->kept_weights = hp.kept_weights;
    out->executed_weights = hp.executed_weights;
    out->tile_off = hp.tile_off.data();
    out->tile_cols = hp.tile_cols.data();
    out->tile_len = hp.tile_len.data();
    return PP_OK;
}

pp_status_t pp_block_gemm_unpack(const pp_block_gemm_plan_t* plan, int32_t tile, float* w_out) {
    if (!plan || !w_out) return PP_ERR_NULL;
    return unpack_block_tile(plan->hp, tile, w_out);
}

}  // extern "C"

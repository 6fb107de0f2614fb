// Direct-load matrix-core kernel instantiations (segment widths 32 and 16) and their lookup.
#include "k3_mfma_direct.hpp"

namespace ppc {
namespace {

template <int SW>
void launch(const K3Args& a, int blocks, int lds_bytes, hipStream_t stream) {
    // the kernel may use more than the default 64 KB of dynamic LDS; set once per instantiation
    static const hipError_t lds_attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&k3_mfma<SW>),
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, kMfmaMaxDynamicLds);
    (void)lds_attr;
    hipLaunchKernelGGL((k3_mfma<SW>), dim3(blocks), dim3(64 * kK3Waves), lds_bytes, stream, a);
}

}  // namespace

k3_launch_fn k3_lookup(int sw) {
    if (sw == 32) return launch<32>;
    if (sw == 16) return launch<16>;
    return nullptr;
}

}  // namespace ppc

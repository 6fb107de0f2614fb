// Direct-load matrix-core kernel, split-reduction instantiations (partial sums to a workspace); a translation unit of
// their own so that they compile beside the others.
#include "k3_mfma_direct.hpp"

namespace ppc {
namespace {

template <int SW, int WAVES>
void launch(const K3Args& a, int blocks, int lds_bytes, hipStream_t stream) {
    // the kernel may use more than the default 64 KB of dynamic LDS; set once per instantiation
    static const hipError_t lds_attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&k3_mfma<SW, WAVES, true, false>),
                                                           hipFuncAttributeMaxDynamicSharedMemorySize, kMfmaMaxDynamicLds);
    (void)lds_attr;
    hipLaunchKernelGGL((k3_mfma<SW, WAVES, true, false>), dim3(blocks), dim3(64 * WAVES), lds_bytes, stream, a);
}

}  // namespace

k3_launch_fn k3_lookup_split(int sw, int waves) {
    if (sw == 32 && waves == 4) return launch<32, 4>;
    if (sw == 16 && waves == 4) return launch<16, 4>;
    if (sw == 32 && waves == 8) return launch<32, 8>;
    if (sw == 16 && waves == 8) return launch<16, 8>;
    return nullptr;
}

}  // namespace ppc

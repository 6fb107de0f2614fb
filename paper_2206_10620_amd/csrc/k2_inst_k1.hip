// Matrix-core kernel instantiations: 1x1 kernels.
#define PPC_KS 1
#define PPC_FN k2_lookup_k1
#include "k2_inst.inc"

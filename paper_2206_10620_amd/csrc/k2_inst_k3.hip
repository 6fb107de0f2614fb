// Matrix-core kernel instantiations: 3x3 kernels.
#define PPC_KS 3
#define PPC_FN k2_lookup_k3
#include "k2_inst.inc"

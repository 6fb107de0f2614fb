// Matrix-core kernel instantiations: 5x5 kernels.
#define PPC_KS 5
#define PPC_FN k2_lookup_k5
#include "k2_inst.inc"

// Matrix-core kernel instantiations: 7x7 kernels.
#define PPC_KS 7
#define PPC_FN k2_lookup_k7
#include "k2_inst.inc"

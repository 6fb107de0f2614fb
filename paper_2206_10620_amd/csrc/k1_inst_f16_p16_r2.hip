// Tiled-kernel instantiations: f16 storage, 16 pattern slots, 2 output row(s) per lane.
#define PPC_T _Float16
#define PPC_NP 16
#define PPC_R 2
#define PPC_FN k1_lookup_f16_p16_r2
#include "k1_inst.inc"

// Tiled-kernel instantiations: f16 storage, 8 pattern slots, 2 output row(s) per lane.
#define PPC_T _Float16
#define PPC_NP 8
#define PPC_R 2
#define PPC_FN k1_lookup_f16_p8_r2
#include "k1_inst.inc"

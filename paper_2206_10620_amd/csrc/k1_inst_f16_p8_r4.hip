// Tiled-kernel instantiations: f16 storage, 8 pattern slots, 4 output row(s) per lane.
#define PPC_T _Float16
#define PPC_NP 8
#define PPC_R 4
#define PPC_FN k1_lookup_f16_p8_r4
#include "k1_inst.inc"

// Tiled-kernel instantiations: f16 storage, 16 pattern slots, 4 output row(s) per lane.
#define PPC_T _Float16
#define PPC_NP 16
#define PPC_R 4
#define PPC_FN k1_lookup_f16_p16_r4
#include "k1_inst.inc"

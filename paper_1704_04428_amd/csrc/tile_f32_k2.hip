// Tile kernels: f32 operands, kernel side 2.
#define MCMK_KS 2
#define MCMK_BF16 0
#include "tile_inst.h"

// Tile kernels: f32 operands, kernel side 6.
#define MCMK_KS 6
#define MCMK_BF16 0
#include "tile_inst.h"

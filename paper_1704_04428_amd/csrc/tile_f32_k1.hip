// Tile kernels: f32 operands, kernel side 1.
#define MCMK_KS 1
#define MCMK_BF16 0
#include "tile_inst.h"

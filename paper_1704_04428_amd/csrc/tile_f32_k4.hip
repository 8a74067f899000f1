// Tile kernels: f32 operands, kernel side 4.
#define MCMK_KS 4
#define MCMK_BF16 0
#include "tile_inst.h"

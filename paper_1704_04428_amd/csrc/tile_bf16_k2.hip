// Tile kernels: bf16 operands, kernel side 2.
#define MCMK_KS 2
#define MCMK_BF16 1
#include "tile_inst.h"

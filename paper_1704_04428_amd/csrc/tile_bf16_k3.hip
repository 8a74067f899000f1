// Tile kernels: bf16 operands, kernel side 3.
#define MCMK_KS 3
#define MCMK_BF16 1
#include "tile_inst.h"

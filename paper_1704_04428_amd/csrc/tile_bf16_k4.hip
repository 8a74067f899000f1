// Tile kernels: bf16 operands, kernel side 4.
#define MCMK_KS 4
#define MCMK_BF16 1
#include "tile_inst.h"

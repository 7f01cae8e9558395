// bf16 convolution kernels, second part of the tile list.
#include "gemm_tiles.h"

TSG_DEFINE_MODE_PART(launch_bf16_conv_b, TSG_BF16_TILES_B, A_CONV, 0 TSG_BF16_TILES_A(TSG_COUNT_TILE))

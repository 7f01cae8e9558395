// fp32 convolution kernels, second part of the tile list.
#include "gemm_tiles.h"

TSG_DEFINE_MODE_PART(launch_f32_conv_b, TSG_F32_TILES_B, A_CONV, 0 TSG_F32_TILES_A(TSG_COUNT_TILE))

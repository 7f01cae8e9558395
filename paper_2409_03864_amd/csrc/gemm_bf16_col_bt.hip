// bfloat16 kernels, both operands stored transposed and read in place.
#include "gemm_tiles.h"

TSG_DEFINE_MODE(launch_bf16_col_bt, TSG_BF16_TILES, A_COL_BT)

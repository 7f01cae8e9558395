// fp32 kernels, both operands stored transposed and read in place.
#include "gemm_tiles.h"

TSG_DEFINE_MODE(launch_f32_col_bt, TSG_F32_TILES, A_COL_BT)

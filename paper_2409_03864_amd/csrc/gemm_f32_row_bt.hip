// fp32 kernels, A row-major, B stored transposed (N x K) and read in place.
#include "gemm_tiles.h"

TSG_DEFINE_MODE(launch_f32_row_bt, TSG_F32_TILES, A_ROW_BT)

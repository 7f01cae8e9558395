// bfloat16 kernels, A row-major, B stored transposed (N x K) and read in place.
#include "gemm_tiles.h"

TSG_DEFINE_MODE(launch_bf16_row_bt, TSG_BF16_TILES, A_ROW_BT)

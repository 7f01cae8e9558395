// bfloat16 kernels, op(A)(i,k) = A[k*lda + i] (transposed left operand read in place).
#include "gemm_tiles.h"

TSG_DEFINE_MODE(launch_bf16_col, TSG_BF16_TILES, A_COL)

// fp32 kernels, op(A)(i,k) = A[k*lda + i] (transposed left operand read in place).
#include "gemm_tiles.h"

TSG_DEFINE_MODE(launch_f32_col, TSG_F32_TILES, A_COL)

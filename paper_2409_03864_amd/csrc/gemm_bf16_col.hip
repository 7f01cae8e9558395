// bf16 kernels, transposed left operand read in place: op(A)(i,k) = A[k*lda + i].
#include "gemm_bf16_kernel.h"

TSG_BF16_DEFINE_MODE(launch_bf16_col, A_COL)

// fp32 kernels, transposed left operand read in place: op(A)(i,k) = A[k*lda + i].
#include "gemm_f32_kernel.h"

TSG_F32_DEFINE_MODE(launch_f32_col, A_COL)

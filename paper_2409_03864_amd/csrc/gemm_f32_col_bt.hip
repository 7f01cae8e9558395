// fp32 kernels, both operands stored transposed: op(A)(i,k) = A[k*lda + i], op(B)(k,j) = B[j*ldb + k].
#include "gemm_f32_kernel.h"

TSG_F32_DEFINE_MODE(launch_f32_col_bt, A_COL_BT)

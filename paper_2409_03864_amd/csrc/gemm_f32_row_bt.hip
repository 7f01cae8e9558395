// fp32 kernels, op(A)(i,k) = A[i*lda + k] and op(B)(k,j) = B[j*ldb + k] (both k contiguous).
#include "gemm_f32_kernel.h"

TSG_F32_DEFINE_MODE(launch_f32_row_bt, A_ROW_BT)

// bf16 kernels, op(A)(i,k) = A[i*lda + k] and op(B)(k,j) = B[j*ldb + k] (both k contiguous).
#include "gemm_bf16_kernel.h"

TSG_BF16_DEFINE_MODE(launch_bf16_row_bt, A_ROW_BT)

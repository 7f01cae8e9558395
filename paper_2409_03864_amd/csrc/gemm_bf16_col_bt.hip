// bf16 kernels, both operands stored transposed: op(A)(i,k) = A[k*lda + i], op(B)(k,j) = B[j*ldb + k].
#include "gemm_bf16_kernel.h"

TSG_BF16_DEFINE_MODE(launch_bf16_col_bt, A_COL_BT)

// bf16 kernels, op(A) = implicit im2col matrix of an NHWC tensor (padding never read).
#include "gemm_bf16_kernel.h"

TSG_BF16_DEFINE_MODE(launch_bf16_conv, A_CONV)

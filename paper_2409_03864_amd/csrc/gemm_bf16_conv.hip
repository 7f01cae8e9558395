// bfloat16 kernels, op(A) = implicit im2col matrix of an NHWC tensor (padding never read).
#include "gemm_kernel.h"

TSG_DEFINE_MODE(launch_bf16_conv, TSG_BF16_TILES, A_CONV)

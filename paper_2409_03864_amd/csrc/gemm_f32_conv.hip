// fp32 kernels, op(A) = implicit im2col matrix of an NHWC tensor (padding never read).
#include "gemm_kernel.h"

TSG_DEFINE_MODE(launch_f32_conv, TSG_F32_TILES, A_CONV)

// fp32 kernels, op(A) = implicit im2col matrix of an NHWC tensor (padding never read).
#include "gemm_f32_kernel.h"

TSG_F32_DEFINE_MODE(launch_f32_conv, A_CONV)

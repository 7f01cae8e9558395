// bf16 kernels, op(A) = the implicit im2col matrix of an NHWC tensor (never materialised): the first
// part of the tile list, and the entry that picks the part.
#include "gemm_tiles.h"

TSG_DEFINE_MODE_PART(launch_bf16_conv_a, TSG_BF16_TILES_A, A_CONV, 0)

namespace tsg {
hipError_t launch_bf16_conv_b(int tile, int variant, const KArgs& a, int batch, hipStream_t s);
hipError_t launch_bf16_conv(int tile, int variant, const KArgs& a, int batch, hipStream_t s) {
    constexpr int kFirstB = 0 TSG_BF16_TILES_A(TSG_COUNT_TILE);
    return tile < kFirstB ? launch_bf16_conv_a(tile, variant, a, batch, s) : launch_bf16_conv_b(tile, variant, a, batch, s);
}
}  // namespace tsg

// bfloat16 kernels, op(A)(i,k) = A[i*lda + k], and the table of instantiated tiles.
#include "gemm_tiles.h"

TSG_DEFINE_MODE(launch_bf16_row, TSG_BF16_TILES, A_ROW)

namespace tsg {
hipError_t launch_bf16_col(int tile, int variant, const KArgs& a, int batch, hipStream_t s);
hipError_t launch_bf16_conv(int tile, int variant, const KArgs& a, int batch, hipStream_t s);
hipError_t launch_bf16_row_bt(int tile, int variant, const KArgs& a, int batch, hipStream_t s);
hipError_t launch_bf16_col_bt(int tile, int variant, const KArgs& a, int batch, hipStream_t s);

namespace {
hipError_t launch_any(int tile, int amode, int variant, const KArgs& a, int batch, hipStream_t s) {
    switch (amode) {
        case A_ROW: return launch_bf16_row(tile, variant, a, batch, s);
        case A_COL: return launch_bf16_col(tile, variant, a, batch, s);
        case A_ROW_BT: return launch_bf16_row_bt(tile, variant, a, batch, s);
        case A_COL_BT: return launch_bf16_col_bt(tile, variant, a, batch, s);
        default: return launch_bf16_conv(tile, variant, a, batch, s);
    }
}
const KernelEntry kTable[] = {TSG_BF16_TILES(TSG_TABLE_ENTRY)};
}  // namespace

const KernelEntry* bf16_kernels(int* count) {
    *count = (int)(sizeof(kTable) / sizeof(kTable[0]));
    return kTable;
}
}  // namespace tsg

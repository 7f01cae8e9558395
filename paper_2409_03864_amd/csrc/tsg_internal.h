// Internal glue between the C-ABI layer (api.cpp) and the kernel translation units.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace tsg {

// How op(A)(i,k) is addressed.
enum AMode : int {
    A_ROW = 0,   // A stored M x K, k contiguous
    A_COL = 1,   // A stored K x M, i contiguous (transposed left operand read in place)
    A_CONV = 2,  // A is the implicit im2col matrix of an NHWC tensor, never materialised
    // the same two GEMM forms with the right operand stored transposed too (B is N x K,
    // k contiguous, read in place); only the direct-to-LDS kernel forms take these
    A_ROW_BT = 3,
    A_COL_BT = 4
};

// Kernel arguments, passed by value.
struct KArgs {
    const void* A;
    const void* B;
    float* C;
    long long lda, ldb, ldc;
    long long stride_a, stride_b, stride_c;   // batch strides (elements)
    int M, N, K;
    int tiles_m, tiles_n;
    int m_main, n_main;      // extents of the divisible (unmasked) part of i and j
    int k_full;              // number of complete BK steps (the rest of k is masked)
    unsigned flags;
    int raster;
    // split of the k loop over `split_k` workgroups per tile (1 = none) for the tiles from
    // `split_first` on; partial tiles meet in `ws` ([batch][split tile][split][BM*BN] floats,
    // register order) and `counters` ([batch][split tile]) counts the arrivals: the last
    // workgroup to arrive sums the partials in split order.  Workgroup ids below split_first
    // are whole tiles; the rest are (split index, split tile) with the split index slow.
    int split_k;
    int split_first;   // tiles below this index are not split (0: the split applies to every tile)
    float* ws;
    int* counters;
    // convolution geometry (A_CONV only)
    int H, W, Cin, Ho, Wo, KW, sh, sw, ph, pw;
    // convolution output written into a window of a larger NHWC tensor: pixel (n, ho, wo) at
    // C + n*y_sn + ho*y_sh + wo*y_sw (elements) instead of row m of a matrix with pitch ldc
    int y_window;
    long long y_sn, y_sh, y_sw;
};

// One instantiated tile shape.  `launch` takes the entry's index in its table.
struct KernelEntry {
    int bm, bn, bk, wm, wn;
    int sched;       // kernel form, see gemm_kernel.h
    int mfma;        // MFMA block: 0 = 32 x 32, 1 = 16 x 16
    int threads;
    int vec;         // elements per 16-byte access for this dtype
    int lds_bytes;   // LDS per workgroup (all stages, k-contiguous A layout)
    int modes;       // bit m set: the tile exists for address mode m (AMode)
    // variant: 0 = vec, no remainder path; 1 = vec with remainder path; 3 = vec with the remainder
    // path that clamps and peels (every operand at least one access wide); 2 = scalar
    // accesses with remainder path
    hipError_t (*launch)(int tile, int amode, int variant, const KArgs& a, int batch, hipStream_t s);
};

// The caller's workspace (tsg_workspace_set, tsg_workspace_set_stream): arrival counters in the
// first kWorkspaceCounterBytes, partial results after them.  The GEMM kernels count arrivals in
// slots [0, kWorkspaceReduceSlot), the full reduce in slot kWorkspaceReduceSlot.  workspace_get
// returns the buffer a call on `stream` uses, false if there is none.
constexpr long long kWorkspaceCounterBytes = 16384 * 4;
constexpr long long kWorkspaceReduceSlot = 16383;
bool workspace_get(void* stream, void** ws, long long* bytes);

const KernelEntry* f32_kernels(int* count);
const KernelEntry* bf16_kernels(int* count);

}  // namespace tsg

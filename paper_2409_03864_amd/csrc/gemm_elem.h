// Element traits of the contraction kernels: what differs between operand types and MFMA
// block shapes, and nothing else.  A trait fixes
//   - the operand element and the 16-byte chunk that global loads, LDS staging and
//     k-contiguous fragment reads all move;
//   - the MFMA block (BLK x BLK outputs per instruction), how its 64 lanes split into a
//     position inside the block (lane % BLK) and a k slot (lane / BLK), and how many MFMAs
//     one 16-byte fragment feeds;
//   - how a fragment is gathered from a tile stored [k][j] (contiguous along i or j, the way a
//     row-major B and a transposed A lie in memory);
//   - the paddings of the register-staged LDS layout and the swizzle of the unpadded one.
// The fixed-size inner matmul that Case Study 4 hands to a microkernel library is, here, one
// of these MFMA sequences.
#pragma once
#include "tsg_internal.h"

namespace tsg {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
// 16-byte global access that only promises element alignment: rows of an operand with an
// odd leading dimension start on any element boundary, and the hardware fetches such a chunk
// with one instruction all the same
typedef f32x4 f32x4_u __attribute__((aligned(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef unsigned short u16;
typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));
typedef u16x8 u16x8_u __attribute__((aligned(2)));
typedef __attribute__((address_space(3))) bf16x4* lds_bf16x4_ptr;

// fp32 operands, v_mfma_f32_32x32x2_f32.  A k group is 8 values of k consumed in the order
// (t, t + 4), t = 0..3: lanes 0-31 feed k = t and lanes 32-63 feed k = t + 4 of MFMA t.  Any
// order is legal as long as both operands use it, and this one lets a k-contiguous row be
// fetched with a single 16-byte LDS read per four MFMAs.
struct F32 {
    using elem = float;
    using chunk = f32x4;
    using chunk_u = f32x4_u;
    using frag = f32x4;
    using acc_t = f32x16;
    static constexpr int V = 4;        // elements per 16-byte chunk
    static constexpr int BLK = 32;     // MFMA block edge
    static constexpr int LK = 2;       // k slots across the wave (64 / BLK)
    static constexpr int KG = 8;       // k values per group (LK chunks)
    static constexpr int TPG = 4;      // MFMAs per block and group
    static constexpr int NRJ = 4;      // LDS reads per fragment of a [k][j] tile
    static constexpr int NACC = 16;    // accumulator registers per block
    static constexpr int PAD_K = 4, PAD_J = 8;   // register-staged layout: [row][BK + 4], [k][BN + 8]
    static constexpr bool kHasGeneral = true;
    static __device__ __forceinline__ chunk zero() { return chunk{0.f, 0.f, 0.f, 0.f}; }
    static __device__ __forceinline__ int swz_j(int) { return 0; }
    // part t of a [k][j] fragment: the value at k = k0 + 4 (lane / 32) + t, column col0 + lane % 32
    static __device__ __forceinline__ void read_j(frag& f, int t, const elem* tile, int ld, int k0, int col0, int lane,
                                                  bool) {
        f[t] = tile[(k0 + 4 * (lane >> 5) + t) * ld + col0 + (lane & 31)];
    }
    static __device__ __forceinline__ acc_t mfma(const frag& a, const frag& b, const acc_t& c, int t) {
        return __builtin_amdgcn_mfma_f32_32x32x2f32(a[t], b[t], c, 0, 0, 0);
    }
    // accumulator register r of a block: row and column inside the block
    static __device__ __forceinline__ int acc_row(int r, int lane) { return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); }
};

// fp32 operands, v_mfma_f32_16x16x4_f32: wave tiles in 16-row steps, for extents that a
// 32-row block would pad (196 rows -> 208 instead of 224).  A k group is 16 values of k:
// lane slot q = lane / 16 feeds k = 4 q + t of MFMA t, so a k-contiguous row is again one
// 16-byte read per four MFMAs.  A [k][j] tile is read with four lane slots per access, rows
// k, k + 4, k + 8, k + 12 at the same columns: chunk c of row k sits at c ^ 4 ((k / 4) % 2),
// which keeps the two rows of one 32-lane pass in different banks.
struct F32B16 {
    using elem = float;
    using chunk = f32x4;
    using chunk_u = f32x4_u;
    using frag = f32x4;
    using acc_t = f32x4;
    static constexpr int V = 4;
    static constexpr int BLK = 16;
    static constexpr int LK = 4;
    static constexpr int KG = 16;
    static constexpr int TPG = 4;
    static constexpr int NRJ = 4;
    static constexpr int NACC = 4;
    static constexpr int PAD_K = 4, PAD_J = 8;
    static constexpr bool kHasGeneral = false;   // exists in the direct-to-LDS forms only
    static __device__ __forceinline__ chunk zero() { return chunk{0.f, 0.f, 0.f, 0.f}; }
    static __device__ __forceinline__ int swz_j(int krow) { return ((krow >> 2) & 1) << 2; }
    static __device__ __forceinline__ void read_j(frag& f, int t, const elem* tile, int ld, int k0, int col0, int lane,
                                                  bool swizzled) {
        const int k = k0 + 4 * (lane >> 4) + t, c = col0 + (lane & 15);
        f[t] = tile[k * ld + (swizzled ? ((((c >> 2) ^ swz_j(k)) << 2) | (c & 3)) : c)];
    }
    static __device__ __forceinline__ acc_t mfma(const frag& a, const frag& b, const acc_t& c, int t) {
        return __builtin_amdgcn_mfma_f32_16x16x4f32(a[t], b[t], c, 0, 0, 0);
    }
    static __device__ __forceinline__ int acc_row(int r, int lane) { return 4 * (lane >> 4) + r; }
};

// bfloat16 operands (bit patterns), v_mfma_f32_32x32x16_bf16, fp32 accumulate.  The MFMA wants,
// per lane, eight consecutive k values of one row of op(A) (one column of B): a k group is 16
// values of k and one MFMA per block.  A [k][j] tile is fetched with the transposing LDS read
// ds_read_b64_tr_b16: within a 16-lane group, lane l receives element (l % 4) of the four
// 8-byte rows addressed by lanes l/4, l/4 + 4, l/4 + 8, l/4 + 12.  Pointing lane s of a group
// at row k0 + s/4, columns j0 + 4 (s % 4) .. +3 therefore hands lane l the four values
// B[k0 .. k0+3][j0 + l]: no transposition in registers or on the store side.  Two such reads
// (rows +0 and +4) make a fragment.  Unpadded tiles: chunk c (8 values of j) of row k sits at
// c ^ 2 (k % 4), which puts the four rows of one read in four different 32-byte bank ranges.
struct BF16 {
    using elem = u16;
    using chunk = u16x8;
    using chunk_u = u16x8_u;
    using frag = bf16x8;
    using acc_t = f32x16;
    static constexpr int V = 8;
    static constexpr int BLK = 32;
    static constexpr int LK = 2;
    static constexpr int KG = 16;
    static constexpr int TPG = 1;
    static constexpr int NRJ = 2;
    static constexpr int NACC = 16;
    static constexpr int PAD_K = 8, PAD_J = 32;   // [row][BK + 8], [k][BN + 32]
    static constexpr bool kHasGeneral = true;
    static __device__ __forceinline__ chunk zero() { return chunk{0, 0, 0, 0, 0, 0, 0, 0}; }
    static __device__ __forceinline__ int swz_j(int krow) { return (krow & 3) << 1; }
    // half h of a [k][j] fragment: k = k0 + 8 (lane / 32) + 4 h .. + 3, column col0 + lane % 32
    static __device__ __forceinline__ void read_j(frag& f, int h, const elem* tile, int ld, int k0, int col0, int lane,
                                                  bool swizzled) {
        const int krow = k0 + 8 * (lane >> 5) + ((lane & 15) >> 2) + 4 * h;
        const int c = col0 + (lane & 16) + 4 * (lane & 3);
        const elem* p0 = tile + krow * ld + (swizzled ? ((((c >> 3) ^ swz_j(krow)) << 3) | (c & 7)) : c);
        const bf16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(p0));
        const bf16x4 lo = h == 0 ? v : __builtin_shufflevector(f, f, 0, 1, 2, 3);
        const bf16x4 hi = h == 1 ? v : __builtin_shufflevector(f, f, 4, 5, 6, 7);
        f = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    }
    static __device__ __forceinline__ acc_t mfma(const frag& a, const frag& b, const acc_t& c, int) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int acc_row(int r, int lane) { return 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3); }
};

// bfloat16 operands, v_mfma_f32_16x16x32_bf16: wave tiles in 16-row steps, as F32B16 for fp32.  Lane
// slot q = lane / 16 feeds k = 8 q .. 8 q + 7 of the one MFMA of a 32-wide k group, so a k-contiguous
// row is one 16-byte read per MFMA.  A [k][j] tile is fetched with the same transposing read as BF16:
// a 16-lane group covers the 16 columns of the block and four rows of k per read, two reads per fragment.
struct BF16B16 {
    using elem = u16;
    using chunk = u16x8;
    using chunk_u = u16x8_u;
    using frag = bf16x8;
    using acc_t = f32x4;
    static constexpr int V = 8;
    static constexpr int BLK = 16;
    static constexpr int LK = 4;
    static constexpr int KG = 32;
    static constexpr int TPG = 1;
    static constexpr int NRJ = 2;
    static constexpr int NACC = 4;
    static constexpr int PAD_K = 8, PAD_J = 32;
    static constexpr bool kHasGeneral = false;   // exists in the direct-to-LDS forms only
    static __device__ __forceinline__ chunk zero() { return chunk{0, 0, 0, 0, 0, 0, 0, 0}; }
    static __device__ __forceinline__ int swz_j(int krow) { return (krow & 3) << 1; }
    // half h of a [k][j] fragment: k = k0 + 8 (lane / 16) + 4 h .. + 3, column col0 + lane % 16
    static __device__ __forceinline__ void read_j(frag& f, int h, const elem* tile, int ld, int k0, int col0, int lane,
                                                  bool swizzled) {
        const int krow = k0 + 8 * (lane >> 4) + ((lane & 15) >> 2) + 4 * h;
        const int c = col0 + 4 * (lane & 3);
        const elem* p0 = tile + krow * ld + (swizzled ? ((((c >> 3) ^ swz_j(krow)) << 3) | (c & 7)) : c);
        const bf16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(p0));
        const bf16x4 lo = h == 0 ? v : __builtin_shufflevector(f, f, 0, 1, 2, 3);
        const bf16x4 hi = h == 1 ? v : __builtin_shufflevector(f, f, 4, 5, 6, 7);
        f = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    }
    static __device__ __forceinline__ acc_t mfma(const frag& a, const frag& b, const acc_t& c, int) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int acc_row(int r, int lane) { return 4 * (lane >> 4) + r; }
};

}  // namespace
}  // namespace tsg

// Which tiles of gemm_kernel.h are instantiated, and the glue that gives every (element type,
// address mode) pair a translation unit of its own.
#pragma once
#include "gemm_kernel.h"

// The instantiated tile shapes: X(element traits, BM, BN, BK, WM, WN, min waves per SIMD, sched).
// The register-staged forms that pipeline by hand (fragments one group or one MFMA ahead, three
// padded stages) were measured on ten workloads and never came within 2 % of the best direct
// form; they are no longer built.  The staged form that remains serves scalar accesses.
// (each list in two parts: the convolution units, the slowest to compile, take a part each)
#define TSG_F32_TILES_A(X)               \
    X(F32, 128, 128, 16, 64, 64, 2, 0)   \
    X(F32, 64, 64, 32, 32, 32, 2, 0)     \
    X(F32, 64, 64, 64, 32, 32, 2, 0)     \
    X(F32, 128, 64, 32, 64, 32, 2, 0)    \
    X(F32, 256, 128, 16, 64, 64, 2, 0)   \
    X(F32, 256, 256, 16, 128, 64, 2, 0)  \
    X(F32, 64, 64, 32, 32, 32, 2, 4)     \
    X(F32, 64, 64, 64, 32, 32, 2, 4)     \
    X(F32, 64, 64, 64, 32, 32, 1, 5)     \
    X(F32, 128, 64, 32, 64, 32, 2, 4)    \
    X(F32, 128, 128, 16, 64, 64, 2, 4)
#define TSG_F32_TILES_B(X)               \
    X(F32, 128, 128, 32, 64, 64, 2, 4)   \
    X(F32, 256, 128, 16, 64, 64, 2, 4)   \
    X(F32, 256, 128, 16, 64, 64, 2, 5)   \
    X(F32, 256, 256, 16, 128, 64, 2, 4)  \
    X(F32, 64, 64, 32, 32, 32, 2, 5)     \
    X(F32B16, 112, 64, 32, 112, 16, 2, 4) \
    X(F32B16, 112, 64, 32, 112, 16, 2, 5) \
    X(F32B16, 112, 64, 64, 112, 16, 1, 4) \
    X(F32B16, 64, 64, 32, 64, 16, 2, 4)  \
    X(F32B16, 16, 16, 64, 16, 16, 1, 1)  \
    X(F32, 32, 32, 32, 32, 32, 1, 1)
#define TSG_F32_TILES(X) TSG_F32_TILES_A(X) TSG_F32_TILES_B(X)

#define TSG_BF16_TILES_A(X)                \
    X(BF16, 256, 256, 64, 128, 64, 2, 0)   \
    X(BF16, 128, 128, 32, 64, 64, 2, 0)    \
    X(BF16, 64, 64, 64, 32, 32, 2, 0)      \
    X(BF16, 64, 64, 64, 32, 32, 2, 4)      \
    X(BF16, 128, 128, 64, 64, 64, 2, 4)    \
    X(BF16, 128, 128, 32, 64, 64, 2, 5)    \
    X(BF16, 256, 128, 64, 64, 64, 2, 4)
#define TSG_BF16_TILES_B(X)                \
    X(BF16, 256, 256, 32, 128, 64, 2, 4)   \
    X(BF16, 256, 256, 32, 128, 64, 2, 5)   \
    X(BF16, 256, 256, 32, 128, 128, 1, 4)  \
    X(BF16, 256, 256, 32, 128, 128, 1, 5)  \
    X(BF16B16, 112, 64, 64, 112, 16, 1, 4) \
    X(BF16B16, 112, 64, 32, 112, 16, 2, 5) \
    X(BF16B16, 64, 64, 64, 64, 16, 2, 4)
#define TSG_BF16_TILES(X) TSG_BF16_TILES_A(X) TSG_BF16_TILES_B(X)
#define TSG_COUNT_TILE(el, bm, bn, bk, wm, wn, mw, sc) +1

// Each (element type, address mode) is compiled in its own translation unit: FN(tile index in
// the type's list, variant, ...) launches that tile.
#define TSG_TILE_CASE(AMODE) TSG_TILE_CASE_##AMODE
#define TSG_DEFINE_MODE(FN, TILES, AMODE) TSG_DEFINE_MODE_PART(FN, TILES, AMODE, 0)
// (a part of a list: FIRST is the index of its first tile in the whole list)
#define TSG_DEFINE_MODE_PART(FN, TILES, AMODE, FIRST)                                               \
    namespace tsg {                                                                                 \
    hipError_t FN(int tile, int variant, const KArgs& a, int batch, hipStream_t s) {                \
        int idx = FIRST;                                                                            \
        TILES(TSG_TILE_CASE_##AMODE)                                                                \
        return hipErrorInvalidValue;                                                                \
    }                                                                                               \
    }
#define TSG_TILE_CASE_A_ROW(el, bm, bn, bk, wm, wn, mw, sc) \
    if (tile == idx++) return launch_mode<Tile<el, bm, bn, bk, wm, wn, mw, sc>, A_ROW>(variant, a, batch, s);
#define TSG_TILE_CASE_A_COL(el, bm, bn, bk, wm, wn, mw, sc) \
    if (tile == idx++) return launch_mode<Tile<el, bm, bn, bk, wm, wn, mw, sc>, A_COL>(variant, a, batch, s);
#define TSG_TILE_CASE_A_CONV(el, bm, bn, bk, wm, wn, mw, sc) \
    if (tile == idx++) return launch_mode<Tile<el, bm, bn, bk, wm, wn, mw, sc>, A_CONV>(variant, a, batch, s);
#define TSG_TILE_CASE_A_ROW_BT(el, bm, bn, bk, wm, wn, mw, sc) \
    if (tile == idx++) return launch_mode<Tile<el, bm, bn, bk, wm, wn, mw, sc>, A_ROW_BT>(variant, a, batch, s);
#define TSG_TILE_CASE_A_COL_BT(el, bm, bn, bk, wm, wn, mw, sc) \
    if (tile == idx++) return launch_mode<Tile<el, bm, bn, bk, wm, wn, mw, sc>, A_COL_BT>(variant, a, batch, s);

// The table of a type's tiles (one translation unit per type defines it).
#define TSG_TABLE_ENTRY(el, bm, bn, bk, wm, wn, mw, sc)                                                      \
    KernelEntry{bm, bn, bk, wm, wn, sc, el::BLK == 16 ? 1 : 0, Tile<el, bm, bn, bk, wm, wn, mw, sc>::NT, el::V, \
                lds_bytes_of<Tile<el, bm, bn, bk, wm, wn, mw, sc>>(),                                           \
                mode_mask_of<Tile<el, bm, bn, bk, wm, wn, mw, sc>>(), &launch_any},

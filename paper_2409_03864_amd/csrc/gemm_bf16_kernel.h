// bfloat16-operand contraction kernels for gfx950: C(fp32) = +-op(A).B (+C) with
// v_mfma_f32_32x32x16_bf16 (fp32 accumulate).  Same tiling, split and address generators
// as the fp32 kernels.  The MFMA wants, per lane, eight consecutive k values of one row
// of op(A) (one column of B).  A k-contiguous operand (A_ROW, A_CONV) is staged as
// [row][k] and fetched with one 16-byte LDS read.  An operand that is contiguous along
// i or j instead (B, and op(A) when the left operand is stored transposed) is staged
// exactly as it lies in memory, [k][j], and fetched with the transposing LDS read
// ds_read_b64_tr_b16: within a 16-lane group, lane l receives element (l % 4) of the four
// 8-byte rows addressed by lanes l/4, l/4 + 4, l/4 + 8, l/4 + 12.  Pointing lane s of a
// group at row k0 + s/4, columns j0 + 4*(s%4) .. +3 therefore hands lane l the four
// values B[k0 .. k0+3][j0 + l]: no transposition in registers or on the store side.
#pragma once
#include <atomic>
#include <type_traits>

#include "tsg_internal.h"

namespace tsg {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned short u16;
typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));
// 16-byte global access that only promises element alignment (odd leading dimensions)
typedef u16x8 u16x8_u __attribute__((aligned(2)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) bf16x4* lds_bf16x4_ptr;

constexpr unsigned FLAG_NEGATE = 1u, FLAG_ACCUMULATE = 2u;
constexpr int kXcds = 8, kGroupM = 8;

// SCHED: 0 = instruction order inside a k step left to the compiler, 1 = fragments of
// k step g+1 read while the MFMAs of step g run, next tile written to LDS mid-step.
template <int BM_, int BN_, int BK_, int WM_, int WN_, int MINW_, int SCHED_>
struct Tile {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_, MINW = MINW_, SCHED = SCHED_;
    static constexpr int WAVES_M = BM / WM, WAVES_N = BN / WN;
    static constexpr int NT = 64 * WAVES_M * WAVES_N;
    static constexpr int MI = WM / 32, NI = WN / 32;
    // LDS pitches in elements.  [row][k] tiles: +8 (16 B) makes the 16-byte reads of 16
    // consecutive rows hit distinct banks.  [k][j] tiles: +32 (64 B) puts the four rows of
    // one transposing read in four different 64-byte bank ranges.
    static constexpr int LDK = BK + 8;
    static constexpr int LDA_T = BM + 32, LDB = BN + 32;
    static_assert(BM % WM == 0 && BN % WN == 0 && WM % 32 == 0 && WN % 32 == 0 && BK % 16 == 0, "tile");
};

__device__ __forceinline__ void tile_coords(const KArgs& p, int bid, int& tm, int& tn) {
    if (p.raster) {
        // (every quantity is non-negative: unsigned divisions, which are cheaper)
        const unsigned T = (unsigned)(p.tiles_m * p.tiles_n), ub = (unsigned)bid;
        const unsigned xcd = ub % kXcds, loc = ub / kXcds;
        const unsigned q = T / kXcds, r = T % kXcds;
        const unsigned uid = (xcd < r) ? xcd * (q + 1) + loc : r * (q + 1) + (xcd - r) * q + loc;
        const unsigned gsize = kGroupM * (unsigned)p.tiles_n;
        const unsigned g = uid / gsize, in_g = uid - g * gsize;
        const unsigned first_m = g * kGroupM;
        const unsigned gm = min((unsigned)p.tiles_m - first_m, (unsigned)kGroupM);
        const unsigned tnu = in_g / gm;
        tm = (int)(first_m + (in_g - tnu * gm));
        tn = (int)tnu;
        return;
    }
    tm = (int)((unsigned)bid / (unsigned)p.tiles_n);
    tn = bid - tm * p.tiles_n;
}

// Which tile, and which part of its k loop, a workgroup takes: ids below split_first are
// whole tiles; after them come the split tiles, split index slow, so the parts of one tile
// are dispatched a whole round apart and no part ever waits for another.
__device__ __forceinline__ void decode_block(const KArgs& p, int tiles, int& tile, int& split, int& nsplit, int& slot) {
    const int bid = blockIdx.x;
    if (bid < p.split_first) {
        tile = bid; split = 0; nsplit = 1; slot = 0;
        return;
    }
    const int r = bid - p.split_first, rem = tiles - p.split_first;
    split = (int)((unsigned)r / (unsigned)rem);
    const int t = r - split * rem;
    tile = p.split_first + t;
    nsplit = p.split_k;
    slot = blockIdx.y * rem + t;
}

// What follows the k loop: the split-k reduction (see the fp32 kernels) and the epilogue.
template <class T>
__device__ __forceinline__ void finish_tile(const KArgs& p, f32x16 (&acc)[T::MI][T::NI], float* __restrict__ C,
                                            int slot, int split, int nsplit, int m0, int n0, int wm0, int wn0,
                                            bool interior) {
    constexpr int BM = T::BM, BN = T::BN, NT = T::NT, MI = T::MI, NI = T::NI;
    const int tid = threadIdx.x, lane = tid & 63, li = lane & 31, lh = lane >> 5;
    // split k: park the partial tile, count the arrival, and let the last arrival reduce
    if (nsplit > 1) {
        __shared__ int arrived;
        float* ws = p.ws + (long long)slot * nsplit * (BM * BN);
        // A partial tile is kept in register order.  Partials cross between L2 domains, so
        // they are written and read with device-scope accesses that go through to memory; once
        // a wave's stores are acknowledged (the wait) and all waves are at the barrier, the
        // arrival is counted, and whoever sees the last count finds every partial in memory.
        // This takes no cache-wide write-back or invalidate.
        float* mine = ws + (long long)split * (BM * BN);
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    __hip_atomic_store(mine + ((i * NI + j) * 16 + r) * NT + tid, acc[i][j][r], __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (tid == 0) arrived = __hip_atomic_fetch_add(p.counters + slot, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        if (arrived != nsplit - 1) return;
        // acc = ((P0 + P1) + P2) + ...: a row of MFMA blocks of one partial tile at a time, all of
        // its loads in flight together
#pragma unroll
        for (int i = 0; i < MI; ++i)
            for (int sp = 0; sp < nsplit; ++sp) {
                const float* part = ws + (long long)sp * (BM * BN);
                float t[NI][16];
#pragma unroll
                for (int j = 0; j < NI; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        t[j][r] = __hip_atomic_load(part + ((i * NI + j) * 16 + r) * NT + tid, __ATOMIC_RELAXED,
                                                    __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
                for (int j = 0; j < NI; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[i][j][r] = sp == 0 ? t[j][r] : acc[i][j][r] + t[j][r];
            }
        if (tid == 0)   // ready for the next launch on this workspace
            __hip_atomic_store(p.counters + slot, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }

    // With ACCUMULATE the old values of a block are all loaded before its first store: a load
    // behind a store to an address the compiler cannot tell apart would wait for it, one round
    // trip to memory per element.
    const bool neg = p.flags & FLAG_NEGATE, accum = p.flags & FLAG_ACCUMULATE;
    // The bounds tests and the read of the old values are compiled into copies of their own,
    // chosen once per tile: with the tests beside every element an interior tile of the
    // remainder variant spent three times as long here.
    auto emit = [&](auto check_tag, auto accum_tag) {
    constexpr bool CHECK = decltype(check_tag)::value, ACCUM = decltype(accum_tag)::value;
    if (p.y_window) {
        // output pixel row -> (n, ho, wo) -> its place in the larger tensor.  A lane holds runs of
        // four consecutive rows: the first of a run is decoded, the others step from it
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                const int row0 = m0 + wm0 + i * 32 + 8 * rg + 4 * lh;
                // (non-negative: unsigned divisions)
                const unsigned tq = (unsigned)row0 / (unsigned)p.Wo, nq = tq / (unsigned)p.Ho;
                int wo = row0 - (int)tq * p.Wo, ho = (int)(tq - nq * (unsigned)p.Ho), n = (int)nq;
                float* dst[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    dst[e] = C + ((long long)n * p.y_sn + (long long)ho * p.y_sh + (long long)wo * p.y_sw) + n0 + wn0 + li;
                    if (++wo == p.Wo) {
                        wo = 0;
                        if (++ho == p.Ho) { ho = 0; ++n; }
                    }
                }
                float old[4][NI];
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int j = 0; j < NI; ++j) {
                        const bool ok = !CHECK || (row0 + e < p.M && n0 + wn0 + j * 32 + li < p.N);
                        old[e][j] = (ACCUM && ok) ? dst[e][j * 32] : 0.f;
                    }
#pragma unroll
                for (int e = 0; e < 4; ++e)
#pragma unroll
                    for (int j = 0; j < NI; ++j) {
                        const bool ok = !CHECK || (row0 + e < p.M && n0 + wn0 + j * 32 + li < p.N);
                        const float v = acc[i][j][rg * 4 + e];
                        const float sv = neg ? -v : v;
                        if (ok) dst[e][j * 32] = ACCUM ? sv + old[e][j] : sv;   // no add without the flag: -0 stays -0
                    }
            }
        return;
    }
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j) {
            const int col = n0 + wn0 + j * 32 + li;
            float* c0 = C + (long long)(m0 + wm0 + i * 32 + 4 * lh) * p.ldc + col;   // row of r = 0
            // element r sits 8 (r / 4) + r % 4 rows below: the row pointer steps, no multiply per element
            float old[16];
            if constexpr (ACCUM) {
                float* rp = c0;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int dr = 8 * (r >> 2) + (r & 3);
                    const bool ok = !CHECK || (m0 + wm0 + i * 32 + 4 * lh + dr < p.M && col < p.N);
                    old[r] = ok ? *rp : 0.f;
                    rp += (r & 3) == 3 ? 5 * p.ldc : p.ldc;
                }
            }
            float* rp = c0;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int dr = 8 * (r >> 2) + (r & 3);
                const bool ok = !CHECK || (m0 + wm0 + i * 32 + 4 * lh + dr < p.M && col < p.N);
                const float v = acc[i][j][r];
                const float sv = neg ? -v : v;
                if (ok) *rp = ACCUM ? sv + old[r] : sv;   // no add without the flag: -0 stays -0
                rp += (r & 3) == 3 ? 5 * p.ldc : p.ldc;
            }
        }
    };
    if (interior) {
        if (accum) emit(std::false_type{}, std::true_type{});
        else emit(std::false_type{}, std::false_type{});
    } else {
        if (accum) emit(std::true_type{}, std::true_type{});
        else emit(std::true_type{}, std::false_type{});
    }
}

template <class T, int AMODE, int VEC, bool EDGE>
__global__ void __launch_bounds__(T::NT, T::MINW) gemm_bf16_kernel(const KArgs p) {
    constexpr int BM = T::BM, BN = T::BN, BK = T::BK, NT = T::NT, MI = T::MI, NI = T::NI;
    constexpr bool A_KMAJ = (AMODE != A_COL);
    constexpr int LDA = A_KMAJ ? T::LDK : T::LDA_T, LDB = T::LDB;
    constexpr int A_SIZE = A_KMAJ ? BM * LDA : BK * LDA, B_SIZE = BK * LDB, STAGE = A_SIZE + B_SIZE;
    extern __shared__ __attribute__((aligned(16))) u16 smem16[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave / T::WAVES_N) * T::WM, wn0 = (wave % T::WAVES_N) * T::WN;
    const int li = lane & 31, lh = lane >> 5;

    const int tiles = p.tiles_m * p.tiles_n;
    int tile, split, nsplit, slot;
    decode_block(p, tiles, tile, split, nsplit, slot);
    int tm, tn;
    tile_coords(p, tile, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;
    const u16* __restrict__ A = (const u16*)p.A + (long long)blockIdx.y * p.stride_a;
    const u16* __restrict__ B = (const u16*)p.B + (long long)blockIdx.y * p.stride_b;
    float* __restrict__ C = p.C + (long long)blockIdx.y * p.stride_c;

    const bool interior = !EDGE || (m0 + BM <= p.m_main && n0 + BN <= p.n_main);
    // this workgroup's k steps: [kb, kb + nk) of the whole loop (split k, see the fp32 kernels)
    const int nk_all = (p.K + BK - 1) / BK;
    // (unsigned 32-bit: nk_all < 2^27 and nsplit <= 16; an unsplit tile divides nothing)
    int kb = 0, nk = nk_all;
    if (nsplit > 1) {
        kb = (int)((unsigned)(nk_all * split) / (unsigned)nsplit);
        nk = (int)((unsigned)(nk_all * (split + 1)) / (unsigned)nsplit) - kb;
    }

    // 8-element (16-byte) chunks along the contiguous dimension of each stored operand.
    // kmaj == true: the stored rows run along k (A_ROW, A_CONV); false: along i or j.
    constexpr int A_CPR = A_KMAJ ? BK / 8 : BM / 8;
    constexpr int A_ROWS = A_KMAJ ? BM : BK;
    constexpr int A_RPP = NT / A_CPR, PA = A_ROWS / A_RPP;
    constexpr int B_CPR = BN / 8, B_RPP = NT / B_CPR, PB = BK / B_RPP;
    static_assert(NT % A_CPR == 0 && A_ROWS % A_RPP == 0 && PA >= 1, "A staging shape");
    static_assert(NT % B_CPR == 0 && BK % B_RPP == 0 && PB >= 1, "B staging shape");
    const int a_r = tid / A_CPR, a_c = (tid % A_CPR) * 8;
    const int b_r = tid / B_CPR, b_c = (tid % B_CPR) * 8;

    int cv_base[PA], cv_hi0[PA], cv_wi0[PA];
    if constexpr (AMODE == A_CONV) {
#pragma unroll
        for (int q = 0; q < PA; ++q) {
            const int m = m0 + a_r + q * A_RPP;
            if (m < p.M) {
                const int wo = m % p.Wo, t = m / p.Wo;
                const int ho = t % p.Ho, n = t / p.Ho;
                cv_base[q] = n * p.H;
                cv_hi0[q] = ho * p.sh - p.ph;
                cv_wi0[q] = wo * p.sw - p.pw;
            } else {
                cv_base[q] = 0;
                cv_hi0[q] = -(1 << 28);
                cv_wi0[q] = 0;
            }
        }
    }

    // convolution: (kh, kw, ci) of the first k of the next step to load, advanced step by step
    // (steps are loaded in order); with Cin a multiple of BK a step lies inside one tap
    int cs_kh = 0, cs_kw = 0, cs_ci = 0;
    const bool one_tap = AMODE == A_CONV && p.Cin % BK == 0;
    if constexpr (AMODE == A_CONV) {
        const int k = kb * BK, tap = k / p.Cin;
        cs_ci = k - tap * p.Cin;
        cs_kh = tap / p.KW;
        cs_kw = tap - cs_kh * p.KW;
    }

    u16x8 ra[PA], rb[PB];

    auto a_elem = [&](int q, int row_or_k, int e) -> u16 {
        if constexpr (AMODE == A_ROW) {
            const int m = m0 + row_or_k, k = e;
            return (m < p.M && k < p.K) ? A[(long long)m * p.lda + k] : (u16)0;
        } else if constexpr (AMODE == A_COL) {
            const int k = row_or_k, m = e;
            return (k < p.K && m < p.M) ? A[(long long)k * p.lda + m] : (u16)0;
        } else {
            const int k = e;
            if (k >= p.K) return 0;
            const int tap = k / p.Cin, ci = k - tap * p.Cin;
            const int kh = tap / p.KW, kw = tap - kh * p.KW;
            const int hi = cv_hi0[q] + kh, wi = cv_wi0[q] + kw;
            if (hi < 0 || hi >= p.H || wi < 0 || wi >= p.W) return 0;
            return A[((long long)(cv_base[q] + hi) * p.W + wi) * p.Cin + ci];
        }
    };

    auto load_tiles = [&](int kt_local) {
        const int kt = kb + kt_local;
        const bool fast = EDGE ? (interior && kt < p.k_full) : true;
        const int k0 = kt * BK;
#pragma unroll
        for (int q = 0; q < PA; ++q) {
            const int r = a_r + q * A_RPP;
            if constexpr (AMODE == A_ROW) {
                const int k = k0 + a_c;
                if (VEC == 8 && (fast || (m0 + r < p.M && k + 8 <= p.K))) {
                    ra[q] = *(const u16x8_u*)(A + (long long)(m0 + r) * p.lda + k);
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) ra[q][e] = a_elem(q, r, k + e);
                }
            } else if constexpr (AMODE == A_COL) {
                const int k = k0 + r, m = m0 + a_c;
                if (VEC == 8 && (fast || (k < p.K && m + 8 <= p.M))) {
                    ra[q] = *(const u16x8_u*)(A + (long long)k * p.lda + m);
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) ra[q][e] = a_elem(q, k, m + e);
                }
            } else {
                const int k = k0 + a_c;
                if constexpr (VEC == 8) {
                    u16x8 v = {0, 0, 0, 0, 0, 0, 0, 0};
                    if (fast || k < p.K) {
                        int kh = cs_kh, kw = cs_kw, ci = cs_ci + a_c;
                        if (!one_tap) {
                            const int tap = k / p.Cin;
                            ci = k - tap * p.Cin;
                            kh = tap / p.KW;
                            kw = tap - kh * p.KW;
                        }
                        const int hi = cv_hi0[q] + kh, wi = cv_wi0[q] + kw;
                        if (hi >= 0 && hi < p.H && wi >= 0 && wi < p.W)
                            v = *(const u16x8_u*)(A + ((long long)(cv_base[q] + hi) * p.W + wi) * p.Cin + ci);
                    }
                    ra[q] = v;
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) ra[q][e] = a_elem(q, r, k + e);
                }
            }
        }
        if constexpr (AMODE == A_CONV) {
            cs_ci += BK;
            while (cs_ci >= p.Cin) {
                cs_ci -= p.Cin;
                if (++cs_kw == p.KW) { cs_kw = 0; ++cs_kh; }
            }
        }
#pragma unroll
        for (int q = 0; q < PB; ++q) {
            const int k = k0 + b_r + q * B_RPP, n = n0 + b_c;
            if (VEC == 8 && (fast || (k < p.K && n + 8 <= p.N))) {
                rb[q] = *(const u16x8_u*)(B + (long long)k * p.ldb + n);
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    rb[q][e] = (k < p.K && n + e < p.N) ? B[(long long)k * p.ldb + n + e] : (u16)0;
            }
        }
    };

    auto store_tiles = [&](int stage) {
        u16* As = smem16 + stage * STAGE;
        u16* Bs = As + A_SIZE;
#pragma unroll
        for (int q = 0; q < PA; ++q)
            *(u16x8*)(As + (a_r + q * A_RPP) * LDA + a_c) = ra[q];
#pragma unroll
        for (int q = 0; q < PB; ++q)
            *(u16x8*)(Bs + (b_r + q * B_RPP) * LDB + b_c) = rb[q];
    };

    // lane -> source row / column of the transposing read (see the header comment)
    const int tr_row = 8 * lh + ((lane & 15) >> 2);          // k offset inside a 16-wide k step
    const int tr_col = (lane & 16) + 4 * (lane & 3);         // i or j offset inside a 32-wide block

    auto read_tr = [&](const u16* tile, int ld, int k, int col) -> bf16x8 {
        const u16* p0 = tile + (k + tr_row) * ld + col + tr_col;
        const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(p0));
        const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(p0 + 4 * ld));
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    };

    f32x16 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    auto load_frags = [&](const u16* As, const u16* Bs, int kk, bf16x8 (&af)[MI], bf16x8 (&bf)[NI]) {
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            if constexpr (A_KMAJ)
                af[i] = *(const bf16x8*)(As + (wm0 + i * 32 + li) * LDA + kk + 8 * lh);
            else
                af[i] = read_tr(As, LDA, kk, wm0 + i * 32);
        }
#pragma unroll
        for (int j = 0; j < NI; ++j) bf[j] = read_tr(Bs, LDB, kk, wn0 + j * 32);
    };

    // Fragments of k step g+1 are fetched from LDS while the MFMAs of step g run; the next
    // tile (already in registers) is written to the other LDS stage half way through.  The
    // scheduling barriers keep the compiler from sinking the reads back to their first use.
    auto compute = [&](int stage, int kt) {
        const u16* As = smem16 + stage * STAGE;
        const u16* Bs = As + A_SIZE;
        constexpr int G = BK / 16;
        bf16x8 af[2][MI], bf[2][NI];
        load_frags(As, Bs, 0, af[0], bf[0]);
#pragma unroll
        for (int g = 0; g < G; ++g) {
            if (g + 1 < G) load_frags(As, Bs, (g + 1) * 16, af[(g + 1) & 1], bf[(g + 1) & 1]);
            if (g == G / 2) {
                // tile kt+1 has had a whole step to arrive: park it in the other stage, then
                // reuse the same registers for the loads of tile kt+2
                if (kt + 1 < nk) store_tiles(stage ^ 1);
                if (kt + 2 < nk) load_tiles(kt + 2);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[g & 1][i], bf[g & 1][j], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // SCHED 0: the plain form of the same step
    auto compute_plain = [&](int stage) {
        const u16* As = smem16 + stage * STAGE;
        const u16* Bs = As + A_SIZE;
#pragma unroll
        for (int kk = 0; kk < BK; kk += 16) {
            bf16x8 af[MI], bf[NI];
            load_frags(As, Bs, kk, af, bf);
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf[j], acc[i][j], 0, 0, 0);
        }
    };

    // tile t+1 sits in registers and tile t+2 is in flight while step t is multiplied
    load_tiles(0);
    store_tiles(0);
    if (nk > 1) load_tiles(1);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        if constexpr (T::SCHED == 1) {
            compute(kt & 1, kt);
        } else {
            compute_plain(kt & 1);
            if (kt + 1 < nk) store_tiles((kt & 1) ^ 1);
            if (kt + 2 < nk) load_tiles(kt + 2);
        }
        __syncthreads();
    }

    finish_tile<T>(p, acc, C, slot, split, nsplit, m0, n0, wm0, wn0, interior);
}

// ---------------------------------------------------------------------------------------
// SCHED 4 / 5: operand tiles travel from global memory straight into a ring of 3 / 4 LDS
// stages, as in the fp32 kernels (one direct load = 64 lanes x 16 bytes = 1 KiB of
// consecutive LDS; chunks wholly outside the operand come from a block of zeros; steps or
// tiles with chunks cut by the end of a row go through registers with masks).
//
// Unpadded tiles need a swizzle on both kinds of fragment read.  [row][k] tiles: chunk c
// (8 values of k) of row r sits at position c ^ swz(r), so the 16-byte reads of 16
// consecutive rows cover all banks.  [k][j] tiles: the transposing read of a 16-lane group
// touches four consecutive k rows, 32 bytes each, at the same j; chunk c of row k sits at
// position c ^ 2 (k % 4), which puts those four pieces in four different 32-byte bank ranges.
__device__ __attribute__((aligned(16))) u16 g_zero_chunk[8] = {0, 0, 0, 0, 0, 0, 0, 0};

__device__ __forceinline__ void load_to_lds16(const void* g, unsigned lds_byte_base) {
    // M0 carries the wave's LDS destination; lane l lands at base + 16 * l
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(lds_byte_base)
                 : "memory", "m0");
}
template <int N>
__device__ __forceinline__ void wait_loads_outstanding() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

template <class T>
struct LdsDirect {
    static constexpr int STAGES = T::SCHED == 5 ? 4 : 3;
    static constexpr int A_ELEMS = T::BM * T::BK, B_ELEMS = T::BK * T::BN, STAGE = A_ELEMS + B_ELEMS;
    static constexpr int BYTES = STAGES * STAGE * 2;
};

// EDGEV: 0 = every loop divides (no remainder code); 1 = remainder code with the masked register
// path compiled into the ring (kept for operands narrower than one access); 2 = the remainder
// variant in use: rows and columns past the end are clamped, the ring runs the full k steps without
// a test as one scheduling region, and the last k step is peeled off when it is partial or when the
// tile's chunks are cut along M or N (the masked path and its branch inside the ring cost a 64 x 64
// tile a third of its speed even when never taken).
// ONE_TAP (convolution only): Cin is a multiple of BK, so a k step lies inside one filter tap.
// A template parameter rather than a test at run time: the general form divides per chunk, and
// a two-sided branch between the MFMAs of a step splits the step's scheduling region.
template <class T, int MODE, int EDGEV, bool ONE_TAP = false>
__global__ void __launch_bounds__(T::NT, T::MINW) gemm_bf16_direct_kernel(const KArgs p) {
    constexpr bool EDGE = EDGEV != 0, CUT = EDGEV == 1;
    // EDGEV 2: rows and columns past M or N are read from the last valid row or chunk instead of
    // being tested at every step: their products only reach elements of C that are never stored
    // (k past K still reads the block of zeros: both factors must vanish there)
    constexpr bool CLAMP = EDGEV == 2;
    // address mode of the left operand, and whether the right one is stored transposed (N x K)
    constexpr int AMODE = MODE == A_ROW_BT ? A_ROW : MODE == A_COL_BT ? A_COL : MODE;
    constexpr bool B_KMAJ = MODE == A_ROW_BT || MODE == A_COL_BT;
    constexpr int BM = T::BM, BN = T::BN, BK = T::BK, NT = T::NT, MI = T::MI, NI = T::NI;
    using L = LdsDirect<T>;
    constexpr int STAGES = L::STAGES, D = STAGES - 1;
    constexpr bool A_KMAJ = AMODE != A_COL;
    constexpr int A_CPR = A_KMAJ ? BK / 8 : BM / 8;   // 16-byte chunks per stored row of A
    constexpr int A_ROWS = A_KMAJ ? BM : BK;
    constexpr int A_RPP = NT / A_CPR, PA = A_ROWS / A_RPP;
    constexpr int B_CPR = B_KMAJ ? BK / 8 : BN / 8;
    constexpr int B_ROWS = B_KMAJ ? BN : BK;
    constexpr int B_RPP = NT / B_CPR, PB = B_ROWS / B_RPP;
    constexpr int LPT = PA + PB;
    static_assert(NT % A_CPR == 0 && A_ROWS % A_RPP == 0 && PA >= 1, "A staging shape");
    static_assert(NT % B_CPR == 0 && B_ROWS % B_RPP == 0 && PB >= 1, "B staging shape");
    static_assert((D - 1) * LPT <= 63, "outstanding-load counter range");
    static_assert((B_KMAJ || B_CPR >= 8) && (A_KMAJ || A_CPR >= 8), "the [k][j] swizzle permutes chunks in groups of eight");
    constexpr int K_CPR = BK / 8;   // chunks per row of a [row][k] tile
    constexpr int SW_MOD = K_CPR < 16 ? K_CPR : 16, SW_DIV = 16 / SW_MOD;
    extern __shared__ __attribute__((aligned(16))) u16 smem16[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave / T::WAVES_N) * T::WM, wn0 = (wave % T::WAVES_N) * T::WN;
    const int li = lane & 31, lh = lane >> 5;

    const int tiles = p.tiles_m * p.tiles_n;
    int tile, split, nsplit, slot;
    decode_block(p, tiles, tile, split, nsplit, slot);
    int tm, tn;
    tile_coords(p, tile, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;
    const u16* __restrict__ A = (const u16*)p.A + (long long)blockIdx.y * p.stride_a;
    const u16* __restrict__ B = (const u16*)p.B + (long long)blockIdx.y * p.stride_b;
    float* __restrict__ C = p.C + (long long)blockIdx.y * p.stride_c;

    const bool interior = !EDGE || (m0 + BM <= p.m_main && n0 + BN <= p.n_main);
    const int nk_all = (p.K + BK - 1) / BK;
    // (unsigned 32-bit: nk_all < 2^27 and nsplit <= 16; an unsplit tile divides nothing)
    int kb = 0, nk = nk_all;
    if (nsplit > 1) {
        kb = (int)((unsigned)(nk_all * split) / (unsigned)nsplit);
        nk = (int)((unsigned)(nk_all * (split + 1)) / (unsigned)nsplit) - kb;
    }

    // leading steps of this workgroup whose chunks are all whole (inside or outside)
    // EDGEV 2 peels the k loop like Fig. 8: the ring runs the steps that lie wholly below K
    // without any test, and a last partial step is staged through registers after it
    // A tile whose chunks are cut by the end of a row along N (row-major B) or M (transposed A)
    // still takes whole 16-byte loads in the ring: the bytes past the end of a row are the start
    // of the next row, and only feed columns / rows of C that are never stored.  The last row of
    // the operand has no next row, so for such a tile the last k step is always peeled.
    const bool cut_tile = CLAMP && ((!B_KMAJ && (p.N % 8) && n0 + BN > p.N) || (AMODE == A_COL && (p.M % 8) && m0 + BM > p.M));
    int nkp_ = CLAMP ? min(nk, max(0, p.k_full - kb)) : nk;
    if (cut_tile && kb + nk == nk_all) nkp_ = min(nkp_, nk - 1);
    const int nkp = nkp_;   // steps that go through the ring
    int n_direct = nkp;
    if constexpr (CUT) {
        bool whole_tile = !(!B_KMAJ && (p.N & 7) && n0 + BN > p.N);
        if (AMODE == A_COL && (p.M & 7) && m0 + BM > p.M) whole_tile = false;
        if (!whole_tile) n_direct = 0;
        else if ((AMODE == A_ROW || B_KMAJ) && (p.K & 7)) n_direct = max(0, min(nk, p.k_full - kb));
    }

    // The address of the block of zeros, taken once and kept in registers: derived where it is
    // used, it costs a scalar load and a wait for every outstanding LDS read in the middle of
    // the MFMA sequence of every step.
    const u16* zero_chunk = g_zero_chunk;
    asm volatile("" : "+s"(zero_chunk));

    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) u16*)smem16 +
                          (unsigned)__builtin_amdgcn_readfirstlane(tid & ~63) * 16u;
    const int a_r = tid / A_CPR, a_cp = tid % A_CPR;
    const int b_r = tid / B_CPR, b_cp = tid % B_CPR;
    auto swz_k = [](int row) -> int { return (row / SW_DIV) % SW_MOD; };   // [row][k] tiles
    auto swz_j = [](int krow) -> int { return (krow & 3) << 1; };          // [k][j] tiles

    const u16* a_src[PA];
    int a_k[PA];
    bool a_in[PA];
    int cv_base[PA], cv_hi0[PA], cv_wi0[PA];
    long long cv_off[PA];   // element offset of tap (0, 0), channel a_k of the chunk's pixel (may lie outside the tensor)
#pragma unroll
    for (int q = 0; q < PA; ++q) {
        const int row = a_r + q * A_RPP;
        if constexpr (AMODE == A_ROW) {
            a_k[q] = (a_cp ^ swz_k(row)) * 8;
            a_in[q] = !CUT || m0 + row < p.M;
            a_src[q] = A + (long long)(CLAMP ? min(m0 + row, p.M - 1) : m0 + row) * p.lda + a_k[q];
        } else if constexpr (AMODE == A_COL) {
            a_k[q] = row;   // the stored row is the k index
            const int mc = (a_cp ^ swz_j(row)) * 8;
            a_in[q] = !CUT || m0 + mc < p.M;
            a_src[q] = A + (long long)row * p.lda + (CLAMP && m0 + mc >= p.M ? max(p.M - 8, 0) : m0 + mc);
        } else {
            a_k[q] = (a_cp ^ swz_k(row)) * 8;
            const int m = m0 + row;
            a_in[q] = !CUT || m < p.M;
            a_src[q] = A;
            const int mm = CLAMP ? min(m, p.M - 1) : a_in[q] ? m : 0;
            // (non-negative: unsigned divisions)
            const unsigned tq = (unsigned)mm / (unsigned)p.Wo, nq = tq / (unsigned)p.Ho;
            const int wo = mm - (int)tq * p.Wo, ho = (int)(tq - nq * (unsigned)p.Ho), n = (int)nq;
            cv_base[q] = n * p.H;
            cv_hi0[q] = ho * p.sh - p.ph;
            cv_wi0[q] = wo * p.sw - p.pw;
            cv_off[q] = ((long long)(cv_base[q] + cv_hi0[q]) * p.W + cv_wi0[q]) * p.Cin + a_k[q];
        }
    }
    int cs_kh = 0, cs_kw = 0, cs_ci = 0;
    long long cs_off = 0;   // element offset of (cs_kh, cs_kw, cs_ci) from tap (0, 0), channel 0 of a pixel
    constexpr bool one_tap = AMODE == A_CONV && ONE_TAP;
    if constexpr (AMODE == A_CONV) {
        const int k = kb * BK, tap = k / p.Cin;
        cs_ci = k - tap * p.Cin;
        cs_kh = tap / p.KW;
        cs_kw = tap - cs_kh * p.KW;
        cs_off = ((long long)cs_kh * p.W + cs_kw) * p.Cin + cs_ci;
    }
    const u16* b_src[PB];
    int b_k[PB];          // k offset of the chunk inside a step
    bool b_in[PB];
#pragma unroll
    for (int q = 0; q < PB; ++q) {
        const int row = b_r + q * B_RPP;
        if constexpr (B_KMAJ) {
            b_k[q] = (b_cp ^ swz_k(row)) * 8;
            b_in[q] = !CUT || n0 + row < p.N;
            b_src[q] = B + (long long)(CLAMP ? min(n0 + row, p.N - 1) : n0 + row) * p.ldb + b_k[q];
        } else {
            const int nc = (b_cp ^ swz_j(row)) * 8;
            b_k[q] = row;
            b_in[q] = !CUT || n0 + nc < p.N;
            b_src[q] = B + (long long)row * p.ldb + (CLAMP && n0 + nc >= p.N ? max(p.N - 8, 0) : n0 + nc);
        }
    }

    auto issue_direct = [&](int kt, int stage) {
        const int k0 = kt * BK;
        const unsigned as = lds0 + (unsigned)(stage * L::STAGE) * 2u;
        const unsigned bs = as + (unsigned)L::A_ELEMS * 2u;
#pragma unroll
        for (int q = 0; q < PA; ++q) {
            const u16* src;
            if constexpr (AMODE == A_ROW) {
                const bool in = a_in[q] && (!CUT || k0 + a_k[q] < p.K);
                src = in ? a_src[q] + k0 : zero_chunk;
            } else if constexpr (AMODE == A_COL) {
                const bool in = a_in[q] && (!CUT || k0 + a_k[q] < p.K);
                src = in ? a_src[q] + (long long)k0 * p.lda : zero_chunk;
            } else {
                if constexpr (one_tap) {
                    // the whole step lies in tap (cs_kh, cs_kw), whose offset is the same for every
                    // thread and moves on with the tap state: one add and two compares per chunk
                    const int hi = cv_hi0[q] + cs_kh, wi = cv_wi0[q] + cs_kw;
                    const bool in = a_in[q] && (unsigned)hi < (unsigned)p.H && (unsigned)wi < (unsigned)p.W;
                    const u16* inside = A + (cv_off[q] + cs_off);
                    src = in ? inside : zero_chunk;
                } else {
                    const int k = k0 + a_k[q];
                    const int tap = k / p.Cin, ci = k - tap * p.Cin;
                    const int kh = tap / p.KW, kw = tap - kh * p.KW;
                    const int hi = cv_hi0[q] + kh, wi = cv_wi0[q] + kw;
                    const bool in = a_in[q] && k < p.K && hi >= 0 && hi < p.H && wi >= 0 && wi < p.W;
                    src = in ? A + ((long long)(cv_base[q] + hi) * p.W + wi) * p.Cin + ci : zero_chunk;
                }
            }
            load_to_lds16(src, as + (unsigned)(q * NT) * 16u);
        }
#pragma unroll
        for (int q = 0; q < PB; ++q) {
            const bool in = b_in[q] && (!CUT || k0 + b_k[q] < p.K);
            const u16* src = in ? b_src[q] + (B_KMAJ ? (long long)k0 : (long long)k0 * p.ldb) : zero_chunk;
            load_to_lds16(src, bs + (unsigned)(q * NT) * 16u);
        }
    };

    auto issue_masked = [&](int kt, int stage) {
        const int k0 = kt * BK;
        u16* As = smem16 + stage * L::STAGE;
        u16* Bs = As + L::A_ELEMS;
#pragma unroll
        for (int q = 0; q < PA; ++q) {
            const int row = a_r + q * A_RPP;
            u16x8 v = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                if constexpr (AMODE == A_ROW) {
                    const int m = m0 + row, k = k0 + a_k[q] + e;
                    if (m < p.M && k < p.K) v[e] = A[(long long)m * p.lda + k];
                } else if constexpr (AMODE == A_COL) {
                    const int k = k0 + row, m = m0 + (a_cp ^ swz_j(row)) * 8 + e;
                    if (k < p.K && m < p.M) v[e] = A[(long long)k * p.lda + m];
                } else {
                    const int k = k0 + a_k[q] + e;
                    const int tap = k / p.Cin, ci = k - tap * p.Cin;
                    const int kh = tap / p.KW, kw = tap - kh * p.KW;
                    const int hi = cv_hi0[q] + kh, wi = cv_wi0[q] + kw;
                    if (a_in[q] && k < p.K && hi >= 0 && hi < p.H && wi >= 0 && wi < p.W)
                        v[e] = A[((long long)(cv_base[q] + hi) * p.W + wi) * p.Cin + ci];
                }
            }
            *(u16x8*)(As + (q * NT + tid) * 8) = v;
        }
#pragma unroll
        for (int q = 0; q < PB; ++q) {
            const int row = b_r + q * B_RPP;
            u16x8 v = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                if constexpr (B_KMAJ) {
                    const int n = n0 + row, k = k0 + b_k[q] + e;
                    if (n < p.N && k < p.K) v[e] = B[(long long)n * p.ldb + k];
                } else {
                    const int k = k0 + row, n = n0 + (b_cp ^ swz_j(row)) * 8 + e;
                    if (k < p.K && n < p.N) v[e] = B[(long long)k * p.ldb + n];
                }
            }
            *(u16x8*)(Bs + (q * NT + tid) * 8) = v;
        }
    };
    auto issue = [&](int kt_local, int stage) {
        if (!CUT || kt_local < n_direct) issue_direct(kb + kt_local, stage);
        else issue_masked(kb + kt_local, stage);
        if constexpr (AMODE == A_CONV) {
            cs_ci += BK;
            cs_off += BK;   // along ci and from one kw to the next the pixels' channels are consecutive
            while (cs_ci >= p.Cin) {
                cs_ci -= p.Cin;
                if (++cs_kw == p.KW) { cs_kw = 0; ++cs_kh; cs_off += (long long)(p.W - p.KW) * p.Cin; }
            }
        }
    };

    f32x16 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // [row][k] fragment: row wm0 + 32 i + li, chunk 2 g + lh of k step g, swizzled by the row
    int a_row_off[MI];
#pragma unroll
    for (int i = 0; i < MI; ++i) a_row_off[i] = (wm0 + i * 32 + li) * BK;
    int b_row_off[NI];   // the same for a k-contiguous B, whose rows are columns of C
#pragma unroll
    for (int j = 0; j < NI; ++j) b_row_off[j] = (wn0 + j * 32 + li) * BK;
    const int a_x = lh ^ swz_k(li);
    // [k][j] fragment by transposing reads: lane s of a 16-lane group points at row
    // 8 lh + s / 4 (and that row + 4) of the k step, columns 16 (lane / 16 % 2) + 4 (s % 4) of the block
    const int tr_row = 8 * lh + ((lane & 15) >> 2);
    const int tr_col = (lane & 16) + 4 * (lane & 3);
    const int tr_x = swz_j(tr_row);   // (row + 4) % 4 == row % 4: both reads share the mask

    // ---- one direct load: the x-th of the LPT loads that bring a tile in
    // (`ktest`: also test the chunk's k against K, which the ring of the peeled variant never needs)
    auto load_one = [&](int kt, int stage, int x, bool ktest) {
        const int k0 = kt * BK;
        const unsigned as = lds0 + (unsigned)(stage * L::STAGE) * 2u;
        const unsigned bs = as + (unsigned)L::A_ELEMS * 2u;
        if (x < PA) {
            const int q = x;
            const u16* src;
            if constexpr (AMODE == A_ROW) {
                const bool in = a_in[q] && (!(CUT || ktest) || k0 + a_k[q] < p.K);
                src = in ? a_src[q] + k0 : zero_chunk;
            } else if constexpr (AMODE == A_COL) {
                const bool in = a_in[q] && (!(CUT || ktest) || k0 + a_k[q] < p.K);
                src = in ? a_src[q] + (long long)k0 * p.lda : zero_chunk;
            } else {
                if constexpr (one_tap) {
                    // the whole step lies in tap (cs_kh, cs_kw), whose offset is the same for every
                    // thread and moves on with the tap state: one add and two compares per chunk
                    const int hi = cv_hi0[q] + cs_kh, wi = cv_wi0[q] + cs_kw;
                    const bool in = a_in[q] && (unsigned)hi < (unsigned)p.H && (unsigned)wi < (unsigned)p.W;
                    const u16* inside = A + (cv_off[q] + cs_off);
                    src = in ? inside : zero_chunk;
                } else {
                    const int k = k0 + a_k[q];
                    const int tap = k / p.Cin, ci = k - tap * p.Cin;
                    const int kh = tap / p.KW, kw = tap - kh * p.KW;
                    const int hi = cv_hi0[q] + kh, wi = cv_wi0[q] + kw;
                    const bool in = a_in[q] && k < p.K && hi >= 0 && hi < p.H && wi >= 0 && wi < p.W;
                    src = in ? A + ((long long)(cv_base[q] + hi) * p.W + wi) * p.Cin + ci : zero_chunk;
                }
            }
            load_to_lds16(src, as + (unsigned)(q * NT) * 16u);
        } else {
            const int q = x - PA;
            const bool in = b_in[q] && (!(CUT || ktest) || k0 + b_k[q] < p.K);
            const u16* src = in ? b_src[q] + (B_KMAJ ? (long long)k0 : (long long)k0 * p.ldb) : zero_chunk;
            load_to_lds16(src, bs + (unsigned)(q * NT) * 16u);
        }
    };
    auto issue_part = [&](int kt_local, int stage, int x) {
        if (!CUT || kt_local < n_direct) load_one(kb + kt_local, stage, x, false);
        else if (x == 0) issue_masked(kb + kt_local, stage);
        if constexpr (AMODE == A_CONV) {
            if (x == LPT - 1) {
                cs_ci += BK;
                cs_off += BK;   // along ci and from one kw to the next the pixels' channels are consecutive
                while (cs_ci >= p.Cin) {
                    cs_ci -= p.Cin;
                    if (++cs_kw == p.KW) { cs_kw = 0; ++cs_kh; cs_off += (long long)(p.W - p.KW) * p.Cin; }
                }
            }
        }
    };

    // ---- fragments: a k group (16 values of k = one MFMA per block) is fetched while the group
    // before it is multiplied, its LDS reads spread over that group's MFMAs.  A transposing
    // read returns half a fragment (4 values of k), so those operands are kept as two halves.
    constexpr int G = BK / 16;
    static_assert(G % 2 == 0, "the fragment double buffer alternates per group across steps");
    constexpr int NFRAG = (A_KMAJ ? MI : 2 * MI) + (B_KMAJ ? NI : 2 * NI);
    constexpr int NM = MI * NI;
    bf16x8 af[2][MI], bfull[2][NI];
    bf16x4 ah[2][MI][2], bh[2][NI][2];
    auto read_half = [&](const u16* t, int ld, int k, int col, int h) -> bf16x4 {
        const int c = col + tr_col;
        const u16* p0 = t + (k + tr_row + 4 * h) * ld + (((c >> 3) ^ tr_x) << 3) + (c & 7);
        return __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4_ptr)(p0));
    };
    auto frag_read = [&](int stage, int g, int x) {
        const u16* As = smem16 + stage * L::STAGE;
        const u16* Bs = As + L::A_ELEMS;
        if constexpr (A_KMAJ) {
            if (x < MI) {
                af[g & 1][x] = *(const bf16x8*)(As + a_row_off[x] + (((2 * g) ^ a_x) << 3));
                return;
            }
            x -= MI;
        } else {
            if (x < 2 * MI) {
                ah[g & 1][x >> 1][x & 1] = read_half(As, BM, g * 16, wm0 + (x >> 1) * 32, x & 1);
                return;
            }
            x -= 2 * MI;
        }
        if constexpr (B_KMAJ) bfull[g & 1][x] = *(const bf16x8*)(Bs + b_row_off[x] + (((2 * g) ^ a_x) << 3));
        else bh[g & 1][x >> 1][x & 1] = read_half(Bs, BN, g * 16, wn0 + (x >> 1) * 32, x & 1);
    };

    // ---- ring, as in the fp32 kernels: the one barrier of a step sits before its last k group
    for (int t = 0; t < D; ++t)
        if (t < nkp) issue(t, t);
    if (D <= n_direct) wait_loads_outstanding<(D - 1) * LPT>();
    else wait_loads_outstanding<0>();
    __syncthreads();
#pragma unroll
    for (int x = 0; x < NFRAG; ++x) frag_read(0, 0, x);
    int cur = 0;
    for (int kt = 0; kt < nkp; ++kt) {
        const int nxt = cur + 1 == STAGES ? 0 : cur + 1;
        const int fill = cur == 0 ? STAGES - 1 : cur - 1;
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const bool last = g == G - 1;
            if (last) {
                if (D >= 3 && kt + D <= n_direct) wait_loads_outstanding<(D >= 3 ? (D - 2) * LPT : 0)>();
                else wait_loads_outstanding<0>();
                __syncthreads();
            }
            // Behind the MFMAs of this group: first the fragments of the next one, all of them within
            // the first quarter of the group (a wave that is alone on its SIMD has nobody to hide an
            // LDS wait behind), then, in a step's last group, the loads of tile kt+D.
            constexpr int FQ = NM / 4 > 0 ? NM / 4 : 1;
            constexpr int FPER = (NFRAG + FQ - 1) / FQ;      // fragment reads behind one MFMA
            constexpr int FM = (NFRAG + FPER - 1) / FPER;    // MFMAs that carry them
            constexpr int LM = NM - FM > 0 ? NM - FM : 1;    // MFMAs that carry loads: the rest, or the last one
            constexpr int L0 = NM - LM;
            constexpr int LPER = (LPT + LM - 1) / LM;
#pragma unroll
            for (int m = 0; m < NM; ++m) {
                const int i = m / NI, j = m % NI;
                bf16x8 a;
                if constexpr (A_KMAJ) a = af[g & 1][i];
                else a = __builtin_shufflevector(ah[g & 1][i][0], ah[g & 1][i][1], 0, 1, 2, 3, 4, 5, 6, 7);
                bf16x8 b;
                if constexpr (B_KMAJ) b = bfull[g & 1][j];
                else b = __builtin_shufflevector(bh[g & 1][j][0], bh[g & 1][j][1], 0, 1, 2, 3, 4, 5, 6, 7);
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i][j], 0, 0, 0);
                if (m < FM) {
#pragma unroll
                    for (int u = 0; u < FPER; ++u) {
                        const int e = m * FPER + u;
                        if (e >= NFRAG) continue;
                        if (last) frag_read(nxt, 0, e);   // after the last step this reads a stage nobody multiplies
                        else frag_read(cur, g + 1, e);
                    }
                }
                if (last && m >= L0) {
#pragma unroll
                    for (int u = 0; u < LPER; ++u) {
                        const int e = (m - L0) * LPER + u;
                        if (e >= LPT) continue;
                        if (kt + D < nkp) issue_part(kt + D, fill, e);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        cur = nxt;
    }

    if constexpr (CLAMP) {
        if (nkp < nk) {
            // the partial last step into stage 0, multiplied group by group: chunks past K come
            // from the block of zeros, or, when K cuts a chunk of a k-contiguous operand or the
            // tile's chunks are cut along M or N, the whole tile goes through registers with
            // element masks
            __syncthreads();   // everybody has left the ring
            if ((p.K % 8) || cut_tile) {
                issue_masked(kb + nkp, 0);
            } else {
#pragma unroll
                for (int x = 0; x < LPT; ++x) load_one(kb + nkp, 0, x, true);
                wait_loads_outstanding<0>();
            }
            __syncthreads();
#pragma unroll
            for (int g = 0; g < G; ++g) {
#pragma unroll
                for (int x = 0; x < NFRAG; ++x) frag_read(0, g, x);
#pragma unroll
                for (int m = 0; m < NM; ++m) {
                const int i = m / NI, j = m % NI;
                bf16x8 a;
                if constexpr (A_KMAJ) a = af[g & 1][i];
                else a = __builtin_shufflevector(ah[g & 1][i][0], ah[g & 1][i][1], 0, 1, 2, 3, 4, 5, 6, 7);
                bf16x8 b;
                if constexpr (B_KMAJ) b = bfull[g & 1][j];
                else b = __builtin_shufflevector(bh[g & 1][j][0], bh[g & 1][j][1], 0, 1, 2, 3, 4, 5, 6, 7);
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i][j], 0, 0, 0);
                }
            }
        }
    }
    finish_tile<T>(p, acc, C, slot, split, nsplit, m0, n0, wm0, wn0, interior);
}

template <class T, int AMODE>
hipError_t launch_mode(int variant, const KArgs& a, int batch, hipStream_t s) {
    const dim3 grid(a.split_first + (a.tiles_m * a.tiles_n - a.split_first) * a.split_k, batch, 1), block(T::NT, 1, 1);
    void (*fn)(const KArgs) = nullptr;
    int bytes, one_tap = 0;
    if constexpr ((AMODE == A_ROW_BT || AMODE == A_COL_BT) && T::SCHED < 4) {
        return hipErrorInvalidValue;   // a transposed right operand exists in the direct-to-LDS forms only
    } else if constexpr (T::SCHED >= 4) {
        if (variant == 2) return hipErrorInvalidValue;   // whole 16-byte chunks only
        bytes = LdsDirect<T>::BYTES;
        fn = variant == 0 ? gemm_bf16_direct_kernel<T, AMODE, 0>
             : variant == 3 ? gemm_bf16_direct_kernel<T, AMODE, 2> : gemm_bf16_direct_kernel<T, AMODE, 1>;
        if constexpr (AMODE == A_CONV) {
            if (a.Cin % T::BK == 0) {
                one_tap = 1;
                fn = variant == 0 ? gemm_bf16_direct_kernel<T, AMODE, 0, true>
                     : variant == 3 ? gemm_bf16_direct_kernel<T, AMODE, 2, true> : gemm_bf16_direct_kernel<T, AMODE, 1, true>;
            }
        }
    } else {
        constexpr int A_SIZE = (AMODE != A_COL) ? T::BM * T::LDK : T::BK * T::LDA_T;
        bytes = 2 * (A_SIZE + T::BK * T::LDB) * 2;
        switch (variant) {
            case 0: fn = gemm_bf16_kernel<T, AMODE, 8, false>; break;
            case 1:
            case 3: fn = gemm_bf16_kernel<T, AMODE, 8, true>; break;
            default: fn = gemm_bf16_kernel<T, AMODE, 1, true>; break;
        }
    }
    static std::atomic<bool> attr_done[8];   // per kernel function; setting the attribute twice is harmless
    const int fi = variant + 4 * one_tap;
    if (bytes > 48 * 1024 && !attr_done[fi].load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute((const void*)fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
        if (e != hipSuccess) return e;
        attr_done[fi].store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL(fn, grid, block, bytes, s, a);
    return hipGetLastError();
}

}  // namespace
}  // namespace tsg

// The instantiated tile shapes: X(BM, BN, BK, WM, WN, min waves per SIMD, SCHED).
#define TSG_BF16_TILES(X)           \
    X(256, 256, 64, 128, 64, 2, 1)  \
    X(256, 256, 64, 128, 64, 2, 0)  \
    X(256, 256, 64, 64, 128, 2, 1)  \
    X(256, 256, 32, 128, 64, 2, 1)  \
    X(256, 128, 64, 64, 64, 2, 1)   \
    X(128, 128, 64, 64, 64, 2, 1)   \
    X(128, 128, 32, 64, 64, 2, 1)   \
    X(128, 128, 32, 64, 64, 2, 0)   \
    X(64, 64, 64, 32, 32, 2, 1)     \
    X(64, 64, 64, 32, 32, 2, 0)     \
    X(256, 256, 32, 128, 64, 2, 4)  \
    X(256, 256, 32, 128, 64, 2, 5)  \
    X(256, 256, 32, 128, 128, 1, 4) \
    X(256, 256, 32, 128, 128, 1, 5) \
    X(256, 128, 64, 64, 64, 2, 4)   \
    X(128, 128, 64, 64, 64, 2, 4)   \
    X(128, 128, 32, 64, 64, 2, 5)   \
    X(64, 64, 64, 32, 32, 2, 4)

#define TSG_BF16_DEFINE_MODE(FN, AMODE)                                                             \
    namespace tsg {                                                                                 \
    hipError_t FN(int tile, int variant, const KArgs& a, int batch, hipStream_t s) {                \
        int idx = 0;                                                                                \
        TSG_BF16_TILES(TSG_BF16_CASE_##AMODE)                                                       \
        return hipErrorInvalidValue;                                                                \
    }                                                                                               \
    }
#define TSG_BF16_CASE_A_ROW(bm, bn, bk, wm, wn, mw, sc) \
    if (tile == idx++) return launch_mode<Tile<bm, bn, bk, wm, wn, mw, sc>, A_ROW>(variant, a, batch, s);
#define TSG_BF16_CASE_A_COL(bm, bn, bk, wm, wn, mw, sc) \
    if (tile == idx++) return launch_mode<Tile<bm, bn, bk, wm, wn, mw, sc>, A_COL>(variant, a, batch, s);
#define TSG_BF16_CASE_A_CONV(bm, bn, bk, wm, wn, mw, sc) \
    if (tile == idx++) return launch_mode<Tile<bm, bn, bk, wm, wn, mw, sc>, A_CONV>(variant, a, batch, s);
#define TSG_BF16_CASE_A_ROW_BT(bm, bn, bk, wm, wn, mw, sc) \
    if (tile == idx++) return launch_mode<Tile<bm, bn, bk, wm, wn, mw, sc>, A_ROW_BT>(variant, a, batch, s);
#define TSG_BF16_CASE_A_COL_BT(bm, bn, bk, wm, wn, mw, sc) \
    if (tile == idx++) return launch_mode<Tile<bm, bn, bk, wm, wn, mw, sc>, A_COL_BT>(variant, a, batch, s);

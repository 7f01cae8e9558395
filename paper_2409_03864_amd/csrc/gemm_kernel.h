// Contraction kernels for gfx950: C = +-op(A).op(B) (+C), fp32 accumulate on the matrix cores.
// One skeleton for every operand type and MFMA block shape (gemm_elem.h holds what differs).
//
// One workgroup computes a BM x BN tile of C (the i/j tiling of Case Study 4, Fig. 8); the k
// loop advances in BK steps.  Each wavefront owns a WM x WN sub-tile built from MFMA blocks:
// the fixed-size inner matmul that the paper hands to a microkernel library is here an MFMA
// sequence.
//
// The rewrites of Case Study 3 live in the address generators only:
//   A_ROW  : op(A)(i,k) = A[i*lda + k]
//   A_COL  : op(A)(i,k) = A[k*lda + i]        transposed operand, read in place
//   A_CONV : op(A)(m,k) = x[n][ho*sh+kh-ph][wo*sw+kw-pw][ci], k = (kh*KW+kw)*Cin+ci,
//            and 0 WITHOUT a memory access where the coordinate is in the padding
//   *_BT   : the right operand stored transposed too (B is N x K), read in place
// The main/remainder split of Fig. 8 is taken per tile: tiles inside [0,m_main) x [0,n_main)
// and k steps below k_full run unmasked, the remainder runs the masked or clamped forms,
// chosen by a wavefront-uniform branch.
//
// Split k: with split_k = S > 1, S workgroups share one tile of C, each taking a contiguous
// range of k steps.  Each parks its partial tile in the workspace and bumps the tile's arrival
// counter; the workgroup that arrives last adds the S partials in split order (so the sum does
// not depend on who was last), applies the epilogue and resets the counter.
//
// Three kernel forms (`sched`, a tunable like the tile sizes):
//   1     one MFMA block of C per workgroup, k dealt over its four waves, operands straight
//         from global memory into the MFMA's registers: for products too small to give the
//         forms below a tile per compute unit.  fp32 GEMM only, no k split across workgroups.
//   0     register staging: the tiles of step t+1 are fetched into registers while step t is
//         multiplied from LDS (two padded stages, one barrier per step, instruction order left
//         to the compiler).  Serves every access width, so it is also the last alternative.
//   4, 5  direct staging: tiles travel from global memory straight into a ring of 3 / 4
//         unpadded LDS stages (two / three k steps in flight), 16-byte accesses only.
#pragma once
#include <atomic>
#include <type_traits>

#include "gemm_elem.h"

namespace tsg {
namespace {

constexpr unsigned FLAG_NEGATE = 1u, FLAG_ACCUMULATE = 2u;
constexpr int kXcds = 8;      // workgroup ids are dealt round-robin over this many L2 domains
constexpr int kGroupM = 8;    // tile rows per raster group

template <class E_, int BM_, int BN_, int BK_, int WM_, int WN_, int MINW_, int SCHED_>
struct Tile {
    using E = E_;
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_, MINW = MINW_, SCHED = SCHED_;
    static constexpr int WAVES_M = BM / WM, WAVES_N = BN / WN;
    static constexpr int NT = SCHED == 1 ? 256 : 64 * WAVES_M * WAVES_N;   // (sched 1: four waves share one block along k)
    static constexpr int MI = WM / E::BLK, NI = WN / E::BLK;
    static_assert(BM % WM == 0 && BN % WN == 0 && WM % E::BLK == 0 && WN % E::BLK == 0 && BK % E::KG == 0, "tile");
    static_assert(SCHED == 0 || SCHED == 1 || SCHED == 4 || SCHED == 5, "kernel form");
    static_assert(SCHED != 1 || (BM == E::BLK && BN == E::BLK && WM == BM && WN == BN && BK == 4 * E::KG), "block form");
};

__device__ __forceinline__ void tile_coords(const KArgs& p, int bid, int& tm, int& tn) {
    if (p.raster) {
        // Give each XCD a contiguous range of tile ids, then walk the range in groups of
        // kGroupM tile rows so that concurrently resident tiles share A and B panels in
        // that XCD's L2.  (every quantity is non-negative: unsigned divisions, which are cheaper)
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

// This workgroup's k steps: [kb, kb + nk) of the (K + BK - 1) / BK steps of the whole loop.
// (unsigned 32-bit: nk_all < 2^27 and nsplit <= 16; an unsplit tile divides nothing)
__device__ __forceinline__ void k_range(int nk_all, int split, int nsplit, int& kb, int& nk) {
    kb = 0;
    nk = nk_all;
    if (nsplit > 1) {
        kb = (int)((unsigned)(nk_all * split) / (unsigned)nsplit);
        nk = (int)((unsigned)(nk_all * (split + 1)) / (unsigned)nsplit) - kb;
    }
}

// Where a run of four accumulator rows starts in a window of a larger NHWC tensor: element
// offset of its first pixel, and that pixel's (wo, ho).  A lane's runs lie a fixed number of rows
// apart down its wave tile (8 with 32 x 32 blocks, 16 with 16 x 16), so only the first is decoded
// with divisions (about forty four-cycle instructions each, which made the windowed epilogue a
// microsecond longer than the plain one); the others step from it, wrapping wo and ho.
struct RunStart { long long off; int wo, ho; };

template <class T>
struct WindowCursor {
    RunStart cur;
    bool started = false, seeded = false;
    // start from a first run that somebody decoded before (the early read of the old values)
    __device__ __forceinline__ void seed(const RunStart& first) { cur = first; started = true; seeded = true; }
    // the run that starts at row `row`; calls come in increasing row order, `step` rows apart
    __device__ __forceinline__ void next(const KArgs& p, int row, RunStart& out) {
        constexpr int STEP = T::E::BLK == 32 ? 8 : 16;
        static_assert(T::E::BLK == 32 ? T::E::NACC == 16 : T::E::NACC == 4, "accumulator rows per block");
        if (seeded) {
            seeded = false;   // the seed is this first run
        } else if (!started) {
            // (non-negative: unsigned divisions)
            const unsigned tq = (unsigned)row / (unsigned)p.Wo, nq = tq / (unsigned)p.Ho;
            cur.wo = row - (int)tq * p.Wo;
            cur.ho = (int)(tq - nq * (unsigned)p.Ho);
            cur.off = (long long)nq * p.y_sn + (long long)cur.ho * p.y_sh + (long long)cur.wo * p.y_sw;
            started = true;
        } else {
            const long long wrap_w = p.y_sh - (long long)p.Wo * p.y_sw, wrap_h = p.y_sn - (long long)p.Ho * p.y_sh;
            cur.wo += STEP;
            cur.off += STEP * p.y_sw;
            while (cur.wo >= p.Wo) {
                cur.wo -= p.Wo;
                cur.off += wrap_w;
                if (++cur.ho == p.Ho) { cur.ho = 0; cur.off += wrap_h; }
            }
        }
        out = cur;
    }
    // the run starts of block row i of the wave tile (nothing to do for a plain matrix)
    __device__ __forceinline__ void block(const KArgs& p, int m0, int wm0, int i, RunStart (&rs)[T::E::NACC / 4]) {
        if (!p.y_window) return;
        const int lane = threadIdx.x & 63;
#pragma unroll
        for (int rg = 0; rg < T::E::NACC / 4; ++rg) next(p, m0 + wm0 + i * T::E::BLK + T::E::acc_row(4 * rg, lane), rs[rg]);
    }
};

// The outputs a lane holds for MFMA block (i, j) of its wave tile, in accumulator order:
// f(r, address of the element, whether it lies inside C).  The rows of a run of four registers
// are consecutive and runs lie 8 rows apart: in a plain matrix the row pointer steps, no
// multiply per element; in a window of a larger NHWC tensor the first row of a run is decoded
// to (n, ho, wo) and the others step from it.
template <class T, bool CHECK, class F>
__device__ __forceinline__ void visit_block(const KArgs& p, float* __restrict__ C, int m0, int n0, int wm0, int wn0,
                                            int i, int j, const RunStart (&rs)[T::E::NACC / 4], F&& f) {
    using E = typename T::E;
    constexpr int BLK = E::BLK, NACC = E::NACC;
    const int lane = threadIdx.x & 63;
    const int col = n0 + wn0 + j * BLK + (lane & (BLK - 1));
    const int row_b = m0 + wm0 + i * BLK;
    if (p.y_window) {
        if ((p.Wo & 3) == 0) {
            // a run starts at a multiple of four rows, so with Wo a multiple of four it never
            // crosses from one image row into the next: four pixels a fixed stride apart
#pragma unroll
            for (int rg = 0; rg < NACC / 4; ++rg) {
                const int row0 = row_b + E::acc_row(4 * rg, lane);
                float* ptr = C + rs[rg].off + col;
#pragma unroll
                for (int e = 0; e < 4; ++e) f(4 * rg + e, ptr + e * p.y_sw, !CHECK || (row0 + e < p.M && col < p.N));
            }
            return;
        }
        const long long wrap_w = p.y_sh - (long long)p.Wo * p.y_sw, wrap_h = p.y_sn - (long long)p.Ho * p.y_sh;
#pragma unroll
        for (int rg = 0; rg < NACC / 4; ++rg) {
            const int row0 = row_b + E::acc_row(4 * rg, lane);
            int wo = rs[rg].wo, ho = rs[rg].ho;
            float* ptr = C + rs[rg].off + col;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                f(4 * rg + e, ptr, !CHECK || (row0 + e < p.M && col < p.N));
                ptr += p.y_sw;
                if (++wo == p.Wo) {
                    wo = 0;
                    ptr += wrap_w;
                    if (++ho == p.Ho) { ho = 0; ptr += wrap_h; }
                }
            }
        }
        return;
    }
    float* rp = C + (long long)(row_b + E::acc_row(0, lane)) * p.ldc + col;   // row of r = 0
#pragma unroll
    for (int r = 0; r < NACC; ++r) {
        f(r, rp, !CHECK || (row_b + E::acc_row(r, lane) < p.M && col < p.N));
        rp += (r & 3) == 3 ? 5 * p.ldc : p.ldc;
    }
}

// The old values of C for `C += ...` (the form of Fig. 7), fetched BEFORE the k loop by tiles
// small enough to spare the registers: the epilogue of a small tile is a large part of its run
// time, and reading the old values there added a round trip to memory to it.  Nobody else
// writes this tile of C during the launch, so the early read sees the same values.  Not used
// when k is split: only the last arrival adds the old values, and it is not known in advance.
template <class T>
struct OldC {
    static constexpr bool ON = T::MI * T::NI * T::E::NACC <= 32;
    float v[ON ? T::MI : 1][ON ? T::NI : 1][ON ? T::E::NACC : 1];
    bool loaded = false;
    RunStart first;   // the lane's first run in a window, decoded here once for the epilogue too

    __device__ __forceinline__ void fetch(const KArgs& p, float* __restrict__ C, int m0, int n0, int wm0, int wn0,
                                          bool interior, int nsplit) {
        if constexpr (ON) {
            if (!(p.flags & FLAG_ACCUMULATE) || nsplit > 1) return;
            loaded = true;
            WindowCursor<T> wc;
#pragma unroll
            for (int i = 0; i < T::MI; ++i) {
                RunStart rs[T::E::NACC / 4];
                wc.block(p, m0, wm0, i, rs);
                if (i == 0 && p.y_window) first = rs[0];
#pragma unroll
                for (int j = 0; j < T::NI; ++j) {
                    if (interior)
                        visit_block<T, false>(p, C, m0, n0, wm0, wn0, i, j, rs, [&](int r, float* ptr, bool) { v[i][j][r] = *ptr; });
                    else
                        visit_block<T, true>(p, C, m0, n0, wm0, wn0, i, j, rs,
                                             [&](int r, float* ptr, bool ok) { v[i][j][r] = ok ? *ptr : 0.f; });
                }
            }
        }
    }
};

// What follows the k loop.  Split k: park the partial tile, count the arrival, and let the
// last arrival add the partials in split order.  Epilogue: sign, optional accumulate, masked
// at the remainder, optionally addressed into a window of a larger NHWC tensor.
//
// The hand-off of the partial tiles uses device-scope relaxed atomics and no fence.  What it
// relies on: a device-scope store is written through to the memory side of the per-XCD L2s
// (the point where the eight L2s of the device agree) and is counted by vmcnt until that write
// is acknowledged; a device-scope load is served from there, never from a line cached before;
// a device-scope read-modify-write is performed there.  So: every wave waits for its stores
// (s_waitcnt vmcnt(0), which the compiler may not move code across), the barrier collects the
// waves, one lane counts the arrival, and whoever draws the last count reads partials that are
// all in memory.  A release / acquire pair at device scope would give the language-level edge
// but costs a write-back and an invalidate of the whole L2 per workgroup (measured: 25 us per
// launch), for lines this protocol never needs.
template <class T>
__device__ __forceinline__ void finish_tile(const KArgs& p, typename T::E::acc_t (&acc)[T::MI][T::NI],
                                            float* __restrict__ C, int slot, int split, int nsplit, int m0, int n0,
                                            int wm0, int wn0, bool interior, const OldC<T>& oldc) {
    using E = typename T::E;
    constexpr int BM = T::BM, BN = T::BN, NT = T::NT, MI = T::MI, NI = T::NI, NACC = E::NACC;
    const int tid = threadIdx.x;
    if (nsplit > 1) {
        __shared__ int arrived;
        float* ws = p.ws + (long long)slot * nsplit * (BM * BN);
        // a partial tile is kept in register order
        float* mine = ws + (long long)split * (BM * BN);
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int r = 0; r < NACC; ++r)
                    __hip_atomic_store(mine + ((i * NI + j) * NACC + r) * NT + tid, acc[i][j][r], __ATOMIC_RELAXED,
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
                float t[NI][NACC];
#pragma unroll
                for (int j = 0; j < NI; ++j)
#pragma unroll
                    for (int r = 0; r < NACC; ++r)
                        t[j][r] = __hip_atomic_load(part + ((i * NI + j) * NACC + r) * NT + tid, __ATOMIC_RELAXED,
                                                    __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
                for (int j = 0; j < NI; ++j)
#pragma unroll
                    for (int r = 0; r < NACC; ++r) acc[i][j][r] = sp == 0 ? t[j][r] : acc[i][j][r] + t[j][r];
            }
        if (tid == 0)   // ready for the next launch on this workspace
            __hip_atomic_store(p.counters + slot, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }

    // With ACCUMULATE the old values of a block are all loaded before its first store: a load
    // behind a store to an address the compiler cannot tell apart would wait for it, one round
    // trip to memory per element.  Small tiles bring them in before the k loop (OldC).
    const bool neg = p.flags & FLAG_NEGATE, accum = p.flags & FLAG_ACCUMULATE;
    // The bounds tests and the read of the old values are compiled into copies of their own,
    // chosen once per tile: with the tests beside every element an interior tile of the
    // remainder variant spent three times as long here.
    auto emit = [&](auto check_tag, auto accum_tag) {
        constexpr bool CHECK = decltype(check_tag)::value, ACCUM = decltype(accum_tag)::value;
        WindowCursor<T> wc;
        if constexpr (OldC<T>::ON) {
            if (oldc.loaded && p.y_window) wc.seed(oldc.first);
        }
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            RunStart rs[NACC / 4];
            wc.block(p, m0, wm0, i, rs);
#pragma unroll
            for (int j = 0; j < NI; ++j) {
                float old[NACC];
                if constexpr (ACCUM) {
                    bool have = false;
                    if constexpr (OldC<T>::ON) {
                        if (oldc.loaded) {
                            have = true;
#pragma unroll
                            for (int r = 0; r < NACC; ++r) old[r] = oldc.v[i][j][r];
                        }
                    }
                    if (!have)
                        visit_block<T, CHECK>(p, C, m0, n0, wm0, wn0, i, j, rs,
                                              [&](int r, float* ptr, bool ok) { old[r] = ok ? *ptr : 0.f; });
                }
                visit_block<T, CHECK>(p, C, m0, n0, wm0, wn0, i, j, rs, [&](int r, float* ptr, bool ok) {
                    const float v = acc[i][j][r];
                    const float sv = neg ? -v : v;
                    if (ok) *ptr = ACCUM ? sv + old[r] : sv;   // no add without the flag: -0 stays -0
                });
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

// ---------------------------------------------------------------------------------------
// sched 1: one MFMA block of C per workgroup, for products so small that the tiled forms leave
// most of the chip idle (256^3 is 16 tiles of 64 x 64, but 256 blocks of 16 x 16).  The k loop
// is dealt over the four waves of the workgroup, one per SIMD: k group g belongs to wave g % 4,
// and a step of BK = 4 groups is one group per wave.  Operands go from global memory straight
// into the MFMA's operand registers (lane (l, q) of a wave holds k = 4 q .. 4 q + 3 of row or
// column l of its group: a 16-byte access where the operand is k-contiguous, four coalesced
// scalars where it is not), four groups per wave in flight together: no LDS staging and no
// barrier in the loop.  The waves' partial blocks meet in LDS and wave 0 adds them in wave
// order, so the order of summation is fixed.  Remainder (VARIANT 1): rows and columns past the end
// are clamped to the last valid one (their products only reach elements of C that are never
// stored) and only the last, partial k group is masked, element by element; VARIANT 2 is the
// same with scalar accesses throughout; VARIANT 0 has no remainder code.
template <class T, int AMODE, int VARIANT>
__global__ void __launch_bounds__(256) gemm_block_kernel(const KArgs p) {
    using E = typename T::E;
    using frag = typename E::frag;
    using chunk_u = typename E::chunk_u;
    static_assert(T::SCHED == 1 && T::MI == 1 && T::NI == 1 && sizeof(typename E::elem) == 4, "one fp32 block");
    static_assert(AMODE != A_CONV, "no gathered operand in this form");
    constexpr int BLK = E::BLK, KG = E::KG, NACC = E::NACC, WAVES = 4, U = 4;
    constexpr bool EDGE = VARIANT != 0, WIDE = VARIANT != 2;
    constexpr bool A_KMAJ = AMODE == A_ROW || AMODE == A_ROW_BT;
    constexpr bool B_KMAJ = AMODE == A_ROW_BT || AMODE == A_COL_BT;
    __shared__ float part[WAVES - 1][NACC][64];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int li = lane & (BLK - 1), q = lane / BLK;
    int tm, tn;
    tile_coords(p, blockIdx.x, tm, tn);
    const int m0 = tm * BLK, n0 = tn * BLK;
    const float* __restrict__ A = (const float*)p.A + (long long)blockIdx.y * p.stride_a;
    const float* __restrict__ B = (const float*)p.B + (long long)blockIdx.y * p.stride_b;
    float* __restrict__ C = p.C + (long long)blockIdx.y * p.stride_c;

    const int row = EDGE ? min(m0 + li, p.M - 1) : m0 + li;
    const int col = EDGE ? min(n0 + li, p.N - 1) : n0 + li;
    // the lane's row of op(A) and column of op(B) at k = 0
    const float* a0 = A_KMAJ ? A + (long long)row * p.lda : A + row;
    const float* b0 = B_KMAJ ? B + (long long)col * p.ldb : B + col;
    const bool interior = !EDGE || (m0 + BLK <= p.M && n0 + BLK <= p.N);

    typename E::acc_t acc[1][1];
#pragma unroll
    for (int r = 0; r < NACC; ++r) acc[0][0][r] = 0.f;
    OldC<T> oldc;
    if (wave == 0) oldc.fetch(p, C, m0, n0, 0, 0, interior, 1);

    const int ngroups = (p.K + KG - 1) / KG;
    for (int g0 = wave; g0 < ngroups; g0 += WAVES * U) {
        frag a[U], b[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int g = g0 + WAVES * u;
            const int k = g * KG + 4 * q;
            a[u] = E::zero();
            b[u] = E::zero();
            if (g >= ngroups) continue;   // the same for the whole wave; zeros add nothing
            if (!EDGE || (g + 1) * KG <= p.K) {   // a whole group (again the same for the whole wave)
                if constexpr (A_KMAJ && WIDE) {
                    a[u] = *(const chunk_u*)(a0 + k);
                } else {
#pragma unroll
                    for (int t = 0; t < 4; ++t) a[u][t] = A_KMAJ ? a0[k + t] : a0[(long long)(k + t) * p.lda];
                }
                if constexpr (B_KMAJ && WIDE) {
                    b[u] = *(const chunk_u*)(b0 + k);
                } else {
#pragma unroll
                    for (int t = 0; t < 4; ++t) b[u][t] = B_KMAJ ? b0[k + t] : b0[(long long)(k + t) * p.ldb];
                }
            } else {
#pragma unroll
                for (int t = 0; t < 4; ++t) {
                    const int kk = k + t;
                    if (kk < p.K) {
                        a[u][t] = A_KMAJ ? a0[kk] : a0[(long long)kk * p.lda];
                        b[u][t] = B_KMAJ ? b0[kk] : b0[(long long)kk * p.ldb];
                    }
                }
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int t = 0; t < 4; ++t) acc[0][0] = E::mfma(a[u], b[u], acc[0][0], t);
    }

    if (wave > 0) {
#pragma unroll
        for (int r = 0; r < NACC; ++r) part[wave - 1][r][lane] = acc[0][0][r];
    }
    __syncthreads();
    if (wave != 0) return;
#pragma unroll
    for (int w = 0; w < WAVES - 1; ++w)
#pragma unroll
        for (int r = 0; r < NACC; ++r) acc[0][0][r] += part[w][r][lane];
    finish_tile<T>(p, acc, C, 0, 0, 1, m0, n0, 0, 0, interior, oldc);
}

// ---------------------------------------------------------------------------------------
// sched 0: register staging, two padded LDS stages.
template <class T, int AMODE>
struct Lds {
    using E = typename T::E;
    // k-contiguous rows are padded so that the 16-byte fragment reads of 16 consecutive rows
    // fall in distinct banks; [k][j] tiles so that the k slots of one read do.
    static constexpr int A_LD = (AMODE == A_COL) ? T::BM + E::PAD_J : T::BK + E::PAD_K;
    static constexpr int A_ROWS = (AMODE == A_COL) ? T::BK : T::BM;
    static constexpr int B_LD = T::BN + E::PAD_J;
    static constexpr int A_SIZE = A_ROWS * A_LD, B_SIZE = T::BK * B_LD;
    static constexpr int STAGE = A_SIZE + B_SIZE;
    static constexpr int BYTES = 2 * STAGE * (int)sizeof(typename E::elem);
};

template <class T, int AMODE, int VEC, bool EDGE>
__global__ void __launch_bounds__(T::NT, T::MINW) gemm_staged_kernel(const KArgs p) {
    using E = typename T::E;
    using elem = typename E::elem;
    using chunk = typename E::chunk;
    using chunk_u = typename E::chunk_u;
    using frag = typename E::frag;
    constexpr int BM = T::BM, BN = T::BN, BK = T::BK, NT = T::NT, MI = T::MI, NI = T::NI, V = E::V, BLK = E::BLK;
    static_assert(VEC == 1 || VEC == V, "scalar accesses or whole chunks");
    using L = Lds<T, AMODE>;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    elem* smem = (elem*)smem_raw;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave / T::WAVES_N) * T::WM, wn0 = (wave % T::WAVES_N) * T::WN;
    const int li = lane & (BLK - 1), lk = lane / BLK;

    const int tiles = p.tiles_m * p.tiles_n;
    int tile, split, nsplit, slot;
    decode_block(p, tiles, tile, split, nsplit, slot);
    int tm, tn;
    tile_coords(p, tile, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;
    const elem* __restrict__ A = (const elem*)p.A + (long long)blockIdx.y * p.stride_a;
    const elem* __restrict__ B = (const elem*)p.B + (long long)blockIdx.y * p.stride_b;
    float* __restrict__ C = p.C + (long long)blockIdx.y * p.stride_c;

    // Remainder tiles (Fig. 8's %rest) take the masked loaders for every k step.
    const bool interior = !EDGE || (m0 + BM <= p.m_main && n0 + BN <= p.n_main);
    int kb, nk;
    k_range((p.K + BK - 1) / BK, split, nsplit, kb, nk);

    // ---- per-thread global->LDS assignment: chunks along the contiguous dimension
    constexpr int A_CPR = (AMODE == A_COL) ? BM / V : BK / V;   // chunks per stored row
    constexpr int A_RPP = NT / A_CPR;                            // rows per pass
    constexpr int A_ROWS = L::A_ROWS;
    constexpr int PA = A_ROWS / A_RPP;
    constexpr int B_CPR = BN / V, B_RPP = NT / B_CPR, PB = BK / B_RPP;
    static_assert(NT % A_CPR == 0 && A_ROWS % A_RPP == 0 && PA >= 1, "A staging shape");
    static_assert(NT % B_CPR == 0 && BK % B_RPP == 0 && PB >= 1, "B staging shape");
    const int a_r = tid / A_CPR, a_c = (tid % A_CPR) * V;
    const int b_r = tid / B_CPR, b_c = (tid % B_CPR) * V;

    // convolution: decode this thread's output pixels once
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
                cv_hi0[q] = -(1 << 28);   // every tap reads as padding
                cv_wi0[q] = 0;
            }
        }
    }

    // convolution: (kh, kw, ci) of the first k of the next step to load.  Steps are loaded in
    // order, so the triple is advanced instead of being divided out of k every time; when Cin
    // is a multiple of BK a whole step lies inside one tap and no chunk needs a division.
    int cs_kh = 0, cs_kw = 0, cs_ci = 0;
    const bool one_tap = AMODE == A_CONV && p.Cin % BK == 0;
    if constexpr (AMODE == A_CONV) {
        const int k = kb * BK, tap = k / p.Cin;
        cs_ci = k - tap * p.Cin;
        cs_kh = tap / p.KW;
        cs_kw = tap - cs_kh * p.KW;
    }

    chunk ra[PA], rb[PB];

    // One element of op(A) for the scalar path (row/col relative to the problem).
    auto a_elem = [&](int q, int row_or_k, int e) -> elem {
        if constexpr (AMODE == A_ROW) {
            const int m = m0 + row_or_k, k = e;
            return (m < p.M && k < p.K) ? A[(long long)m * p.lda + k] : (elem)0;
        } else if constexpr (AMODE == A_COL) {
            const int k = row_or_k, m = e;
            return (k < p.K && m < p.M) ? A[(long long)k * p.lda + m] : (elem)0;
        } else {
            const int k = e;
            if (k >= p.K) return (elem)0;
            const int tap = k / p.Cin, ci = k - tap * p.Cin;
            const int kh = tap / p.KW, kw = tap - kh * p.KW;
            const int hi = cv_hi0[q] + kh, wi = cv_wi0[q] + kw;
            if (hi < 0 || hi >= p.H || wi < 0 || wi >= p.W) return (elem)0;
            return A[((long long)(cv_base[q] + hi) * p.W + wi) * p.Cin + ci];
        }
    };

    auto load_tiles = [&](int kt_local) {
        const int kt = kb + kt_local;
        const bool fast = EDGE ? (interior && kt < p.k_full) : true;
        const int k0 = kt * BK;
        // ---------------- A
#pragma unroll
        for (int q = 0; q < PA; ++q) {
            const int r = a_r + q * A_RPP;
            if constexpr (AMODE == A_ROW) {
                const int k = k0 + a_c;
                if (VEC == V && (fast || (m0 + r < p.M && k + V <= p.K))) {
                    ra[q] = *(const chunk_u*)(A + (long long)(m0 + r) * p.lda + k);
                } else {
#pragma unroll
                    for (int e = 0; e < V; ++e) ra[q][e] = a_elem(q, r, k + e);
                }
            } else if constexpr (AMODE == A_COL) {
                const int k = k0 + r, m = m0 + a_c;
                if (VEC == V && (fast || (k < p.K && m + V <= p.M))) {
                    ra[q] = *(const chunk_u*)(A + (long long)k * p.lda + m);
                } else {
#pragma unroll
                    for (int e = 0; e < V; ++e) ra[q][e] = a_elem(q, k, m + e);
                }
            } else {
                const int k = k0 + a_c;
                if constexpr (VEC == V) {
                    // Cin % V == 0: the chunk lies inside one tap
                    chunk v = E::zero();
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
                            v = *(const chunk_u*)(A + ((long long)(cv_base[q] + hi) * p.W + wi) * p.Cin + ci);
                    }
                    ra[q] = v;
                } else {
#pragma unroll
                    for (int e = 0; e < V; ++e) ra[q][e] = a_elem(q, r, k + e);
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
        // ---------------- B (K x N, j contiguous)
#pragma unroll
        for (int q = 0; q < PB; ++q) {
            const int k = k0 + b_r + q * B_RPP, n = n0 + b_c;
            if (VEC == V && (fast || (k < p.K && n + V <= p.N))) {
                rb[q] = *(const chunk_u*)(B + (long long)k * p.ldb + n);
            } else {
#pragma unroll
                for (int e = 0; e < V; ++e)
                    rb[q][e] = (k < p.K && n + e < p.N) ? B[(long long)k * p.ldb + n + e] : (elem)0;
            }
        }
    };

    auto store_tiles = [&](int stage) {
        elem* As = smem + stage * L::STAGE;
        elem* Bs = As + L::A_SIZE;
#pragma unroll
        for (int q = 0; q < PA; ++q)
            *(chunk*)(As + (a_r + q * A_RPP) * L::A_LD + a_c) = ra[q];
#pragma unroll
        for (int q = 0; q < PB; ++q)
            *(chunk*)(Bs + (b_r + q * B_RPP) * L::B_LD + b_c) = rb[q];
    };

    typename E::acc_t acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int r = 0; r < E::NACC; ++r) acc[i][j][r] = 0.f;

    auto compute = [&](int stage) {
        const elem* As = smem + stage * L::STAGE;
        const elem* Bs = As + L::A_SIZE;
#pragma unroll
        for (int kk = 0; kk < BK; kk += E::KG) {
            frag af[MI], bf[NI];
#pragma unroll
            for (int i = 0; i < MI; ++i) {
                if constexpr (AMODE == A_COL) {
#pragma unroll
                    for (int x = 0; x < E::NRJ; ++x) E::read_j(af[i], x, As, L::A_LD, kk, wm0 + i * BLK, lane, false);
                } else {
                    af[i] = *(const frag*)(As + (wm0 + i * BLK + li) * L::A_LD + kk + V * lk);
                }
            }
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
                for (int x = 0; x < E::NRJ; ++x) E::read_j(bf[j], x, Bs, L::B_LD, kk, wn0 + j * BLK, lane, false);
#pragma unroll
            for (int t = 0; t < E::TPG; ++t)
#pragma unroll
                for (int i = 0; i < MI; ++i)
#pragma unroll
                    for (int j = 0; j < NI; ++j) acc[i][j] = E::mfma(af[i], bf[j], acc[i][j], t);
        }
    };

    // ---- main loop: tile t+1 sits in registers and tile t+2 is in flight while step t is multiplied
    load_tiles(0);
    store_tiles(0);
    if (nk > 1) load_tiles(1);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        compute(kt & 1);
        if (kt + 1 < nk) store_tiles((kt & 1) ^ 1);
        if (kt + 2 < nk) load_tiles(kt + 2);
        __syncthreads();
    }

    OldC<T> oldc;
    finish_tile<T>(p, acc, C, slot, split, nsplit, m0, n0, wm0, wn0, interior, oldc);
}

// ---------------------------------------------------------------------------------------
// sched 4 / 5: operand tiles travel from global memory straight into LDS (no register
// staging, no LDS store instructions) through a ring of 3 / 4 stages, so the loads of two /
// three k steps are in flight while one step is multiplied: the form for launches whose few
// resident waves cannot hide the memory latency by themselves.
//
// One direct load moves 64 lanes x 16 bytes to 1 KiB of consecutive LDS, so a tile is kept
// as a plain array of 16-byte chunks in thread order, without row padding.  For k-contiguous
// rows the chunk stored at position c of row r is chunk c ^ swz(r) of that row, which spreads
// the 16-byte fragment reads of 16 consecutive rows over all banks; [k][j] tiles use the
// element type's own swizzle.  Either is applied to the global address on the way in and to
// the LDS address on the way out.
//
// Every lane of every direct load is active: a chunk that lies wholly outside its operand
// (remainder rows, k beyond K, a convolution tap in the zero padding) is fetched from a
// 16-byte block of zeros instead, so padding is still never read and the number of loads in
// flight is known exactly (the wait before a step counts them).  A chunk that straddles the
// end of a row cannot be fetched whole; the steps or tiles where that happens go through
// registers with masked accesses.
__device__ __attribute__((aligned(16))) unsigned g_zero_chunk[4] = {0u, 0u, 0u, 0u};

__device__ __forceinline__ void load_to_lds16(const void* g, unsigned lds_byte_base) {
    // M0 carries the wave's LDS destination; lane l lands at base + 16 * l.  Issued from
    // inline assembly: the compiler's own tracking of LDS DMA would wait for all of them
    // before every fragment read.
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
    // A tile is an array of chunks in thread order, a whole number of passes of the workgroup
    // over it.  A k-contiguous tile whose rows do not fill the last pass (112 or 208 rows) keeps
    // the pass whole: the chunks beyond the tile come from the block of zeros and are never read.
    static constexpr int CHUNKS_PER_PASS = T::NT;
    static constexpr int A_CHUNKS = (T::BM * T::BK / T::E::V + T::NT - 1) / T::NT * T::NT;
    static constexpr int B_CHUNKS = (T::BK * T::BN / T::E::V + T::NT - 1) / T::NT * T::NT;
    static constexpr int A_ELEMS = A_CHUNKS * T::E::V, B_ELEMS = B_CHUNKS * T::E::V, STAGE = A_ELEMS + B_ELEMS;
    static constexpr int BYTES = STAGES * STAGE * (int)sizeof(typename T::E::elem);
};

// Whether a tile shape exists for an address mode in the direct forms: an operand stored
// [k][j] needs rows of whole chunks that divide the workgroup's passes, and a k-contiguous one
// that does not fill its last pass is only handled for the left operand.
template <class T, int MODE>
constexpr bool direct_mode_ok() {
    constexpr int AMODE = MODE == A_ROW_BT ? A_ROW : MODE == A_COL_BT ? A_COL : MODE;
    constexpr bool B_KMAJ = MODE == A_ROW_BT || MODE == A_COL_BT, A_KMAJ = AMODE != A_COL;
    constexpr int V = T::E::V, NT = T::NT;
    constexpr int A_CPR = A_KMAJ ? T::BK / V : T::BM / V, A_ROWS = A_KMAJ ? T::BM : T::BK;
    constexpr int B_CPR = B_KMAJ ? T::BK / V : T::BN / V, B_ROWS = B_KMAJ ? T::BN : T::BK;
    if (NT % A_CPR || NT % B_CPR) return false;
    if (B_ROWS % (NT / B_CPR)) return false;
    if (A_ROWS % (NT / A_CPR) && !A_KMAJ) return false;
    if ((!B_KMAJ && B_CPR < 8) || (!A_KMAJ && A_CPR < 8)) return false;
    return true;
}

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
__global__ void __launch_bounds__(T::NT, T::MINW) gemm_direct_kernel(const KArgs p) {
    using E = typename T::E;
    using elem = typename E::elem;
    using chunk = typename E::chunk;
    using frag = typename E::frag;
    constexpr bool EDGE = EDGEV != 0, CUT = EDGEV == 1;
    // EDGEV 2: rows and columns past M or N are read from the last valid row or chunk instead of
    // being tested at every step: their products only reach elements of C that are never stored
    // (k past K still reads the block of zeros: both factors must vanish there)
    constexpr bool CLAMP = EDGEV == 2;
    // address mode of the left operand, and whether the right one is stored transposed (N x K)
    constexpr int AMODE = MODE == A_ROW_BT ? A_ROW : MODE == A_COL_BT ? A_COL : MODE;
    constexpr bool B_KMAJ = MODE == A_ROW_BT || MODE == A_COL_BT;
    constexpr int BM = T::BM, BN = T::BN, BK = T::BK, NT = T::NT, MI = T::MI, NI = T::NI;
    constexpr int V = E::V, BLK = E::BLK, LK = E::LK, ES = (int)sizeof(elem);
    using L = LdsDirect<T>;
    constexpr int STAGES = L::STAGES, D = STAGES - 1;
    constexpr bool A_KMAJ = AMODE != A_COL;
    constexpr int A_CPR = A_KMAJ ? BK / V : BM / V;   // 16-byte chunks per stored row of A
    constexpr int A_ROWS = A_KMAJ ? BM : BK;
    constexpr int A_RPP = NT / A_CPR, PA = (A_ROWS + A_RPP - 1) / A_RPP;
    constexpr bool A_RAGGED = A_ROWS % A_RPP != 0;    // the last pass runs past the tile's rows
    constexpr int B_CPR = B_KMAJ ? BK / V : BN / V;   // and of B
    constexpr int B_ROWS = B_KMAJ ? BN : BK;
    constexpr int B_RPP = NT / B_CPR, PB = B_ROWS / B_RPP;
    constexpr int LPT = PA + PB;                       // direct loads per thread and step
    static_assert(direct_mode_ok<T, MODE>(), "tile shape and address mode");
    static_assert(PA * NT * V == L::A_ELEMS && PB * NT * V == L::B_ELEMS, "LDS stage layout");
    static_assert((D - 1) * LPT <= 63, "outstanding-load counter range");
    constexpr int K_CPR = BK / V;   // chunks per row of a k-contiguous tile
    constexpr int SW_MOD = K_CPR < 16 ? K_CPR : 16, SW_DIV = 16 / SW_MOD;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    elem* smem = (elem*)smem_raw;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave / T::WAVES_N) * T::WM, wn0 = (wave % T::WAVES_N) * T::WN;
    const int li = lane & (BLK - 1), lk = lane / BLK;

    const int tiles = p.tiles_m * p.tiles_n;
    int tile, split, nsplit, slot;
    decode_block(p, tiles, tile, split, nsplit, slot);
    int tm, tn;
    tile_coords(p, tile, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;
    const elem* __restrict__ A = (const elem*)p.A + (long long)blockIdx.y * p.stride_a;
    const elem* __restrict__ B = (const elem*)p.B + (long long)blockIdx.y * p.stride_b;
    float* __restrict__ C = p.C + (long long)blockIdx.y * p.stride_c;

    const bool interior = !EDGE || (m0 + BM <= p.m_main && n0 + BN <= p.n_main);
    const int nk_all = (p.K + BK - 1) / BK;
    int kb, nk;
    k_range(nk_all, split, nsplit, kb, nk);

    // Leading steps of this workgroup whose chunks are all whole (inside or outside).
    // EDGEV 2 peels the k loop like Fig. 8: the ring runs the steps that lie wholly below K
    // without any test, and a last partial step is staged through registers after it.
    // A tile whose chunks are cut by the end of a row along N (row-major B) or M (transposed A)
    // still takes whole 16-byte loads in the ring: the bytes past the end of a row are the start
    // of the next row, and only feed columns / rows of C that are never stored.  The last row of
    // the operand has no next row, so for such a tile the last k step is always peeled.
    const bool cut_tile = CLAMP && ((!B_KMAJ && (p.N % V) && n0 + BN > p.N) || (AMODE == A_COL && (p.M % V) && m0 + BM > p.M));
    int nkp_ = CLAMP ? min(nk, max(0, p.k_full - kb)) : nk;
    if (cut_tile && kb + nk == nk_all) nkp_ = min(nkp_, nk - 1);
    const int nkp = nkp_;   // steps that go through the ring
    int n_direct = nkp;
    if constexpr (CUT) {
        bool whole_tile = !(!B_KMAJ && (p.N % V) && n0 + BN > p.N);             // rows of B are cut mid-chunk
        if (AMODE == A_COL && (p.M % V) && m0 + BM > p.M) whole_tile = false;   // so are rows of A^T
        if (!whole_tile) n_direct = 0;
        else if ((AMODE == A_ROW || B_KMAJ) && (p.K % V)) n_direct = max(0, min(nk, p.k_full - kb));
    }

    // The address of the block of zeros, taken once and kept in registers: derived where it is
    // used, it costs a scalar load and a wait for every outstanding LDS read in the middle of
    // the MFMA sequence of every step.
    const elem* zero_chunk = (const elem*)g_zero_chunk;
    asm volatile("" : "+s"(zero_chunk));

    // LDS byte address of this wave's 1 KiB slice of pass 0 of stage 0 (wave-uniform)
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) unsigned char*)smem_raw +
                          (unsigned)__builtin_amdgcn_readfirstlane(tid & ~63) * 16u;
    const int a_r = tid / A_CPR, a_cp = tid % A_CPR;
    const int b_r = tid / B_CPR, b_cp = tid % B_CPR;
    auto swz_k = [](int row) -> int { return (row / SW_DIV) % SW_MOD; };   // k-contiguous tiles

    // per-thread source of each of its chunks at k0 = 0
    const elem* a_src[PA];
    int a_k[PA];          // k offset of the chunk inside a step
    bool a_in[PA];        // the chunk's row (A_ROW: m, A_COL: m range) lies inside the operand
    int cv_base[PA], cv_hi0[PA], cv_wi0[PA];
    long long cv_off[PA];   // element offset of tap (0, 0), channel a_k of the chunk's pixel (may lie outside the tensor)
    int px_n = 0, px_ho = 0, px_wo = 0;
#pragma unroll
    for (int q = 0; q < PA; ++q) {
        const int row = a_r + q * A_RPP;
        // (rows of the last pass beyond the tile: nobody reads them, they come from the block of zeros)
        const bool pad_row = A_RAGGED && q == PA - 1 && row >= A_ROWS;
        if constexpr (AMODE == A_ROW) {
            a_k[q] = (a_cp ^ swz_k(row)) * V;
            a_in[q] = (!CUT || m0 + row < p.M) && !pad_row;
            a_src[q] = A + (long long)(CLAMP ? min(m0 + row, p.M - 1) : m0 + row) * p.lda + a_k[q];
        } else if constexpr (AMODE == A_COL) {
            a_k[q] = row;   // the stored row is the k index
            const int mc = (a_cp ^ E::swz_j(row)) * V;
            a_in[q] = !CUT || m0 + mc < p.M;
            a_src[q] = A + (long long)row * p.lda + (CLAMP && m0 + mc >= p.M ? max(p.M - V, 0) : m0 + mc);
        } else {
            a_k[q] = (a_cp ^ swz_k(row)) * V;
            const int m = m0 + row;
            a_in[q] = (!CUT || m < p.M) && !pad_row;
            a_src[q] = A;
            // The thread's first pixel is decoded with divisions (about forty four-cycle
            // instructions each); its other pixels lie A_RPP rows further on each and step from it.
            // A row past the last pixel reads as padding for every tap.
            if (q == 0) {
                const unsigned tq = (unsigned)m / (unsigned)p.Wo, nq = tq / (unsigned)p.Ho;
                px_wo = m - (int)tq * p.Wo;
                px_ho = (int)(tq - nq * (unsigned)p.Ho);
                px_n = (int)nq;
            } else {
                px_wo += A_RPP;
                while (px_wo >= p.Wo) {
                    px_wo -= p.Wo;
                    if (++px_ho == p.Ho) { px_ho = 0; ++px_n; }
                }
            }
            cv_base[q] = px_n * p.H;
            cv_hi0[q] = m < p.M ? px_ho * p.sh - p.ph : -(1 << 28);
            cv_wi0[q] = px_wo * p.sw - p.pw;
            cv_off[q] = ((long long)(cv_base[q] + cv_hi0[q]) * p.W + cv_wi0[q]) * p.Cin + a_k[q];
        }
    }
    // (kh, kw, ci) of the first k of the next step to issue, advanced step by step
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
    const elem* b_src[PB];
    int b_k[PB];          // k offset of the chunk inside a step: its row (B as K x N) or its swizzled chunk (N x K)
    bool b_in[PB];        // the chunk's n range lies inside the operand
#pragma unroll
    for (int q = 0; q < PB; ++q) {
        const int row = b_r + q * B_RPP;
        if constexpr (B_KMAJ) {
            b_k[q] = (b_cp ^ swz_k(row)) * V;
            b_in[q] = !CUT || n0 + row < p.N;
            b_src[q] = B + (long long)(CLAMP ? min(n0 + row, p.N - 1) : n0 + row) * p.ldb + b_k[q];
        } else {
            const int nc = (b_cp ^ E::swz_j(row)) * V;
            b_k[q] = row;
            b_in[q] = !CUT || n0 + nc < p.N;
            b_src[q] = B + (long long)row * p.ldb + (CLAMP && n0 + nc >= p.N ? max(p.N - V, 0) : n0 + nc);
        }
    }

    // ---- one direct load: the x-th of the LPT loads that bring a tile in
    // (`ktest`: also test the chunk's k against K, which the ring of the peeled variant never needs)
    auto load_one = [&](int kt, int stage, int x, bool ktest) {
        const int k0 = kt * BK;
        unsigned as = lds0 + (unsigned)(stage * L::STAGE * ES);
        // (the variant with the masked path in the ring runs out of scalar registers in the larger
        // tiles, and the compiler then keeps this wave-uniform address in a vector register)
        if constexpr (CUT) as = (unsigned)__builtin_amdgcn_readfirstlane((int)as);
        const unsigned bs = as + (unsigned)(L::A_ELEMS * ES);
        if (x < PA) {
            const int q = x;
            const elem* src;
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
                    const elem* inside = A + (cv_off[q] + cs_off);
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
            const elem* src = in ? b_src[q] + (B_KMAJ ? (long long)k0 : (long long)k0 * p.ldb) : zero_chunk;
            load_to_lds16(src, bs + (unsigned)(q * NT) * 16u);
        }
    };

    // ---- the same tile through registers with element masks (chunks cut by the end of a row)
    auto issue_masked = [&](int kt, int stage) {
        const int k0 = kt * BK;
        elem* As = smem + stage * L::STAGE;
        elem* Bs = As + L::A_ELEMS;
#pragma unroll
        for (int q = 0; q < PA; ++q) {
            const int row = a_r + q * A_RPP;
            chunk v = E::zero();
#pragma unroll
            for (int e = 0; e < V; ++e) {
                if constexpr (AMODE == A_ROW) {
                    const int m = m0 + row, k = k0 + a_k[q] + e;
                    if (m < p.M && k < p.K) v[e] = A[(long long)m * p.lda + k];
                } else if constexpr (AMODE == A_COL) {
                    const int k = k0 + row, m = m0 + (a_cp ^ E::swz_j(row)) * V + e;
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
            *(chunk*)(As + (q * NT + tid) * V) = v;
        }
#pragma unroll
        for (int q = 0; q < PB; ++q) {
            const int row = b_r + q * B_RPP;
            chunk v = E::zero();
#pragma unroll
            for (int e = 0; e < V; ++e) {
                if constexpr (B_KMAJ) {
                    const int n = n0 + row, k = k0 + b_k[q] + e;
                    if (n < p.N && k < p.K) v[e] = B[(long long)n * p.ldb + k];
                } else {
                    const int k = k0 + row, n = n0 + (b_cp ^ E::swz_j(row)) * V + e;
                    if (k < p.K && n < p.N) v[e] = B[(long long)k * p.ldb + n];
                }
            }
            *(chunk*)(Bs + (q * NT + tid) * V) = v;
        }
    };
    // the convolution's tap state moves on once per tile
    auto advance_tap = [&]() {
        if constexpr (AMODE == A_CONV) {
            cs_ci += BK;
            cs_off += BK;   // along ci and from one kw to the next the pixels' channels are consecutive
            while (cs_ci >= p.Cin) {
                cs_ci -= p.Cin;
                if (++cs_kw == p.KW) { cs_kw = 0; ++cs_kh; cs_off += (long long)(p.W - p.KW) * p.Cin; }
            }
        }
    };
    // the x-th part of bringing in tile kt_local: one direct load, or (steps with cut chunks)
    // the whole masked tile at x = 0
    auto issue_part = [&](int kt_local, int stage, int x) {
        if (!CUT || kt_local < n_direct) load_one(kb + kt_local, stage, x, false);
        else if (x == 0) issue_masked(kb + kt_local, stage);
        if (x == LPT - 1) advance_tap();
    };
    auto issue = [&](int kt_local, int stage) {
#pragma unroll
        for (int x = 0; x < LPT; ++x) issue_part(kt_local, stage, x);
    };

    typename E::acc_t acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int r = 0; r < E::NACC; ++r) acc[i][j][r] = 0.f;

    // fragment addressing of k-contiguous tiles: lane (li, lk) reads row w0 + BLK i + li, chunk
    // LK g + lk of k group g, swizzled by the row (w0 + BLK i is a multiple of 16, so the
    // swizzle depends on li alone)
    int a_row_off[MI];
#pragma unroll
    for (int i = 0; i < MI; ++i) a_row_off[i] = (wm0 + i * BLK + li) * BK;
    int b_row_off[NI];   // the same for a k-contiguous B, whose rows are columns of C
#pragma unroll
    for (int j = 0; j < NI; ++j) b_row_off[j] = (wn0 + j * BLK + li) * BK;
    const int k_x = lk ^ swz_k(li);

    // ---- fragments: a k group is fetched while the group before it is multiplied
    constexpr int G = BK / E::KG;
    static_assert(G == 1 || G % 2 == 0, "the fragment double buffer alternates per group across steps");
    constexpr int GP = G == 1 ? 1 : 0;   // with one group per step the buffers alternate per step
    constexpr int NFRAG = (A_KMAJ ? MI : E::NRJ * MI) + (B_KMAJ ? NI : E::NRJ * NI);   // LDS reads of one group's fragments
    constexpr int NM = E::TPG * MI * NI;                                                // MFMAs of one group
    frag af[2][MI], bf[2][NI];
    auto frag_read = [&](int buf, int stage, int g, int x) {
        const elem* As = smem + stage * L::STAGE;
        const elem* Bs = As + L::A_ELEMS;
        if constexpr (A_KMAJ) {
            if (x < MI) {
                af[buf][x] = *(const frag*)(As + a_row_off[x] + (((LK * g) ^ k_x) * V));
                return;
            }
            x -= MI;
        } else {
            if (x < E::NRJ * MI) {
                E::read_j(af[buf][x / E::NRJ], x % E::NRJ, As, BM, g * E::KG, wm0 + (x / E::NRJ) * BLK, lane, true);
                return;
            }
            x -= E::NRJ * MI;
        }
        if constexpr (B_KMAJ) bf[buf][x] = *(const frag*)(Bs + b_row_off[x] + (((LK * g) ^ k_x) * V));
        else E::read_j(bf[buf][x / E::NRJ], x % E::NRJ, Bs, BN, g * E::KG, wn0 + (x / E::NRJ) * BLK, lane, true);
    };

    // ---- ring.  Step kt is multiplied from stage kt % STAGES.  The one barrier of a step sits
    // before its LAST k group: by then tile kt+1 has landed (own loads: the wait; everybody's:
    // the barrier) and everybody has left step kt-1, so during that last group the loads of
    // tile kt+D go into the stage step kt-1 used and the first fragments of step kt+1 are
    // fetched.  No wave ever starts a step, or leaves a barrier, with its MFMA operands missing.
    // (the old values of C, for small tiles: ordinary loads, older than every load of the ring, so
    // the ring's counted waits only become stricter until they have landed)
    OldC<T> oldc;
    oldc.fetch(p, C, m0, n0, wm0, wn0, interior, nsplit);
    for (int t = 0; t < D; ++t)
        if (t < nkp) issue(t, t);
    if (D <= n_direct) wait_loads_outstanding<(D - 1) * LPT>();
    else wait_loads_outstanding<0>();
    __syncthreads();
#pragma unroll
    for (int x = 0; x < NFRAG; ++x) frag_read(0, 0, 0, x);
    int cur = 0;
    auto step = [&](auto parity_tag, auto loads_tag, int kt) {
        // PAR: which fragment buffer group 0 of this step uses (only alternates per step when a
        // step is a single group).  LOADS: 0 = every load of tile kt+D is guarded by a test that the
        // tile exists; 1 = the caller knows it exists (no test); 2 = the caller knows it does not
        // (no loads).  Small tiles run their steps as 1 then 2: a test beside each load cut the
        // step's scheduling region at every one (1-2 % of the layer and of 1024^3); the large
        // tiles keep the tests, where the split cost 13 %.
        constexpr int PAR = decltype(parity_tag)::value;
        constexpr int LOADS = decltype(loads_tag)::value;
        const int nxt = cur + 1 == STAGES ? 0 : cur + 1;
        const int fill = cur == 0 ? STAGES - 1 : cur - 1;
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const bool last = g == G - 1;
            const int buf = (g + PAR) & 1;
            if (last) {
                // issued so far: tiles up to kt+D-1, so D-2 tiles may stay in flight behind tile kt+1
                if (D >= 3 && kt + D <= n_direct) wait_loads_outstanding<(D >= 3 ? (D - 2) * LPT : 0)>();
                else wait_loads_outstanding<0>();
                __syncthreads();
            }
            // Behind the MFMAs of this group: first the fragments of the next one, all of them within
            // the first quarter of the group (a wave that is alone on its SIMD has nobody to hide an
            // LDS wait behind), then, in a step's last group, the loads of tile kt+D.  Where the reads
            // fall among the MFMAs moves a kernel by up to 13 %, and not monotonically: the quarter is
            // the best of the spreads measured (all behind the first MFMA, an eighth, a quarter, a half,
            // the whole group) for every fp32 tile; the four-stage bf16 tiles, whose group is 8 or 16
            // long MFMAs, do 2 % better with the reads over the first half.
            constexpr int FDIV = (E::TPG == 1 && T::SCHED == 5) ? 2 : 4;
            constexpr int FQ = NM / FDIV > 0 ? NM / FDIV : 1;
            constexpr int FPER = (NFRAG + FQ - 1) / FQ;      // fragment reads behind one MFMA
            constexpr int FM = (NFRAG + FPER - 1) / FPER;    // MFMAs that carry them
            constexpr int LM = NM - FM > 0 ? NM - FM : 1;    // MFMAs that carry loads: the rest, or the last one
            constexpr int L0 = NM - LM;
            constexpr int LPER = (LPT + LM - 1) / LM;
#pragma unroll
            for (int m = 0; m < NM; ++m) {
                const int t = m / (MI * NI), i = (m / NI) % MI, j = m % NI;
                acc[i][j] = E::mfma(af[buf][i], bf[buf][j], acc[i][j], t);
                if (m < FM) {
#pragma unroll
                    for (int u = 0; u < FPER; ++u) {
                        const int e = m * FPER + u;
                        if (e >= NFRAG) continue;
                        if (last) frag_read(buf ^ 1, nxt, 0, e);   // after the last step this reads a stage nobody multiplies
                        else frag_read(buf ^ 1, cur, g + 1, e);
                    }
                }
                if (LOADS != 2 && last && m >= L0) {
#pragma unroll
                    for (int u = 0; u < LPER; ++u) {
                        const int e = (m - L0) * LPER + u;
                        if (e >= LPT) continue;
                        if (LOADS == 1 || kt + D < nkp) issue_part(kt + D, fill, e);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        cur = nxt;
    };
    {
        using P0 = std::integral_constant<int, 0>;
        using P1 = std::integral_constant<int, 1>;
        using Guarded = std::integral_constant<int, 0>;
        using Live = std::integral_constant<int, 1>;
        using Dead = std::integral_constant<int, 2>;
        constexpr bool SMALL = MI * NI * E::NACC <= 32;
        if constexpr (!SMALL) {
            if constexpr (GP == 0) {
                for (int kt = 0; kt < nkp; ++kt) step(P0{}, Guarded{}, kt);
            } else {
                int kt = 0;
                for (; kt + 1 < nkp; kt += 2) {
                    step(P0{}, Guarded{}, kt);
                    step(P1{}, Guarded{}, kt + 1);
                }
                if (kt < nkp) step(P0{}, Guarded{}, kt);
            }
        } else {
            const int n_live = max(0, nkp - D);   // steps kt with a tile kt+D to bring in
            int kt = 0;
            if constexpr (GP == 0) {
                for (; kt < n_live; ++kt) step(P0{}, Live{}, kt);
                for (; kt < nkp; ++kt) step(P0{}, Dead{}, kt);
            } else {
                for (; kt < n_live; ++kt) {
                    if (kt & 1) step(P1{}, Live{}, kt);
                    else step(P0{}, Live{}, kt);
                }
                for (; kt < nkp; ++kt) {
                    if (kt & 1) step(P1{}, Dead{}, kt);
                    else step(P0{}, Dead{}, kt);
                }
            }
        }
    }

    if constexpr (CLAMP) {
        if (nkp < nk) {
            // the partial last step into stage 0, multiplied group by group: chunks past K come
            // from the block of zeros, or, when K cuts a chunk of a k-contiguous operand or the
            // tile's chunks are cut along M or N, the whole tile goes through registers with
            // element masks
            __syncthreads();   // everybody has left the ring
            if ((p.K % V) || cut_tile) {
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
                for (int x = 0; x < NFRAG; ++x) frag_read(0, 0, g, x);
#pragma unroll
                for (int m = 0; m < NM; ++m) {
                    const int t = m / (MI * NI), i = (m / NI) % MI, j = m % NI;
                    acc[i][j] = E::mfma(af[0][i], bf[0][j], acc[i][j], t);
                }
            }
        }
    }
    finish_tile<T>(p, acc, C, slot, split, nsplit, m0, n0, wm0, wn0, interior, oldc);
}

template <class T, int AMODE>
hipError_t launch_mode(int variant, const KArgs& a, int batch, hipStream_t s) {
    using E = typename T::E;
    const dim3 grid(a.split_first + (a.tiles_m * a.tiles_n - a.split_first) * a.split_k, batch, 1), block(T::NT, 1, 1);
    void (*fn)(const KArgs) = nullptr;
    int bytes = 0, one_tap = 0;
    if constexpr (T::SCHED == 1) {
        if constexpr (AMODE == A_CONV) {
            return hipErrorInvalidValue;   // the block form takes matrices only
        } else {
            if (a.split_k != 1) return hipErrorInvalidValue;   // k is split inside the workgroup only
            fn = variant == 0 ? gemm_block_kernel<T, AMODE, 0>
                 : variant == 2 ? gemm_block_kernel<T, AMODE, 2> : gemm_block_kernel<T, AMODE, 1>;
            hipLaunchKernelGGL(fn, grid, block, 0, s, a);
            (void)one_tap;
            return hipGetLastError();
        }
    } else if constexpr (T::SCHED >= 4 && !direct_mode_ok<T, AMODE>()) {
        return hipErrorInvalidValue;   // this tile shape does not exist for this operand layout
    } else if constexpr (T::SCHED >= 4) {
        // the direct-to-LDS forms move whole 16-byte chunks only
        if (variant == 2) return hipErrorInvalidValue;
        bytes = LdsDirect<T>::BYTES;
        fn = variant == 0 ? gemm_direct_kernel<T, AMODE, 0>
             : variant == 3 ? gemm_direct_kernel<T, AMODE, 2> : gemm_direct_kernel<T, AMODE, 1>;
        if constexpr (AMODE == A_CONV) {
            if (a.Cin % T::BK == 0) {
                one_tap = 1;
                fn = variant == 0 ? gemm_direct_kernel<T, AMODE, 0, true>
                     : variant == 3 ? gemm_direct_kernel<T, AMODE, 2, true> : gemm_direct_kernel<T, AMODE, 1, true>;
            }
        }
    } else if constexpr (AMODE == A_ROW_BT || AMODE == A_COL_BT || !E::kHasGeneral) {
        return hipErrorInvalidValue;   // a transposed right operand exists in the direct-to-LDS forms only
    } else {
        bytes = Lds<T, AMODE>::BYTES;
        switch (variant) {
            case 0: fn = gemm_staged_kernel<T, AMODE, E::V, false>; break;
            case 1:
            case 3: fn = gemm_staged_kernel<T, AMODE, E::V, true>; break;
            default: fn = gemm_staged_kernel<T, AMODE, 1, true>; break;
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

// bit m set: the tile exists for address mode m
template <class T>
constexpr int mode_mask_of() {
    if constexpr (T::SCHED == 1)
        return (1 << A_ROW) | (1 << A_COL) | (1 << A_ROW_BT) | (1 << A_COL_BT);
    else if constexpr (T::SCHED >= 4)
        return (direct_mode_ok<T, A_ROW>() << A_ROW) | (direct_mode_ok<T, A_COL>() << A_COL) |
               (direct_mode_ok<T, A_CONV>() << A_CONV) | (direct_mode_ok<T, A_ROW_BT>() << A_ROW_BT) |
               (direct_mode_ok<T, A_COL_BT>() << A_COL_BT);
    else
        return T::E::kHasGeneral ? (1 << A_ROW) | (1 << A_COL) | (1 << A_CONV) : 0;
}

template <class T>
constexpr int lds_bytes_of() {
    if constexpr (T::SCHED == 1) return 3 * T::E::NACC * 64 * 4;
    else if constexpr (T::SCHED >= 4) return LdsDirect<T>::BYTES;
    else return Lds<T, A_ROW>::BYTES;
}

}  // namespace
}  // namespace tsg

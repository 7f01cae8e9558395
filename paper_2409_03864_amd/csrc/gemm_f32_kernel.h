// fp32 contraction kernels for gfx950: C = +-op(A).B (+C), fp32 MFMA accumulate.
//
// One workgroup computes a BM x BN tile of C (the i/j tiling of Case Study 4, Fig. 8);
// the k loop advances in BK steps with the operand tiles of step t+1 fetched from
// global memory into registers while step t is consumed from LDS (two LDS stages,
// one barrier per step).  Each wavefront owns a WM x WN sub-tile built from 32x32
// MFMA blocks: the fixed-size inner matmul that the paper hands to a microkernel
// library is here the v_mfma_f32_32x32x2_f32 sequence.
//
// The rewrites of Case Study 3 live in the address generators only:
//   A_ROW  : op(A)(i,k) = A[i*lda + k]
//   A_COL  : op(A)(i,k) = A[k*lda + i]        transposed operand, read in place
//   A_CONV : op(A)(m,k) = x[n][ho*sh+kh-ph][wo*sw+kw-pw][ci], k = (kh*KW+kw)*Cin+ci,
//            and 0 WITHOUT a memory access where the coordinate is in the padding
// The main/remainder split of Fig. 8 is taken per tile: tiles inside
// [0,m_main) x [0,n_main) and k steps below k_full run the unmasked loaders, the
// remainder runs masked ones (zero fill), chosen by a wavefront-uniform branch.
//
// Split k: with split_k = S > 1, S workgroups share one tile of C, each taking a contiguous
// range of k steps.  Each parks its partial tile in the workspace and bumps the tile's
// arrival counter; the workgroup that arrives last adds the S partials in split order (so
// the sum does not depend on who was last), applies the epilogue and resets the counter.
#pragma once
#include <atomic>
#include <type_traits>

#include "tsg_internal.h"

namespace tsg {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
// 16-byte global access that only promises element alignment: rows of an operand with an
// odd leading dimension start on any 4-byte boundary, and the hardware fetches such a chunk
// with one instruction all the same
typedef f32x4 f32x4_u __attribute__((aligned(4)));

constexpr unsigned FLAG_NEGATE = 1u, FLAG_ACCUMULATE = 2u;
constexpr int kXcds = 8;      // workgroup ids are dealt round-robin over this many L2 domains
constexpr int kGroupM = 8;    // tile rows per raster group

// SCHED selects the shape of the inner loop, a tunable like the tile sizes:
//   0  fragments are read from LDS group by group where they are used; the instruction
//      order inside a k step is left to the compiler
//   1  fragments of k group g+1 are read while the MFMAs of group g run and the next tile
//      is written to LDS half way through the step, both pinned by scheduling barriers
//   2  as 1 but one MFMA k pair ahead instead of one group of four: every wave always has
//      the operands of its next MFMAs in registers, so waves that the issue arbiter has
//      put in lock step never wait for LDS together
//   3  as 2 with THREE LDS stages: the one barrier of a step sits in its middle, right after
//      the next tile has been parked, and the first operands of the next step are fetched
//      before the current step ends, so no wave drains its MFMA queue around the barrier
template <int BM_, int BN_, int BK_, int WM_, int WN_, int MINW_, int SCHED_>
struct Tile {
    static constexpr int BM = BM_, BN = BN_, BK = BK_, WM = WM_, WN = WN_, MINW = MINW_, SCHED = SCHED_;
    static constexpr int WAVES_M = BM / WM, WAVES_N = BN / WN;
    static constexpr int NT = 64 * WAVES_M * WAVES_N;
    static constexpr int MI = WM / 32, NI = WN / 32;
    static_assert(BM % WM == 0 && BN % WN == 0 && WM % 32 == 0 && WN % 32 == 0 && BK % 8 == 0, "tile");
};

template <class T, int AMODE>
struct Lds {
    // k-contiguous A rows are padded by 4 floats so that the 16-byte fragment reads of
    // 16 consecutive rows fall in distinct banks; i/j-contiguous tiles are padded by 8 so
    // the two half-waves (k and k+4) read different bank halves.
    static constexpr int A_LD = (AMODE == A_COL) ? T::BM + 8 : T::BK + 4;
    static constexpr int A_ROWS = (AMODE == A_COL) ? T::BK : T::BM;
    static constexpr int B_LD = T::BN + 8;
    static constexpr int A_SIZE = A_ROWS * A_LD, B_SIZE = T::BK * B_LD;
    static constexpr int STAGE = A_SIZE + B_SIZE;
    static constexpr int STAGES = T::SCHED == 3 ? 3 : 2;
    static constexpr int BYTES = STAGES * STAGE * (int)sizeof(float);
};

__device__ __forceinline__ void tile_coords(const KArgs& p, int bid, int& tm, int& tn) {
    int id = bid;
    if (p.raster) {
        // Give each XCD a contiguous range of tile ids, then walk the range in groups of
        // kGroupM tile rows so that concurrently resident tiles share A and B panels in
        // that XCD's L2.
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
    tm = (int)((unsigned)id / (unsigned)p.tiles_n);
    tn = id - tm * p.tiles_n;
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

// What follows the k loop.  Split k: park the partial tile, count the arrival, and let the
// last arrival add the partials in split order.  Epilogue: sign, optional accumulate, masked
// at the remainder.
template <class T>
__device__ __forceinline__ void finish_tile(const KArgs& p, f32x16 (&acc)[T::MI][T::NI], float* __restrict__ C,
                                            int slot, int split, int nsplit, int m0, int n0, int wm0, int wn0,
                                            bool interior) {
    constexpr int BM = T::BM, BN = T::BN, NT = T::NT, MI = T::MI, NI = T::NI;
    const int tid = threadIdx.x, lane = tid & 63, li = lane & 31, lh = lane >> 5;
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
__global__ void __launch_bounds__(T::NT, T::MINW) gemm_f32_kernel(const KArgs p) {
    constexpr int BM = T::BM, BN = T::BN, BK = T::BK, NT = T::NT, MI = T::MI, NI = T::NI;
    using L = Lds<T, AMODE>;
    extern __shared__ __attribute__((aligned(16))) float smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave / T::WAVES_N) * T::WM, wn0 = (wave % T::WAVES_N) * T::WN;
    const int li = lane & 31, lh = lane >> 5;

    const int tiles = p.tiles_m * p.tiles_n;
    int tile, split, nsplit, slot;
    decode_block(p, tiles, tile, split, nsplit, slot);
    int tm, tn;
    tile_coords(p, tile, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;
    const float* __restrict__ A = (const float*)p.A + (long long)blockIdx.y * p.stride_a;
    const float* __restrict__ B = (const float*)p.B + (long long)blockIdx.y * p.stride_b;
    float* __restrict__ C = p.C + (long long)blockIdx.y * p.stride_c;

    // Remainder tiles (Fig. 8's %rest) take the masked loaders for every k step.
    const bool interior = !EDGE || (m0 + BM <= p.m_main && n0 + BN <= p.n_main);
    // this workgroup's k steps: [kb, kb + nk) of the (K + BK - 1) / BK steps of the whole loop
    const int nk_all = (p.K + BK - 1) / BK;
    // (unsigned 32-bit: nk_all < 2^27 and nsplit <= 16; an unsplit tile divides nothing)
    int kb = 0, nk = nk_all;
    if (nsplit > 1) {
        kb = (int)((unsigned)(nk_all * split) / (unsigned)nsplit);
        nk = (int)((unsigned)(nk_all * (split + 1)) / (unsigned)nsplit) - kb;
    }

    // ---- per-thread global->LDS assignment: 4-element chunks along the contiguous dim
    constexpr int A_CPR = (AMODE == A_COL) ? BM / 4 : BK / 4;   // chunks per stored row
    constexpr int A_RPP = NT / A_CPR;                            // rows per pass
    constexpr int A_ROWS = L::A_ROWS;
    constexpr int PA = A_ROWS / A_RPP;
    constexpr int B_CPR = BN / 4, B_RPP = NT / B_CPR, PB = BK / B_RPP;
    static_assert(NT % A_CPR == 0 && A_ROWS % A_RPP == 0 && PA >= 1, "A staging shape");
    static_assert(NT % B_CPR == 0 && BK % B_RPP == 0 && PB >= 1, "B staging shape");
    const int a_r = tid / A_CPR, a_c = (tid % A_CPR) * 4;
    const int b_r = tid / B_CPR, b_c = (tid % B_CPR) * 4;

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

    f32x4 ra[PA], rb[PB];

    // One element of op(A) for the scalar path (row/col relative to the problem).
    auto a_elem = [&](int q, int row_or_k, int e) -> float {
        if constexpr (AMODE == A_ROW) {
            const int m = m0 + row_or_k, k = e;
            return (m < p.M && k < p.K) ? A[(long long)m * p.lda + k] : 0.f;
        } else if constexpr (AMODE == A_COL) {
            const int k = row_or_k, m = e;
            return (k < p.K && m < p.M) ? A[(long long)k * p.lda + m] : 0.f;
        } else {
            const int k = e;
            if (k >= p.K) return 0.f;
            const int tap = k / p.Cin, ci = k - tap * p.Cin;
            const int kh = tap / p.KW, kw = tap - kh * p.KW;
            const int hi = cv_hi0[q] + kh, wi = cv_wi0[q] + kw;
            if (hi < 0 || hi >= p.H || wi < 0 || wi >= p.W) return 0.f;
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
                if (VEC == 4 && (fast || (m0 + r < p.M && k + 4 <= p.K))) {
                    ra[q] = *(const f32x4_u*)(A + (long long)(m0 + r) * p.lda + k);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) ra[q][e] = a_elem(q, r, k + e);
                }
            } else if constexpr (AMODE == A_COL) {
                const int k = k0 + r, m = m0 + a_c;
                if (VEC == 4 && (fast || (k < p.K && m + 4 <= p.M))) {
                    ra[q] = *(const f32x4_u*)(A + (long long)k * p.lda + m);
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) ra[q][e] = a_elem(q, k, m + e);
                }
            } else {
                const int k = k0 + a_c;
                if constexpr (VEC == 4) {
                    // Cin % 4 == 0: the chunk lies inside one tap
                    f32x4 v = {0.f, 0.f, 0.f, 0.f};
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
                            v = *(const f32x4_u*)(A + ((long long)(cv_base[q] + hi) * p.W + wi) * p.Cin + ci);
                    }
                    ra[q] = v;
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e) ra[q][e] = a_elem(q, r, k + e);
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
            if (VEC == 4 && (fast || (k < p.K && n + 4 <= p.N))) {
                rb[q] = *(const f32x4_u*)(B + (long long)k * p.ldb + n);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    rb[q][e] = (k < p.K && n + e < p.N) ? B[(long long)k * p.ldb + n + e] : 0.f;
            }
        }
    };

    auto store_tiles = [&](int stage) {
        float* As = smem + stage * L::STAGE;
        float* Bs = As + L::A_SIZE;
#pragma unroll
        for (int q = 0; q < PA; ++q)
            *(f32x4*)(As + (a_r + q * A_RPP) * L::A_LD + a_c) = ra[q];
#pragma unroll
        for (int q = 0; q < PB; ++q)
            *(f32x4*)(Bs + (b_r + q * B_RPP) * L::B_LD + b_c) = rb[q];
    };

    f32x16 acc[MI][NI];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // The k values of an 8-wide group are consumed in the order (t, t+4), t = 0..3: lanes
    // 0-31 feed k = t and lanes 32-63 feed k = t+4 of MFMA number t.  Any order is legal as
    // long as both operands use it, and this one lets a k-contiguous A row be fetched with
    // a single 16-byte LDS read.
    auto load_frags = [&](const float* As, const float* Bs, int kk, f32x4 (&af)[MI], f32x4 (&bf)[NI]) {
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            if constexpr (AMODE == A_COL) {
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    af[i][t] = As[(kk + 4 * lh + t) * L::A_LD + wm0 + i * 32 + li];
            } else {
                af[i] = *(const f32x4*)(As + (wm0 + i * 32 + li) * L::A_LD + kk + 4 * lh);
            }
        }
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int t = 0; t < 4; ++t)
                bf[j][t] = Bs[(kk + 4 * lh + t) * L::B_LD + wn0 + j * 32 + li];
    };

    // Fragments of k group g+1 are fetched from LDS while the MFMAs of group g run; the
    // next tile (already in registers) is written to the other LDS stage half way through,
    // so that neither LDS latency is exposed at the barrier.  The scheduling barriers keep
    // the compiler from sinking the reads back to their first use.
    auto compute = [&](int stage, int kt) {
        const float* As = smem + stage * L::STAGE;
        const float* Bs = As + L::A_SIZE;
        constexpr int G = BK / 8;
        f32x4 af[2][MI], bf[2][NI];
        load_frags(As, Bs, 0, af[0], bf[0]);
#pragma unroll
        for (int g = 0; g < G; ++g) {
            if (g + 1 < G) load_frags(As, Bs, (g + 1) * 8, af[(g + 1) & 1], bf[(g + 1) & 1]);
            if (g == G / 2) {
                // tile kt+1 has had a whole step to arrive: park it in the other stage, then
                // reuse the same registers for the loads of tile kt+2
                if (kt + 1 < nk) store_tiles(stage ^ 1);
                if (kt + 2 < nk) load_tiles(kt + 2);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int i = 0; i < MI; ++i)
#pragma unroll
                    for (int j = 0; j < NI; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[g & 1][i][t], bf[g & 1][j][t], acc[i][j], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // SCHED 2: operands are fetched one k pair (= one MFMA per block) ahead.
    auto compute_fine = [&](int stage, int kt) {
        const float* As = smem + stage * L::STAGE;
        const float* Bs = As + L::A_SIZE;
        constexpr int G = BK / 8, S = 4 * G;
        f32x4 ag[2][MI];   // k-contiguous A: one 16-byte read per group of four k pairs
        float av[2][MI];   // i-contiguous A: one value per k pair
        float bv[2][NI];
        auto fetch = [&](int s1) {
            const int g1 = s1 >> 2, t1 = s1 & 3;
            const int krow = g1 * 8 + 4 * lh + t1;
            if constexpr (AMODE == A_COL) {
#pragma unroll
                for (int i = 0; i < MI; ++i) av[s1 & 1][i] = As[krow * L::A_LD + wm0 + i * 32 + li];
            } else {
                if (t1 == 0) {
#pragma unroll
                    for (int i = 0; i < MI; ++i)
                        ag[g1 & 1][i] = *(const f32x4*)(As + (wm0 + i * 32 + li) * L::A_LD + g1 * 8 + 4 * lh);
                }
            }
#pragma unroll
            for (int j = 0; j < NI; ++j) bv[s1 & 1][j] = Bs[krow * L::B_LD + wn0 + j * 32 + li];
        };
        fetch(0);
#pragma unroll
        for (int s = 0; s < S; ++s) {
            if (s + 1 < S) fetch(s + 1);
            if (s == S / 2) {
                if (kt + 1 < nk) store_tiles(stage ^ 1);
                if (kt + 2 < nk) load_tiles(kt + 2);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NI; ++j) {
                    const float a = (AMODE == A_COL) ? av[s & 1][i] : ag[(s >> 2) & 1][i][s & 3];
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, bv[s & 1][j], acc[i][j], 0, 0, 0);
                }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // SCHED 3.  Step kt multiplies stage kt % 3.  Tile kt+1 is written to stage (kt+1) % 3 a
    // quarter of the way in; that stage was last read in step kt-2, which every wave left
    // before it passed the barrier of step kt-1.  The barrier of step kt follows the write,
    // and the operands of step kt+1 are read from the new stage only after it.
    auto run_three_stage = [&]() {
        constexpr int G = BK / 8, S = 4 * G;
        static_assert(G % 2 == 0, "operand double buffers alternate per group across steps");
        f32x4 ag[2][MI];
        float av[2][MI];
        float bv[2][NI];
        auto fetch = [&](int stage, int s1) {
            const float* As = smem + stage * L::STAGE;
            const float* Bs = As + L::A_SIZE;
            const int g1 = s1 >> 2, t1 = s1 & 3;
            const int krow = g1 * 8 + 4 * lh + t1;
            if constexpr (AMODE == A_COL) {
#pragma unroll
                for (int i = 0; i < MI; ++i) av[s1 & 1][i] = As[krow * L::A_LD + wm0 + i * 32 + li];
            } else {
                if (t1 == 0) {
#pragma unroll
                    for (int i = 0; i < MI; ++i)
                        ag[g1 & 1][i] = *(const f32x4*)(As + (wm0 + i * 32 + li) * L::A_LD + g1 * 8 + 4 * lh);
                }
            }
#pragma unroll
            for (int j = 0; j < NI; ++j) bv[s1 & 1][j] = Bs[krow * L::B_LD + wn0 + j * 32 + li];
        };
        fetch(0, 0);
        int cur = 0;
        for (int kt = 0; kt < nk; ++kt) {
            const int nxt = cur == 2 ? 0 : cur + 1;
#pragma unroll
            for (int s = 0; s < S; ++s) {
                // after the last step the fetch reads a stage nobody multiplies: harmless, and
                // keeping it unconditional keeps the whole step one scheduling region
                fetch(s + 1 < S ? cur : nxt, s + 1 < S ? s + 1 : 0);
                if (s == S / 4) {
                    if (kt + 1 < nk) store_tiles(nxt);
                    if (kt + 2 < nk) load_tiles(kt + 2);
                }
                if (s == S / 2) __syncthreads();
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int i = 0; i < MI; ++i)
#pragma unroll
                    for (int j = 0; j < NI; ++j) {
                        const float a = (AMODE == A_COL) ? av[s & 1][i] : ag[(s >> 2) & 1][i][s & 3];
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a, bv[s & 1][j], acc[i][j], 0, 0, 0);
                    }
                __builtin_amdgcn_sched_barrier(0);
            }
            cur = nxt;
        }
    };

    // SCHED 0: the plain form of the same step
    auto compute_plain = [&](int stage) {
        const float* As = smem + stage * L::STAGE;
        const float* Bs = As + L::A_SIZE;
#pragma unroll
        for (int kk = 0; kk < BK; kk += 8) {
            f32x4 af[MI], bf[NI];
            load_frags(As, Bs, kk, af, bf);
#pragma unroll
            for (int t = 0; t < 4; ++t)
#pragma unroll
                for (int i = 0; i < MI; ++i)
#pragma unroll
                    for (int j = 0; j < NI; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[i][t], bf[j][t], acc[i][j], 0, 0, 0);
        }
    };

    // ---- main loop: tile t+1 sits in registers and tile t+2 is in flight while step t is multiplied
    load_tiles(0);
    store_tiles(0);
    if (nk > 1) load_tiles(1);
    __syncthreads();
    if constexpr (T::SCHED == 3) run_three_stage();
    for (int kt = 0; T::SCHED != 3 && kt < nk; ++kt) {
        if constexpr (T::SCHED == 2) {
            compute_fine(kt & 1, kt);
        } else if constexpr (T::SCHED == 1) {
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
// SCHED 4 / 5: operand tiles travel from global memory straight into LDS (no register
// staging, no LDS store instructions) through a ring of 3 / 4 stages, so the loads of two /
// three k steps are in flight while one step is multiplied: the form for launches whose few
// resident waves cannot hide the memory latency by themselves.
//
// One direct load moves 64 lanes x 16 bytes to 1 KiB of consecutive LDS, so a tile is kept
// as a plain array of 16-byte chunks in thread order, without row padding.  For k-contiguous
// rows the chunk stored at position c of row r is chunk c ^ swz(r) of that row, which spreads
// the 16-byte fragment reads of 16 consecutive rows over all banks; the swizzle is applied
// to the global address on the way in and to the LDS address on the way out.
//
// Every lane of every direct load is active: a chunk that lies wholly outside its operand
// (remainder rows, k beyond K, a convolution tap in the zero padding) is fetched from a
// 16-byte block of zeros instead, so padding is still never read and the number of loads in
// flight is known exactly (the wait before a step counts them).  A chunk that straddles the
// end of a row cannot be fetched whole; the steps or tiles where that happens go through
// registers with masked accesses, as in the other forms.
__device__ __attribute__((aligned(16))) float g_zero_chunk[4] = {0.f, 0.f, 0.f, 0.f};

__device__ __forceinline__ void load_to_lds16(const void* g, unsigned lds_byte_base) {
    // M0 carries the wave's LDS destination; lane l lands at base + 16 * l
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(lds_byte_base)
                 : "memory", "m0");
}
template <int N>
__device__ __forceinline__ void wait_loads_outstanding() {
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

template <class T, int AMODE>
struct LdsDirect {
    static constexpr int STAGES = T::SCHED == 5 ? 4 : 3;
    static constexpr int A_FLOATS = T::BM * T::BK, B_FLOATS = T::BK * T::BN, STAGE = A_FLOATS + B_FLOATS;
    static constexpr int BYTES = STAGES * STAGE * (int)sizeof(float);
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
__global__ void __launch_bounds__(T::NT, T::MINW) gemm_f32_direct_kernel(const KArgs p) {
    constexpr bool EDGE = EDGEV != 0, CUT = EDGEV == 1;
    // EDGEV 2: rows and columns past M or N are read from the last valid row or chunk instead of
    // being tested at every step: their products only reach elements of C that are never stored
    // (k past K still reads the block of zeros: both factors must vanish there)
    constexpr bool CLAMP = EDGEV == 2;
    // address mode of the left operand, and whether the right one is stored transposed (N x K)
    constexpr int AMODE = MODE == A_ROW_BT ? A_ROW : MODE == A_COL_BT ? A_COL : MODE;
    constexpr bool B_KMAJ = MODE == A_ROW_BT || MODE == A_COL_BT;
    constexpr int BM = T::BM, BN = T::BN, BK = T::BK, NT = T::NT, MI = T::MI, NI = T::NI;
    using L = LdsDirect<T, AMODE>;
    constexpr int STAGES = L::STAGES, D = STAGES - 1;
    constexpr bool A_KMAJ = AMODE != A_COL;
    constexpr int A_CPR = A_KMAJ ? BK / 4 : BM / 4;   // 16-byte chunks per stored row of A
    constexpr int A_ROWS = A_KMAJ ? BM : BK;
    constexpr int A_RPP = NT / A_CPR, PA = A_ROWS / A_RPP;
    constexpr int B_CPR = B_KMAJ ? BK / 4 : BN / 4;   // and of B
    constexpr int B_ROWS = B_KMAJ ? BN : BK;
    constexpr int B_RPP = NT / B_CPR, PB = B_ROWS / B_RPP;
    constexpr int LPT = PA + PB;                       // direct loads per thread and step
    static_assert(NT % A_CPR == 0 && A_ROWS % A_RPP == 0 && PA >= 1, "A staging shape");
    static_assert(NT % B_CPR == 0 && B_ROWS % B_RPP == 0 && PB >= 1, "B staging shape");
    static_assert((D - 1) * LPT <= 63, "outstanding-load counter range");
    constexpr int K_CPR = BK / 4;   // chunks per row of a k-contiguous tile
    constexpr int SW_MOD = K_CPR < 16 ? K_CPR : 16, SW_DIV = 16 / SW_MOD;
    extern __shared__ __attribute__((aligned(16))) float smem[];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm0 = (wave / T::WAVES_N) * T::WM, wn0 = (wave % T::WAVES_N) * T::WN;
    const int li = lane & 31, lh = lane >> 5;

    const int tiles = p.tiles_m * p.tiles_n;
    int tile, split, nsplit, slot;
    decode_block(p, tiles, tile, split, nsplit, slot);
    int tm, tn;
    tile_coords(p, tile, tm, tn);
    const int m0 = tm * BM, n0 = tn * BN;
    const float* __restrict__ A = (const float*)p.A + (long long)blockIdx.y * p.stride_a;
    const float* __restrict__ B = (const float*)p.B + (long long)blockIdx.y * p.stride_b;
    float* __restrict__ C = p.C + (long long)blockIdx.y * p.stride_c;

    const bool interior = !EDGE || (m0 + BM <= p.m_main && n0 + BN <= p.n_main);
    const int nk_all = (p.K + BK - 1) / BK;
    // (unsigned 32-bit: nk_all < 2^27 and nsplit <= 16; an unsplit tile divides nothing)
    int kb = 0, nk = nk_all;
    if (nsplit > 1) {
        kb = (int)((unsigned)(nk_all * split) / (unsigned)nsplit);
        nk = (int)((unsigned)(nk_all * (split + 1)) / (unsigned)nsplit) - kb;
    }

    // Leading steps of this workgroup whose chunks are all whole (inside or outside).
    // EDGEV 2 peels the k loop like Fig. 8: the ring runs the steps that lie wholly below K
    // without any test, and a last partial step is staged through registers after it
    // A tile whose chunks are cut by the end of a row along N (row-major B) or M (transposed A)
    // still takes whole 16-byte loads in the ring: the bytes past the end of a row are the start
    // of the next row, and only feed columns / rows of C that are never stored.  The last row of
    // the operand has no next row, so for such a tile the last k step is always peeled.
    const bool cut_tile = CLAMP && ((!B_KMAJ && (p.N % 4) && n0 + BN > p.N) || (AMODE == A_COL && (p.M % 4) && m0 + BM > p.M));
    int nkp_ = CLAMP ? min(nk, max(0, p.k_full - kb)) : nk;
    if (cut_tile && kb + nk == nk_all) nkp_ = min(nkp_, nk - 1);
    const int nkp = nkp_;   // steps that go through the ring
    int n_direct = nkp;
    if constexpr (CUT) {
        bool whole_tile = !(!B_KMAJ && (p.N & 3) && n0 + BN > p.N);            // rows of B are cut mid-chunk
        if (AMODE == A_COL && (p.M & 3) && m0 + BM > p.M) whole_tile = false;  // so are rows of A^T
        if (!whole_tile) n_direct = 0;
        else if ((AMODE == A_ROW || B_KMAJ) && (p.K & 3)) n_direct = max(0, min(nk, p.k_full - kb));
    }

    // The address of the block of zeros, taken once and kept in registers: derived where it is
    // used, it costs a scalar load and a wait for every outstanding LDS read in the middle of
    // the MFMA sequence of every step.
    const float* zero_chunk = g_zero_chunk;
    asm volatile("" : "+s"(zero_chunk));

    // LDS byte address of this wave's 1 KiB slice of pass 0 of stage 0 (wave-uniform)
    const unsigned lds0 = (unsigned)(size_t)(__attribute__((address_space(3))) float*)smem +
                          (unsigned)__builtin_amdgcn_readfirstlane(tid & ~63) * 16u;
    const int a_r = tid / A_CPR, a_cp = tid % A_CPR;
    const int b_r = tid / B_CPR, b_cp = tid % B_CPR;
    auto swz = [](int row) -> int { return (row / SW_DIV) % SW_MOD; };   // k-contiguous tiles only

    // per-thread source of each of its chunks at k0 = 0
    const float* a_src[PA];
    int a_k[PA];          // k offset of the chunk inside a step (k-contiguous A)
    bool a_in[PA];        // the chunk's row (A_ROW: m, A_COL: m range) lies inside the operand
    int cv_base[PA], cv_hi0[PA], cv_wi0[PA];
    long long cv_off[PA];   // element offset of tap (0, 0), channel a_k of the chunk's pixel (may lie outside the tensor)
#pragma unroll
    for (int q = 0; q < PA; ++q) {
        const int row = a_r + q * A_RPP;
        if constexpr (AMODE == A_ROW) {
            a_k[q] = (a_cp ^ swz(row)) * 4;
            a_in[q] = !CUT || m0 + row < p.M;
            a_src[q] = A + (long long)(CLAMP ? min(m0 + row, p.M - 1) : m0 + row) * p.lda + a_k[q];
        } else if constexpr (AMODE == A_COL) {
            a_k[q] = row;   // the stored row is the k index
            a_in[q] = !CUT || m0 + a_cp * 4 < p.M;
            a_src[q] = A + (long long)row * p.lda + (CLAMP && m0 + a_cp * 4 >= p.M ? max(p.M - 4, 0) : m0 + a_cp * 4);
        } else {
            a_k[q] = (a_cp ^ swz(row)) * 4;
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
    // (kh, kw, ci) of the first k of the next step to issue, advanced step by step (see the
    // register-staged kernel)
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
    const float* b_src[PB];
    int b_k[PB];          // k offset of the chunk inside a step: its row (B as K x N) or its swizzled chunk (N x K)
    bool b_in[PB];        // the chunk's n range lies inside the operand
#pragma unroll
    for (int q = 0; q < PB; ++q) {
        const int row = b_r + q * B_RPP;
        if constexpr (B_KMAJ) {
            b_k[q] = (b_cp ^ swz(row)) * 4;
            b_in[q] = !CUT || n0 + row < p.N;
            b_src[q] = B + (long long)(CLAMP ? min(n0 + row, p.N - 1) : n0 + row) * p.ldb + b_k[q];
        } else {
            b_k[q] = row;
            b_in[q] = !CUT || n0 + b_cp * 4 < p.N;
            b_src[q] = B + (long long)row * p.ldb + (CLAMP && n0 + b_cp * 4 >= p.N ? max(p.N - 4, 0) : n0 + b_cp * 4);
        }
    }

    // ---- one tile into one stage, direct
    auto issue_direct = [&](int kt, int stage) {
        const int k0 = kt * BK;
        const unsigned as = lds0 + (unsigned)(stage * L::STAGE) * 4u;
        const unsigned bs = as + (unsigned)L::A_FLOATS * 4u;
#pragma unroll
        for (int q = 0; q < PA; ++q) {
            const float* src;
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
                    const float* inside = A + (cv_off[q] + cs_off);
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
            const float* src = in ? b_src[q] + (B_KMAJ ? (long long)k0 : (long long)k0 * p.ldb) : zero_chunk;
            load_to_lds16(src, bs + (unsigned)(q * NT) * 16u);
        }
    };

    // ---- the same tile through registers with element masks (chunks cut by the end of a row)
    auto issue_masked = [&](int kt, int stage) {
        const int k0 = kt * BK;
        float* As = smem + stage * L::STAGE;
        float* Bs = As + L::A_FLOATS;
#pragma unroll
        for (int q = 0; q < PA; ++q) {
            const int row = a_r + q * A_RPP;
            f32x4 v = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if constexpr (AMODE == A_ROW) {
                    const int m = m0 + row, k = k0 + a_k[q] + e;
                    if (m < p.M && k < p.K) v[e] = A[(long long)m * p.lda + k];
                } else if constexpr (AMODE == A_COL) {
                    const int k = k0 + row, m = m0 + a_cp * 4 + e;
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
            *(f32x4*)(As + (q * NT + tid) * 4) = v;
        }
#pragma unroll
        for (int q = 0; q < PB; ++q) {
            const int row = b_r + q * B_RPP;
            f32x4 v = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if constexpr (B_KMAJ) {
                    const int n = n0 + row, k = k0 + b_k[q] + e;
                    if (n < p.N && k < p.K) v[e] = B[(long long)n * p.ldb + k];
                } else {
                    const int k = k0 + row, n = n0 + b_cp * 4 + e;
                    if (k < p.K && n < p.N) v[e] = B[(long long)k * p.ldb + n];
                }
            }
            *(f32x4*)(Bs + (q * NT + tid) * 4) = v;
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

    // fragment addressing: lane (li, lh) reads row wm0 + 32 i + li, chunk 2 g + lh of k group g
    int a_row_off[MI];   // float offset of the lane's row (k-contiguous A)
#pragma unroll
    for (int i = 0; i < MI; ++i) a_row_off[i] = (wm0 + i * 32 + li) * BK;
    int b_row_off[NI];   // the same for a k-contiguous B, whose rows are columns of C
#pragma unroll
    for (int j = 0; j < NI; ++j) b_row_off[j] = (wn0 + j * 32 + li) * BK;
    const int a_x = lh ^ swz(li);   // wm0 + 32 i is a multiple of 32, so the swizzle depends on li alone

    // ---- one direct load: the x-th of the LPT loads that bring a tile in
    // (`ktest`: also test the chunk's k against K, which the ring of the peeled variant never needs)
    auto load_one = [&](int kt, int stage, int x, bool ktest) {
        const int k0 = kt * BK;
        const unsigned as = lds0 + (unsigned)(stage * L::STAGE) * 4u;
        const unsigned bs = as + (unsigned)L::A_FLOATS * 4u;
        if (x < PA) {
            const int q = x;
            const float* src;
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
                    const float* inside = A + (cv_off[q] + cs_off);
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
            const float* src = in ? b_src[q] + (B_KMAJ ? (long long)k0 : (long long)k0 * p.ldb) : zero_chunk;
            load_to_lds16(src, bs + (unsigned)(q * NT) * 16u);
        }
    };
    // the x-th part of bringing in tile kt_local: one direct load, or (steps with cut chunks)
    // the whole masked tile at x = 0; the convolution's tap state moves on after the last part
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

    // ---- fragments: a k group (8 values of k = 4 MFMAs per block) is fetched while the group
    // before it is multiplied, one LDS read after each MFMA
    constexpr int G = BK / 8;
    static_assert(G % 2 == 0, "the fragment double buffer alternates per group across steps");
    constexpr int NFRAG = (A_KMAJ ? MI : 4 * MI) + (B_KMAJ ? NI : 4 * NI);   // LDS reads of one group's fragments
    constexpr int NM = 4 * MI * NI;                            // MFMAs of one group
    f32x4 af[2][MI], bf[2][NI];
    auto frag_read = [&](int stage, int g, int x) {
        const float* As = smem + stage * L::STAGE;
        const float* Bs = As + L::A_FLOATS;
        if constexpr (A_KMAJ) {
            if (x < MI) {
                af[g & 1][x] = *(const f32x4*)(As + a_row_off[x] + (((2 * g) ^ a_x) << 2));
                return;
            }
            x -= MI;
        } else {
            if (x < 4 * MI) {
                af[g & 1][x >> 2][x & 3] = As[(g * 8 + 4 * lh + (x & 3)) * BM + wm0 + (x >> 2) * 32 + li];
                return;
            }
            x -= 4 * MI;
        }
        if constexpr (B_KMAJ) bf[g & 1][x] = *(const f32x4*)(Bs + b_row_off[x] + (((2 * g) ^ a_x) << 2));
        else bf[g & 1][x >> 2][x & 3] = Bs[(g * 8 + 4 * lh + (x & 3)) * BN + wn0 + (x >> 2) * 32 + li];
    };

    // ---- ring.  Step kt is multiplied from stage kt % STAGES.  The one barrier of a step sits
    // before its LAST k group: by then tile kt+1 has landed (own loads: the wait; everybody's:
    // the barrier) and everybody has left step kt-1, so during that last group the loads of
    // tile kt+D go into the stage step kt-1 used and the first fragments of step kt+1 are
    // fetched.  No wave ever starts a step, or leaves a barrier, with its MFMA operands missing.
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
                // issued so far: tiles up to kt+D-1, so D-2 tiles may stay in flight behind tile kt+1
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
                const int t = m / (MI * NI), i = (m / NI) % MI, j = m % NI;
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[g & 1][i][t], bf[g & 1][j][t], acc[i][j], 0, 0, 0);
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
            if ((p.K % 4) || cut_tile) {
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
                const int t = m / (MI * NI), i = (m / NI) % MI, j = m % NI;
                acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[g & 1][i][t], bf[g & 1][j][t], acc[i][j], 0, 0, 0);
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
        // the direct-to-LDS forms move whole 16-byte chunks only
        if (variant == 2) return hipErrorInvalidValue;
        bytes = LdsDirect<T, AMODE>::BYTES;
        fn = variant == 0 ? gemm_f32_direct_kernel<T, AMODE, 0>
             : variant == 3 ? gemm_f32_direct_kernel<T, AMODE, 2> : gemm_f32_direct_kernel<T, AMODE, 1>;
        if constexpr (AMODE == A_CONV) {
            if (a.Cin % T::BK == 0) {
                one_tap = 1;
                fn = variant == 0 ? gemm_f32_direct_kernel<T, AMODE, 0, true>
                     : variant == 3 ? gemm_f32_direct_kernel<T, AMODE, 2, true> : gemm_f32_direct_kernel<T, AMODE, 1, true>;
            }
        }
    } else {
        bytes = Lds<T, AMODE>::BYTES;
        switch (variant) {
            case 0: fn = gemm_f32_kernel<T, AMODE, 4, false>; break;
            case 1:
            case 3: fn = gemm_f32_kernel<T, AMODE, 4, true>; break;
            default: fn = gemm_f32_kernel<T, AMODE, 1, true>; break;
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
#define TSG_F32_TILES(X)           \
    X(128, 128, 32, 64, 64, 2, 0)  \
    X(128, 128, 16, 64, 64, 2, 0)  \
    X(128, 128, 16, 64, 64, 2, 2)  \
    X(128, 128, 16, 64, 64, 2, 3)  \
    X(128, 128, 32, 64, 64, 2, 3)  \
    X(256, 128, 16, 64, 64, 2, 0)  \
    X(256, 128, 16, 64, 64, 2, 1)  \
    X(256, 128, 16, 64, 64, 2, 2)  \
    X(256, 128, 16, 64, 64, 2, 3)  \
    X(256, 128, 32, 64, 64, 2, 0)  \
    X(256, 128, 32, 64, 64, 2, 2)  \
    X(256, 128, 16, 128, 64, 2, 0) \
    X(256, 128, 16, 128, 64, 2, 2) \
    X(256, 256, 16, 128, 64, 2, 0) \
    X(256, 256, 16, 128, 64, 2, 2) \
    X(256, 256, 16, 128, 64, 2, 3) \
    X(128, 64, 32, 64, 32, 2, 0)   \
    X(128, 64, 32, 64, 32, 2, 2)   \
    X(128, 64, 64, 64, 32, 2, 2)   \
    X(64, 64, 32, 32, 32, 2, 0)    \
    X(64, 64, 32, 32, 32, 2, 2)    \
    X(64, 64, 16, 32, 32, 2, 0)    \
    X(64, 64, 64, 32, 32, 2, 0)    \
    X(64, 64, 64, 32, 32, 2, 2)    \
    X(64, 64, 32, 32, 32, 2, 3)    \
    X(128, 64, 32, 64, 32, 2, 3)   \
    X(64, 64, 128, 32, 32, 1, 2)   \
    X(64, 64, 32, 32, 32, 2, 4)    \
    X(64, 64, 64, 32, 32, 2, 4)    \
    X(64, 64, 64, 32, 32, 1, 5)    \
    X(128, 64, 32, 64, 32, 2, 4)   \
    X(128, 128, 16, 64, 64, 2, 4)  \
    X(128, 128, 32, 64, 64, 2, 4)  \
    X(256, 128, 16, 64, 64, 2, 4)  \
    X(256, 128, 16, 64, 64, 2, 5)  \
    X(256, 256, 16, 128, 64, 2, 4)

// Each address mode is compiled in its own translation unit.
#define TSG_F32_DEFINE_MODE(FN, AMODE)                                                              \
    namespace tsg {                                                                                 \
    hipError_t FN(int tile, int variant, const KArgs& a, int batch, hipStream_t s) {                \
        int idx = 0;                                                                                \
        TSG_F32_TILES(TSG_F32_CASE_##AMODE)                                                         \
        return hipErrorInvalidValue;                                                                \
    }                                                                                               \
    }
#define TSG_F32_CASE_A_ROW(bm, bn, bk, wm, wn, mw, sc) \
    if (tile == idx++) return launch_mode<Tile<bm, bn, bk, wm, wn, mw, sc>, A_ROW>(variant, a, batch, s);
#define TSG_F32_CASE_A_COL(bm, bn, bk, wm, wn, mw, sc) \
    if (tile == idx++) return launch_mode<Tile<bm, bn, bk, wm, wn, mw, sc>, A_COL>(variant, a, batch, s);
#define TSG_F32_CASE_A_CONV(bm, bn, bk, wm, wn, mw, sc) \
    if (tile == idx++) return launch_mode<Tile<bm, bn, bk, wm, wn, mw, sc>, A_CONV>(variant, a, batch, s);
#define TSG_F32_CASE_A_ROW_BT(bm, bn, bk, wm, wn, mw, sc) \
    if (tile == idx++) return launch_mode<Tile<bm, bn, bk, wm, wn, mw, sc>, A_ROW_BT>(variant, a, batch, s);
#define TSG_F32_CASE_A_COL_BT(bm, bn, bk, wm, wn, mw, sc) \
    if (tile == idx++) return launch_mode<Tile<bm, bn, bk, wm, wn, mw, sc>, A_COL_BT>(variant, a, batch, s);

// Full additive reduce for gfx950: out = +-sum of every element of a rows x cols view (+ out).
//
// Case Study 3 singles out the rewrite that lets a full additive reduce ignore a reshape or
// transpose of its operand: the sum of all elements does not depend on how they are indexed
// (up to floating-point rounding order), so the reduce can read the tensor as it lies in
// memory.  This is that reduce: one pass over the bytes, bound by HBM bandwidth.
//
// Order of summation (fixed by the launch, so results are repeatable): the view's 16-byte
// chunks are numbered in row-major order over (row, chunk within the row), so a workgroup's
// share spans rows and a view of many short rows fills the chip like a contiguous tensor.
// Thread t of workgroup b adds chunks b*256 + t + j*(G*256), j = 0, 1, ..., into four 4-wide
// partial sums (chunk j goes to sum j % 4); the 16 lanes of those are added in index order; waves
// reduce by halving (lane l += lane l + 32, 16, ..., 1), the four wave sums are added in
// order, and the last workgroup to arrive adds the G workgroup sums the same way.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/tsg.h"
#include "tsg_internal.h"

namespace tsg {
namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef f32x4 f32x4_u __attribute__((aligned(4)));
typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));
typedef u16x8 u16x8_u __attribute__((aligned(2)));

constexpr int kThreads = 256;
constexpr int kMaxGroups = 768;   // three workgroups per compute unit: more resident waves lower the rate (768: 6.8, 1024: 6.7, 2048: 5.7 TB/s)

__device__ __forceinline__ float bf16_bits_to_f32(unsigned short h) { return __uint_as_float((unsigned)h << 16); }

// sum of one workgroup's 256 values, in the fixed order described above; valid in thread 0
__device__ __forceinline__ float block_sum(float v) {
    __shared__ float wave_sums[kThreads / 64];
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_down(v, d, 64);
    if ((threadIdx.x & 63) == 0) wave_sums[threadIdx.x >> 6] = v;
    __syncthreads();
    float s = 0.f;
    if (threadIdx.x == 0) s = ((wave_sums[0] + wave_sums[1]) + wave_sums[2]) + wave_sums[3];
    __syncthreads();
    return s;
}

template <bool BF16>
__global__ void __launch_bounds__(kThreads) reduce_sum_kernel(const void* __restrict__ x, long long rows,
                                                               long long cols, long long ld, float* out,
                                                               unsigned flags, float* partials, int* counter) {
    constexpr int V = BF16 ? 8 : 4;   // elements per 16-byte chunk
    const int tid = threadIdx.x, G = gridDim.x;
    f32x4 acc[4];
#pragma unroll
    for (int a = 0; a < 4; ++a) acc[a] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Every byte is read once and never again: the loads are marked non-temporal, so the stream
    // does not displace what the caches hold (measured on 1 GiB: 6.8 against 6.2 TB/s).
    auto add_chunk = [&](f32x4& a, const void* p, long long valid) {
        // `valid` elements of the chunk exist (>= V for a whole chunk)
        if (valid >= V) {
            if constexpr (BF16) {
                const u16x8 h = __builtin_nontemporal_load((const u16x8_u*)p);
#pragma unroll
                for (int e = 0; e < 8; ++e) a[e & 3] += bf16_bits_to_f32(h[e]);
            } else {
                a += __builtin_nontemporal_load((const f32x4_u*)p);
            }
        } else {
            for (int e = 0; e < valid; ++e) {
                if constexpr (BF16) a[e & 3] += bf16_bits_to_f32(((const unsigned short*)p)[e]);
                else a[e & 3] += ((const float*)p)[e];
            }
        }
    };

    // The view is rows of `cpr` chunks (the last chunk of a row may be short); chunk number c in
    // row-major order over (row, chunk in row) is what the order of summation above counts.  A
    // contiguous tensor arrives as one row.  The (row, chunk) pair of a thread's next chunk is
    // stepped, not divided out: the stride of G*256 chunks is split once into whole rows and a
    // remainder.
    const long long cpr = (cols + V - 1) / V;
    const long long total = rows * cpr;
    const long long stride = (long long)G * kThreads;
    const long long es = BF16 ? 2 : 4;
    long long c = (long long)blockIdx.x * kThreads + tid;
    if (rows == 1 && cols % V == 0) {
        // one contiguous run of whole chunks: nothing to step but the chunk number
        const char* base = (const char*)x;
        for (; c + 3 * stride < total; c += 4 * stride) {
#pragma unroll
            for (int u = 0; u < 4; ++u) add_chunk(acc[u], base + (c + u * stride) * 16, V);
        }
        for (int j = 0; c < total; c += stride, ++j) add_chunk(acc[j & 3], base + c * 16, V);
    } else {
        long long r = c / cpr, cc = c - r * cpr;
        const long long dr = stride / cpr, dc = stride - dr * cpr;
        const char* ptr = (const char*)x + (r * ld + cc * V) * es;
        const long long step_bytes = (dr * ld + dc * V) * es, wrap_bytes = (ld - cpr * V) * es;
        auto advance = [&]() {
            c += stride;
            ptr += step_bytes;
            cc += dc;
            if (cc >= cpr) { cc -= cpr; ptr += wrap_bytes; }
        };
        // four chunks in flight per thread
        while (c + 3 * stride < total) {
            const void* p4[4];
            long long valid[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                p4[u] = ptr;
                valid[u] = cols - cc * V;
                advance();
            }
            // (whole chunks, the usual case, are loaded together; a short chunk at the end of a
            // row takes the element loop)
            if (valid[0] >= V && valid[1] >= V && valid[2] >= V && valid[3] >= V) {
#pragma unroll
                for (int u = 0; u < 4; ++u) add_chunk(acc[u], p4[u], V);
            } else {
#pragma unroll
                for (int u = 0; u < 4; ++u) add_chunk(acc[u], p4[u], valid[u]);
            }
        }
        for (int j = 0; c < total; ++j) {
            add_chunk(acc[j & 3], ptr, cols - cc * V);
            advance();
        }
    }
    float v = 0.f;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int e = 0; e < 4; ++e) v += acc[a][e];
    float s = block_sum(v);

    if (G > 1) {
        // park the workgroup sum, count the arrival; the last arrival adds all G sums
        __shared__ int arrived;
        if (tid == 0) {
            __hip_atomic_store(partials + blockIdx.x, s, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            arrived = __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
        if (arrived != G - 1) return;
        float t = 0.f;
        for (int i = tid; i < G; i += kThreads)
            t += __hip_atomic_load(partials + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s = block_sum(t);
        if (tid == 0) __hip_atomic_store(counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (tid == 0) {
        if (flags & TSG_NEGATE) s = -s;
        if (flags & TSG_ACCUMULATE) s += *out;
        *out = s;
    }
}

}  // namespace
}  // namespace tsg

extern "C" tsg_status tsg_reduce_sum(tsg_dtype dtype, int64_t rows, int64_t cols, const void* x, int64_t ld, float* out,
                                     uint32_t flags, void* stream) {
    if (dtype != TSG_F32 && dtype != TSG_BF16_F32ACC) return TSG_E_INVALID;
    if (!x || !out || rows <= 0 || cols <= 0 || ld < cols) return TSG_E_INVALID;
    if (flags & ~(uint32_t)(TSG_NEGATE | TSG_ACCUMULATE | TSG_STRICT)) return TSG_E_INVALID;
    if (rows > (int64_t)1 << 40 || cols > (int64_t)1 << 40 || rows * cols > (int64_t)1 << 40) return TSG_E_INVALID;
    if (ld == cols) { cols *= rows; ld = cols; rows = 1; }   // a contiguous tensor is one long row
    const int v = dtype == TSG_F32 ? 4 : 8;
    const int64_t chunks = rows * ((cols + v - 1) / v);
    // enough workgroups to keep every CU streaming, each with at least 16 chunks per thread
    int64_t groups = chunks / (tsg::kThreads * 16);
    groups = groups < 1 ? 1 : groups > tsg::kMaxGroups ? tsg::kMaxGroups : groups;
    void* ws = nullptr;
    int64_t ws_bytes = 0;
    long long wsb = 0;
    tsg::workspace_get(stream, &ws, &wsb);
    ws_bytes = wsb;
    if (groups > 1 && (!ws || ws_bytes < tsg::kWorkspaceCounterBytes + groups * 4)) {
        // more than one workgroup needs the workspace for its partial sums
        if (flags & TSG_STRICT) return TSG_E_SILENCEABLE;
        groups = 1;
    }
    float* partials = ws ? (float*)((char*)ws + tsg::kWorkspaceCounterBytes) : nullptr;
    int* counter = ws ? (int*)ws + tsg::kWorkspaceReduceSlot : nullptr;   // its own slot: a GEMM may share the buffer
    const unsigned f = flags & (TSG_NEGATE | TSG_ACCUMULATE);
    if (dtype == TSG_F32)
        hipLaunchKernelGGL(tsg::reduce_sum_kernel<false>, dim3((unsigned)groups), dim3(tsg::kThreads), 0,
                           (hipStream_t)stream, x, (long long)rows, (long long)cols, (long long)ld, out, f, partials,
                           counter);
    else
        hipLaunchKernelGGL(tsg::reduce_sum_kernel<true>, dim3((unsigned)groups), dim3(tsg::kThreads), 0,
                           (hipStream_t)stream, x, (long long)rows, (long long)cols, (long long)ld, out, f, partials,
                           counter);
    return hipGetLastError() == hipSuccess ? TSG_OK : TSG_E_RUNTIME;
}

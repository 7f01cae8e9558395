// Measurement aid for the roofline: what the matrix pipes of this GPU sustain when every operand
// already sits in registers (no LDS, no global memory, no barrier).  The contraction kernels
// are priced against the published peak; this loop gives the practical ceiling under it, and
// shows how far that ceiling moves with the operand VALUES (a power effect: constant operands
// toggle few bits) and with the MFMA block shape.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/tsg.h"

namespace tsg {
namespace {

typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ unsigned mix32(unsigned x) {
    x ^= x >> 16; x *= 0x7feb352du; x ^= x >> 15; x *= 0x846ca68bu; x ^= x >> 16;
    return x;
}
// a value with the distribution of the workloads' entries: N(0,1) / 90.5 (= 1/sqrt(8192)), or a constant
__device__ __forceinline__ float operand(unsigned idx, bool random) {
    if (!random) return 0.5f;
    const float u1 = ((mix32(2u * idx + 1u) >> 8) + 0.5f) * (1.0f / 16777216.0f);
    const float u2 = ((mix32(2u * idx + 2u) >> 8) + 0.5f) * (1.0f / 16777216.0f);
    return sqrtf(-2.0f * __logf(u1)) * __cosf(6.2831853f * u2) * (1.0f / 90.5f);
}

// KIND 0: fp32 32x32x2, 1: fp32 16x16x4, 2: bf16 32x32x16, 3: bf16 16x16x32.
// Eight operand registers are cycled so that consecutive MFMAs do not reuse one pair.
template <int KIND>
__global__ void __launch_bounds__(256) mfma_loop(float* sink, int iters, int random) {
    const unsigned t = blockIdx.x * 256u + threadIdx.x;
    float s = 0.f;
    if constexpr (KIND == 0 || KIND == 1) {
        float xs[8], ys[8];
        for (int e = 0; e < 8; ++e) { xs[e] = operand(t * 16u + e, random); ys[e] = operand(t * 16u + 8u + e, random); }
        f32x16 a[4] = {};
        f32x4 c[8] = {};
        for (int i = 0; i < iters; ++i) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                if constexpr (KIND == 0) {
#pragma unroll
                    for (int u = 0; u < 4; ++u) a[u] = __builtin_amdgcn_mfma_f32_32x32x2f32(xs[e], ys[(e + u) & 7], a[u], 0, 0, 0);
                } else {
#pragma unroll
                    for (int u = 0; u < 8; ++u) c[u] = __builtin_amdgcn_mfma_f32_16x16x4f32(xs[e], ys[(e + u) & 7], c[u], 0, 0, 0);
                }
            }
        }
        for (int u = 0; u < 4; ++u) for (int r = 0; r < 16; ++r) s += a[u][r];
        for (int u = 0; u < 8; ++u) for (int r = 0; r < 4; ++r) s += c[u][r];
    } else {
        bf16x8 xs[8], ys[8];
        for (int e = 0; e < 8; ++e)
            for (int q = 0; q < 8; ++q) {
                xs[e][q] = (__bf16)operand(t * 128u + e * 8u + q, random);
                ys[e][q] = (__bf16)operand(t * 128u + 64u + e * 8u + q, random);
            }
        f32x16 a[4] = {};
        f32x4 c[8] = {};
        for (int i = 0; i < iters; ++i) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                if constexpr (KIND == 2) {
#pragma unroll
                    for (int u = 0; u < 4; ++u) a[u] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xs[e], ys[(e + u) & 7], a[u], 0, 0, 0);
                } else {
#pragma unroll
                    for (int u = 0; u < 8; ++u) c[u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(xs[e], ys[(e + u) & 7], c[u], 0, 0, 0);
                }
            }
        }
        for (int u = 0; u < 4; ++u) for (int r = 0; r < 16; ++r) s += a[u][r];
        for (int u = 0; u < 8; ++u) for (int r = 0; r < 4; ++r) s += c[u][r];
    }
    sink[t] = s;
}

// the fixed cost of a launch: a kernel whose one wave returns at once
__global__ void empty_kernel() {}

}  // namespace
}  // namespace tsg

extern "C" tsg_status tsg_launch_floor(int32_t launches, float* us_per_launch, void* stream) {
    if (launches < 1 || launches > 1000000 || !us_per_launch) return TSG_E_INVALID;
    hipStream_t s = (hipStream_t)stream;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return TSG_E_RUNTIME;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return TSG_E_RUNTIME; }
    tsg_status st = TSG_OK;
    float ms = 0.f;
    // two passes: the first one also pays for loading the code object
    for (int pass = 0; pass < 2 && st == TSG_OK; ++pass) {
        if (hipEventRecord(e0, s) != hipSuccess) { st = TSG_E_RUNTIME; break; }
        for (int l = 0; l < launches; ++l) hipLaunchKernelGGL(tsg::empty_kernel, dim3(1), dim3(64), 0, s);
        if (hipGetLastError() != hipSuccess || hipEventRecord(e1, s) != hipSuccess ||
            hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&ms, e0, e1) != hipSuccess)
            st = TSG_E_RUNTIME;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (st != TSG_OK) return st;
    *us_per_launch = ms * 1000.f / launches;
    return TSG_OK;
}

extern "C" tsg_status tsg_mfma_ceiling(tsg_dtype dtype, int32_t mfma, int32_t random_operands, int32_t waves_per_simd,
                                       int32_t launches, float* sink, int64_t sink_bytes, float* tflops,
                                       void* stream) {
    if ((dtype != TSG_F32 && dtype != TSG_BF16_F32ACC) || (mfma != 0 && mfma != 1)) return TSG_E_INVALID;
    if (waves_per_simd < 1 || waves_per_simd > 2 || launches < 2 || launches > 1000 || !sink || !tflops)
        return TSG_E_INVALID;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
        return TSG_E_RUNTIME;
    const int blocks = cus * waves_per_simd;                 // 256 threads = one wave per SIMD of a CU
    if (sink_bytes < (int64_t)blocks * 256 * 4) return TSG_E_INVALID;
    const int kind = (dtype == TSG_F32 ? 0 : 2) + mfma;
    // every inner pass issues 32 (32 x 32 blocks) or 64 (16 x 16) MFMAs per wave: 131072 flop for
    // fp32 and 1048576 for bf16 either way
    const double flop_per_iter = dtype == TSG_F32 ? 131072.0 : 1048576.0;
    const int iters = (dtype == TSG_F32 ? 6000 : 20000) / waves_per_simd;   // about 10 ms per launch
    hipStream_t s = (hipStream_t)stream;
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return TSG_E_RUNTIME;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return TSG_E_RUNTIME; }
    float best = -1.f;
    double late = 0.0;   // time of the launches in the second half: the rate the chip sustains
    tsg_status st = TSG_OK;
    for (int l = 0; l < launches && st == TSG_OK; ++l) {
        if (hipEventRecord(e0, s) != hipSuccess) { st = TSG_E_RUNTIME; break; }
        switch (kind) {
            case 0: hipLaunchKernelGGL(tsg::mfma_loop<0>, dim3(blocks), dim3(256), 0, s, sink, iters, random_operands); break;
            case 1: hipLaunchKernelGGL(tsg::mfma_loop<1>, dim3(blocks), dim3(256), 0, s, sink, iters, random_operands); break;
            case 2: hipLaunchKernelGGL(tsg::mfma_loop<2>, dim3(blocks), dim3(256), 0, s, sink, iters, random_operands); break;
            default: hipLaunchKernelGGL(tsg::mfma_loop<3>, dim3(blocks), dim3(256), 0, s, sink, iters, random_operands); break;
        }
        float t = 0.f;
        if (hipGetLastError() != hipSuccess || hipEventRecord(e1, s) != hipSuccess ||
            hipEventSynchronize(e1) != hipSuccess || hipEventElapsedTime(&t, e0, e1) != hipSuccess) {
            st = TSG_E_RUNTIME;
            break;
        }
        if (best < 0 || t < best) best = t;
        if (l >= launches / 2) late += t;
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (st != TSG_OK) return st;
    const double flop = flop_per_iter * iters * 4.0 * blocks;
    tflops[0] = (float)(flop / (best * 1e-3) / 1e12);
    tflops[1] = (float)(flop / (late / (launches - launches / 2) * 1e-3) / 1e12);
    return TSG_OK;
}

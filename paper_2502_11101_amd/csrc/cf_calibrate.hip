// Calibration kernels of known size (cf_calibrate): a plain streaming read, a plain copy, and a dense MFMA loop
// without memory traffic.  What they sustain on the GPU at hand is the measured peak that the attention kernels'
// figures are priced against beside the nominal one.  Not part of the method.
#include "cf_common.h"

namespace cf {
namespace {

constexpr int kThreads = 256;
constexpr int kUnroll = 8;          // independent 16-byte loads in flight per thread

// Every workgroup streams a contiguous share of the buffer; the xor of what it read decides a store that never
// happens, so the loads cannot be dropped.
__global__ __launch_bounds__(kThreads) void calib_read_kernel(const uint4* __restrict__ src, size_t n16, uint4* sink) {
    const size_t per_wg = (n16 + gridDim.x - 1) / gridDim.x;
    const size_t lo = (size_t)blockIdx.x * per_wg;
    const size_t hi = lo + per_wg < n16 ? lo + per_wg : n16;
    uint4 acc = make_uint4(0, 0, 0, 0);
    for (size_t i = lo + threadIdx.x; i < hi; i += (size_t)kThreads * kUnroll) {
        uint4 v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const size_t j = i + (size_t)u * kThreads;
            v[u] = src[j < hi ? j : lo];                     // clamped, in bounds: a fixed number of loads per step
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) { acc.x ^= v[u].x; acc.y ^= v[u].y; acc.z ^= v[u].z; acc.w ^= v[u].w; }
    }
    if (acc.x == 0x12345678u && acc.y == 0x9abcdef0u && acc.z == 0x0fedcba9u) sink[0] = acc;
}

__global__ __launch_bounds__(kThreads) void calib_copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
    const size_t per_wg = (n16 + gridDim.x - 1) / gridDim.x;
    const size_t lo = (size_t)blockIdx.x * per_wg;
    const size_t hi = lo + per_wg < n16 ? lo + per_wg : n16;
    for (size_t i = lo + threadIdx.x; i < hi; i += (size_t)kThreads * kUnroll) {
        uint4 v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const size_t j = i + (size_t)u * kThreads;
            v[u] = src[j < hi ? j : lo];
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const size_t j = i + (size_t)u * kThreads;
            if (j < hi) dst[j] = v[u];
        }
    }
}

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
constexpr int kMfmaPerIter = 64;

// Eight independent 32x32 accumulators per wavefront, eight rounds over them per iteration.
template <int DT>
__global__ __launch_bounds__(kThreads) void calib_mfma_kernel(int iters, float* sink) {
    f32x16 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
    const float seed = (float)(threadIdx.x & 3) * 0.25f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int r = 0; r < kMfmaPerIter / 8; ++r)
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                if constexpr (DT == CF_BF16) {
                    bf16x8 a, b;
#pragma unroll
                    for (int e = 0; e < 8; ++e) { a[e] = (__bf16)seed; b[e] = (__bf16)(float)(e & 1); }
                    acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
                } else {
                    f16x8 a, b;
#pragma unroll
                    for (int e = 0; e < 8; ++e) { a[e] = (_Float16)seed; b[e] = (_Float16)(float)(e & 1); }
                    acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc[i], 0, 0, 0);
                }
            }
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) s += acc[i][0] + acc[i][15];
    if (s == -1.f) sink[0] = s;                              // sums of non-negative products: never
}

}  // namespace
}  // namespace cf

using namespace cf;

extern "C" cf_status cf_calibrate(int32_t kind, const void* src, void* dst, size_t bytes, int32_t workgroups, int32_t iters,
                                  void* sink, double* flops, void* stream) {
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (flops) *flops = 0.0;
    CF_REQUIRE(sink != nullptr, CF_ERR_INVALID_ARG, "sink must not be NULL");
    CF_REQUIRE(workgroups >= 1 && workgroups <= (1 << 20), CF_ERR_INVALID_ARG, "workgroups must be in [1, 2^20]");
    if (kind == CF_CALIB_READ || kind == CF_CALIB_COPY) {
        CF_REQUIRE(src != nullptr && bytes >= 16 && bytes % 16 == 0, CF_ERR_INVALID_ARG, "src NULL or bytes not a positive multiple of 16");
        CF_REQUIRE((reinterpret_cast<uintptr_t>(src) & 15u) == 0 && (reinterpret_cast<uintptr_t>(dst) & 15u) == 0 &&
                       (reinterpret_cast<uintptr_t>(sink) & 15u) == 0,
                   CF_ERR_INVALID_ARG, "src, dst and sink must be 16-byte aligned");
        if (kind == CF_CALIB_READ) {
            hipLaunchKernelGGL(calib_read_kernel, dim3(workgroups), dim3(kThreads), 0, s, static_cast<const uint4*>(src), bytes / 16,
                               static_cast<uint4*>(sink));
        } else {
            CF_REQUIRE(dst != nullptr && dst != src, CF_ERR_INVALID_ARG, "a copy needs a dst other than src");
            hipLaunchKernelGGL(calib_copy_kernel, dim3(workgroups), dim3(kThreads), 0, s, static_cast<const uint4*>(src),
                               static_cast<uint4*>(dst), bytes / 16);
        }
    } else if (kind == CF_CALIB_MFMA_BF16 || kind == CF_CALIB_MFMA_F16) {
        CF_REQUIRE(iters >= 1, CF_ERR_INVALID_ARG, "iters must be >= 1");
        if (kind == CF_CALIB_MFMA_BF16)
            hipLaunchKernelGGL((calib_mfma_kernel<CF_BF16>), dim3(workgroups), dim3(kThreads), 0, s, iters, static_cast<float*>(sink));
        else
            hipLaunchKernelGGL((calib_mfma_kernel<CF_F16>), dim3(workgroups), dim3(kThreads), 0, s, iters, static_cast<float*>(sink));
        if (flops) *flops = (double)workgroups * (kThreads / kWave) * (double)iters * kMfmaPerIter * 32768.0;
    } else {
        set_error("unknown calibration kind %d", kind);
        return CF_ERR_INVALID_ARG;
    }
    CF_HIP(hipGetLastError());
    return CF_OK;
}

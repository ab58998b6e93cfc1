// Plain streaming kernels of known traffic: a copy (read n bytes, write n bytes), a read
// (n bytes in, one float per workgroup out) and a fill (n bytes out).  They calibrate the
// HBM byte counters of the profiler against a known size and give the practical
// streaming rate of the device next to the published peak.  The copy and the fill also exist
// with nontemporal stores, which is how the library's own kernels write data they will not read
// again.
#include "../../include/leet_attn.h"
#include "../../include/leet_attn_bench.h"
#include "leet_common.hpp"

namespace leet {

constexpr int kCalibThreads = 256;
constexpr int kCalibUnroll = 8;  // 16-byte accesses in flight per thread

template <bool kNt>
__device__ __forceinline__ void calib_store(f32x4* p, f32x4 v) {
    if (kNt) __builtin_nontemporal_store(v, p);
    else *p = v;
}

template <bool kNt>
__global__ __launch_bounds__(kCalibThreads) void calib_copy_kernel(const f32x4* __restrict__ src,
                                                                   f32x4* __restrict__ dst, size_t n16) {
    const size_t stride = (size_t)gridDim.x * kCalibThreads;
    size_t i = (size_t)blockIdx.x * kCalibThreads + threadIdx.x;
    for (; i + (kCalibUnroll - 1) * stride < n16; i += kCalibUnroll * stride) {
        f32x4 r[kCalibUnroll];
#pragma unroll
        for (int u = 0; u < kCalibUnroll; ++u) r[u] = src[i + u * stride];
#pragma unroll
        for (int u = 0; u < kCalibUnroll; ++u) calib_store<kNt>(&dst[i + u * stride], r[u]);
    }
    for (; i < n16; i += stride) calib_store<kNt>(&dst[i], src[i]);
}

__global__ __launch_bounds__(kCalibThreads) void calib_read_kernel(const f32x4* __restrict__ src,
                                                                   float* __restrict__ sink, size_t n16) {
    const size_t stride = (size_t)gridDim.x * kCalibThreads;
    size_t i = (size_t)blockIdx.x * kCalibThreads + threadIdx.x;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (; i + (kCalibUnroll - 1) * stride < n16; i += kCalibUnroll * stride) {
        f32x4 r[kCalibUnroll];
#pragma unroll
        for (int u = 0; u < kCalibUnroll; ++u) r[u] = src[i + u * stride];
#pragma unroll
        for (int u = 0; u < kCalibUnroll; ++u) acc += r[u];
    }
    for (; i < n16; i += stride) acc += src[i];
    float s = acc[0] + acc[1] + acc[2] + acc[3];
    // keep the loads alive without a measurable write stream: one float per workgroup
    __shared__ float red[kCalibThreads];
    red[threadIdx.x] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        float t = 0.f;
        for (int k = 0; k < kCalibThreads; ++k) t += red[k];
        sink[blockIdx.x] = t;
    }
}

template <bool kNt>
__global__ __launch_bounds__(kCalibThreads) void calib_fill_kernel(f32x4* __restrict__ dst, size_t n16, float value) {
    const size_t stride = (size_t)gridDim.x * kCalibThreads;
    const f32x4 v = {value, value, value, value};
    for (size_t i = (size_t)blockIdx.x * kCalibThreads + threadIdx.x; i < n16; i += stride) calib_store<kNt>(&dst[i], v);
}

}  // namespace leet

extern "C" int leet_attn_calibration_stream(int mode, const void* src, void* dst, size_t bytes, int workgroups,
                                            void* stream) {
    if (bytes == 0 || (bytes & 15u) || workgroups <= 0 || workgroups > (1 << 20)) return LEET_ERR_INVALID_ARG;
    if (mode < 0 || mode > 4) return LEET_ERR_INVALID_ARG;
    if ((mode != 2 && mode != 4 && !src) || !dst) return LEET_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(src) & 15u) || (reinterpret_cast<uintptr_t>(dst) & 15u)) return LEET_ERR_INVALID_ARG;
    const size_t n16 = bytes / 16;
    hipStream_t s = static_cast<hipStream_t>(stream);
    dim3 grid(workgroups), block(leet::kCalibThreads);
    if (mode == 0)
        hipLaunchKernelGGL(leet::calib_copy_kernel<false>, grid, block, 0, s, static_cast<const leet::f32x4*>(src),
                           static_cast<leet::f32x4*>(dst), n16);
    else if (mode == 3)
        hipLaunchKernelGGL(leet::calib_copy_kernel<true>, grid, block, 0, s, static_cast<const leet::f32x4*>(src),
                           static_cast<leet::f32x4*>(dst), n16);
    else if (mode == 4)
        hipLaunchKernelGGL(leet::calib_fill_kernel<true>, grid, block, 0, s, static_cast<leet::f32x4*>(dst), n16, 1.0f);
    else if (mode == 1)
        hipLaunchKernelGGL(leet::calib_read_kernel, grid, block, 0, s, static_cast<const leet::f32x4*>(src),
                           static_cast<float*>(dst), n16);
    else
        hipLaunchKernelGGL(leet::calib_fill_kernel<false>, grid, block, 0, s, static_cast<leet::f32x4*>(dst), n16, 1.0f);
    return hipGetLastError() == hipSuccess ? LEET_OK : LEET_ERR_LAUNCH;
}

// Calibration kernels for the benchmark: a plain copy and register-only MFMA loops (INT8 and
// FP6).  None is part of the layer.
#include "dvdq_internal.h"
#include "../../include/dvdq_bench.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(256) void copy_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst, size_t n) {
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) dst[i] = src[i];
}

__global__ __launch_bounds__(256) void mfma_i8_kernel(int iters, int32_t *sink) {
    v4i a = {(int)threadIdx.x, 1, 2, 3}, b = {3, 2, 1, (int)blockIdx.x};
    v16i acc[16];
#pragma unroll
    for (int t = 0; t < 16; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int t = 0; t < 16; ++t) acc[t] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[t], 0, 0, 0);
    }
    int s = 0;
#pragma unroll
    for (int t = 0; t < 16; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) s ^= acc[t][r];
    if (s == 0x7fffffff) sink[0] = s;  // practically never true; keeps the loop alive
}

typedef int v8i __attribute__((ext_vector_type(8)));
typedef float v16f __attribute__((ext_vector_type(16)));

__global__ __launch_bounds__(256) void mfma_fp6_kernel(int iters, int32_t *sink) {
    // E2M3 patterns of small integers / 8 in every field (values stay finite: the sums are bounded by iters)
    v8i a = {0x04104104, 0x41041041, 0x10410410, 0x04104104, 0x41041041, 0x10410410, 0, 0};
    v8i b = {0x08208208, (int)0x82082082, 0x20820820, 0x08208208, (int)0x82082082, 0x20820820, 0, 0};
    a[0] ^= (int)(threadIdx.x & 3);
    v16f acc[8];
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int t = 0; t < 8; ++t)
            acc[t] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc[t], 2, 2, 0, 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[t][r];
    if (s == -1.f) sink[0] = 1;  // never true (the sums are positive); keeps the loop alive
}

constexpr int kMfmaBlocks = 256 * 2;  // two 4-wave workgroups per compute unit

}  // namespace

extern "C" {

int dvdq_bench_copy(const void *src, void *dst, size_t bytes, void *hip_stream) {
    if (!src || !dst) return DVDQ_ERR_NULL;
    if (bytes == 0 || (bytes % 16) != 0) return DVDQ_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(src) & 15u) || (reinterpret_cast<uintptr_t>(dst) & 15u)) return DVDQ_ERR_ALIGN;
    const size_t n = bytes / 16;
    size_t blocks = (n + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    hipLaunchKernelGGL(copy_kernel, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<const uint4 *>(src), static_cast<uint4 *>(dst), n);
    return dvdq::check_launch();
}

int dvdq_bench_mfma_i8(int iters, int32_t *sink, double *ops_out, void *hip_stream) {
    if (!sink) return DVDQ_ERR_NULL;
    if (iters < 1) return DVDQ_ERR_SHAPE;
    hipLaunchKernelGGL(mfma_i8_kernel, dim3(kMfmaBlocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream), iters,
                       sink);
    if (ops_out) *ops_out = 2.0 * 32 * 32 * 32 * 16.0 * iters * 4.0 * kMfmaBlocks;
    return dvdq::check_launch();
}

int dvdq_bench_mfma_fp6(int iters, int32_t *sink, double *ops_out, void *hip_stream) {
    if (!sink) return DVDQ_ERR_NULL;
    if (iters < 1) return DVDQ_ERR_SHAPE;
    hipLaunchKernelGGL(mfma_fp6_kernel, dim3(kMfmaBlocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream), iters,
                       sink);
    if (ops_out) *ops_out = 2.0 * 32 * 32 * 64 * 8.0 * iters * 4.0 * kMfmaBlocks;
    return dvdq::check_launch();
}

int dvdq_bench_set_gemm_variant(int variant) {
    dvdq::set_gemm_variant(variant);
    return DVDQ_OK;
}

int dvdq_bench_set_gemm_schedule(int schedule) {
    if (schedule < -1 || schedule > 0) return DVDQ_ERR_UNSUPPORTED;
    dvdq::set_gemm_schedule(schedule);
    return DVDQ_OK;
}

}  // extern "C"

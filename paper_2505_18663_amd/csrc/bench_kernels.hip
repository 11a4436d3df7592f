// Calibration kernels for the benchmark: a plain copy and register-only MFMA loops (INT8 and
// FP6, on constant or on random operands).  None is part of the layer.
#include "dvdq_internal.h"
#include "../../include/dvdq_bench.h"

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// Streaming copy used as the yardstick for HBM-bound kernels: every lane keeps four independent 16-byte
// non-temporal loads in flight (a wave instruction covers one contiguous kilobyte), then stores them
// non-temporally; workgroups stride over the buffer.
typedef uint32_t v4u __attribute__((ext_vector_type(4)));
constexpr int kCopyUnroll = 4;
__global__ __launch_bounds__(256) void copy_kernel(const v4u *__restrict__ src, v4u *__restrict__ dst, size_t n) {
    const size_t stride = (size_t)gridDim.x * (256 * kCopyUnroll);
    size_t i = (size_t)blockIdx.x * (256 * kCopyUnroll) + threadIdx.x;
    for (; i + 256 * (kCopyUnroll - 1) < n; i += stride) {
        v4u v[kCopyUnroll];
#pragma unroll
        for (int u = 0; u < kCopyUnroll; ++u) v[u] = __builtin_nontemporal_load(src + i + 256 * u);
#pragma unroll
        for (int u = 0; u < kCopyUnroll; ++u) __builtin_nontemporal_store(v[u], dst + i + 256 * u);
    }
    for (int u = 0; u < kCopyUnroll; ++u)   // the last, partial group of the buffer (at most one workgroup gets here with work)
        if (i + 256 * u < n) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i + 256 * u), dst + i + 256 * u);
}

// Operand words of the MFMA loops.  data 0: the same small constants in every lane (nothing but MFMA issue
// limits the loop); data 1: independent random 4-bit codes in every lane and register, as the layer's
// operands are.  The chip's power management clocks the matrix cores by what they draw, and that depends on
// how many operand bits change from one instruction to the next: the second figure is the rate the chip
// sustains on the layer's kind of data.
__device__ __forceinline__ uint32_t lane_hash(uint32_t i) {
    uint32_t h = (i + 1u + blockIdx.x * 7919u + threadIdx.x * 104729u) * 2654435761u;
    h ^= h >> 15;
    h *= 2246822519u;
    h ^= h >> 13;
    return h;
}
// four random codes in [-7, 7] as int8 bytes
__device__ __forceinline__ int random_i8_codes(uint32_t i) {
    const uint32_t h = lane_hash(i);
    int w = 0;
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        const int c = (int)((h >> (8 * b)) % 15u) - 7;
        w |= (c & 0xFF) << (8 * b);
    }
    return w;
}
// 32 bits of consecutive E2M3 fields (sign << 5 | magnitude <= 7); field boundaries need not line up with the
// word for this purpose: bits 3 and 4 of every 6-bit group starting at bit `phase` are cleared
__device__ __forceinline__ int random_fp6_codes(uint32_t i, int phase) {
    uint32_t h = lane_hash(i);
#pragma unroll
    for (int bit = 0; bit < 32; ++bit) {
        const int f = (bit + phase) % 6;
        if (f == 3 || f == 4) h &= ~(1u << bit);
    }
    return (int)h;
}

__global__ __launch_bounds__(256) void mfma_i8_kernel(int iters, int data, int32_t *sink) {
    v4i a[4], b[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        a[t] = v4i{(int)threadIdx.x, 1, 2, 3};
        b[t] = v4i{3, 2, 1, (int)blockIdx.x};
        if (data) {
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                a[t][r] = random_i8_codes(8 * t + r);
                b[t][r] = random_i8_codes(64 + 8 * t + r);
            }
        }
    }
    v16i acc[16];
#pragma unroll
    for (int t = 0; t < 16; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int t = 0; t < 16; ++t) acc[t] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[t / 4], b[t % 4], acc[t], 0, 0, 0);
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

__global__ __launch_bounds__(256) void mfma_fp6_kernel(int iters, int data, int32_t *sink) {
    // E2M3 patterns of small integers / 8 in every field (values stay finite: the sums are bounded by iters)
    v8i a[2], b[4];
#pragma unroll
    for (int t = 0; t < 4; ++t) {
        if (t < 2) a[t] = v8i{0x04104104, 0x41041041, 0x10410410, 0x04104104, 0x41041041, 0x10410410, 0, 0};
        b[t] = v8i{0x08208208, (int)0x82082082, 0x20820820, 0x08208208, (int)0x82082082, 0x20820820, 0, 0};
        if (data) {
#pragma unroll
            for (int r = 0; r < 6; ++r) {
                if (t < 2) a[t][r] = random_fp6_codes(8 * t + r, (32 * r) % 6);
                b[t][r] = random_fp6_codes(64 + 8 * t + r, (32 * r) % 6);
            }
        }
    }
    a[0][0] ^= (int)(threadIdx.x & 3);
    v16f acc[8];
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int t = 0; t < 8; ++t)
            acc[t] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(b[t / 2], a[t % 2], acc[t], 2, 2, 0, 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int t = 0; t < 8; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[t][r];
    if (s == -1.f) sink[0] = 1;  // practically never true; keeps the loop alive
}

constexpr int kMfmaBlocks = 256 * 2;  // two 4-wave workgroups per compute unit

}  // namespace

extern "C" {

int dvdq_bench_copy(const void *src, void *dst, size_t bytes, void *hip_stream) {
    if (!src || !dst) return DVDQ_ERR_NULL;
    if (bytes == 0 || (bytes % 16) != 0) return DVDQ_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(src) & 15u) || (reinterpret_cast<uintptr_t>(dst) & 15u)) return DVDQ_ERR_ALIGN;
    const size_t n = bytes / 16;
    size_t blocks = (n + 256 * kCopyUnroll - 1) / (256 * kCopyUnroll);
    if (blocks > 256 * 8) blocks = 256 * 8;   // 8 resident workgroups per compute unit stride over the buffer
    hipLaunchKernelGGL(copy_kernel, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                       static_cast<const v4u *>(src), static_cast<v4u *>(dst), n);
    return dvdq::check_launch();
}

int dvdq_bench_mfma_i8(int iters, int data, int32_t *sink, double *ops_out, void *hip_stream) {
    if (!sink) return DVDQ_ERR_NULL;
    if (iters < 1) return DVDQ_ERR_SHAPE;
    if (data < 0 || data > 1) return DVDQ_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(mfma_i8_kernel, dim3(kMfmaBlocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream), iters,
                       data, sink);
    if (ops_out) *ops_out = 2.0 * 32 * 32 * 32 * 16.0 * iters * 4.0 * kMfmaBlocks;
    return dvdq::check_launch();
}

int dvdq_bench_mfma_fp6(int iters, int data, int32_t *sink, double *ops_out, void *hip_stream) {
    if (!sink) return DVDQ_ERR_NULL;
    if (iters < 1) return DVDQ_ERR_SHAPE;
    if (data < 0 || data > 1) return DVDQ_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(mfma_fp6_kernel, dim3(kMfmaBlocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream), iters,
                       data, sink);
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

int dvdq_bench_set_gemm_grid_limit(int workgroups) {
    if (workgroups < 0) return DVDQ_ERR_UNSUPPORTED;
    dvdq::set_gemm_grid_limit(workgroups);
    return DVDQ_OK;
}

int dvdq_bench_fill_tile_counters(uint32_t value, void *hip_stream) {
    return dvdq::fill_sched_slots(value, static_cast<hipStream_t>(hip_stream));
}

}  // extern "C"

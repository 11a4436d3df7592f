// delta-Guided Bit Switching (Sec. 3.3): the relative L1 change between successive model
// outputs, L1(F, t) = ||F_t - F_{t-1}||_1 / ||F_{t-1}||_1, and the controller update that
// turns the running sum of these changes into the activation bit-width of the next
// denoising step.  Two launches, no atomics, fixed summation order (bit-reproducible):
//   1. HBM-bound partial sums: every thread reads 16 bytes of each tensor per step,
//      accumulates |a - b| and |b| in fp32, workgroups reduce and write fp64 partials;
//   2. one wave adds the partials in fp64, forms the ratio and updates the state.
#include "dvdq_internal.h"

namespace dvdq {
namespace {

constexpr int kThreads = 256;
constexpr int kMaxBlocks = 1024;   // partial-sum slots in the workspace

struct GbsState {      // 16 bytes in device memory, layout documented in dvdq.h
    double acc;        // running sum of relative L1 changes since the last reset
    float last_l1;     // the change computed by the latest step (for logging)
    int32_t bits;      // activation bit-width for the next denoising step
};

__device__ __forceinline__ void accum8(const uint4 a, const uint4 b, float &num, float &den) {
    const uint32_t aw[4] = {a.x, a.y, a.z, a.w}, bw[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float a0 = __uint_as_float(aw[i] << 16), a1 = __uint_as_float(aw[i] & 0xFFFF0000u);
        const float b0 = __uint_as_float(bw[i] << 16), b1 = __uint_as_float(bw[i] & 0xFFFF0000u);
        num += fabsf(a0 - b0) + fabsf(a1 - b1);
        den += fabsf(b0) + fabsf(b1);
    }
}

__global__ __launch_bounds__(kThreads) void gbs_partial_kernel(const uint16_t *__restrict__ ft,
                                                               const uint16_t *__restrict__ fp, int64_t n,
                                                               double *__restrict__ partial) {
    __shared__ float s_num[kThreads / 64], s_den[kThreads / 64];
    const int64_t nvec = n / 8;
    const uint4 *a = reinterpret_cast<const uint4 *>(ft), *b = reinterpret_cast<const uint4 *>(fp);
    float num = 0.f, den = 0.f;
    const int64_t stride = (int64_t)gridDim.x * kThreads;
    int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    // two independent loads in flight per tensor
    for (; i + stride < nvec; i += 2 * stride) {
        const uint4 a0 = a[i], b0 = b[i], a1 = a[i + stride], b1 = b[i + stride];
        accum8(a0, b0, num, den);
        accum8(a1, b1, num, den);
    }
    if (i < nvec) accum8(a[i], b[i], num, den);
    if (blockIdx.x == 0 && threadIdx.x == 0) {   // ragged tail of fewer than 8 elements
        for (int64_t e = nvec * 8; e < n; ++e) {
            const float x = __uint_as_float((uint32_t)ft[e] << 16), y = __uint_as_float((uint32_t)fp[e] << 16);
            num += fabsf(x - y);
            den += fabsf(y);
        }
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
        num += __shfl_xor(num, m, 64);
        den += __shfl_xor(den, m, 64);
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) { s_num[wave] = num; s_den[wave] = den; }
    __syncthreads();
    if (threadIdx.x == 0) {
        double dn = 0.0, dd = 0.0;
        for (int w = 0; w < kThreads / 64; ++w) { dn += (double)s_num[w]; dd += (double)s_den[w]; }
        partial[2 * blockIdx.x] = dn;
        partial[2 * blockIdx.x + 1] = dd;
    }
}

__global__ __launch_bounds__(64) void gbs_update_kernel(const double *__restrict__ partial, int blocks, double delta,
                                                        int b_low, int b_high, GbsState *state) {
    double num = 0.0, den = 0.0;
    for (int i = threadIdx.x; i < blocks; i += 64) { num += partial[2 * i]; den += partial[2 * i + 1]; }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
        num += __shfl_xor(num, m, 64);
        den += __shfl_xor(den, m, 64);
    }
    if (threadIdx.x == 0) {
        const double l1 = den > 0.0 ? num / den : (num > 0.0 ? (double)INFINITY : 0.0);
        double acc = state->acc + l1;
        int bits = b_low;
        if (acc >= delta) { acc = 0.0; bits = b_high; }   // the sum reached the threshold: high precision, restart
        state->acc = acc;
        state->last_l1 = (float)l1;
        state->bits = bits;
    }
}

__global__ void gbs_reset_kernel(GbsState *state, int bits) {
    state->acc = 0.0;
    state->last_l1 = 0.f;
    state->bits = bits;
}

}  // namespace

size_t gbs_workspace_bytes() { return sizeof(double) * 2 * kMaxBlocks; }

int launch_gbs_reset(void *state, int bits, hipStream_t stream) {
    hipLaunchKernelGGL(gbs_reset_kernel, dim3(1), dim3(1), 0, stream, static_cast<GbsState *>(state), bits);
    return check_launch();
}

int launch_gbs_step(const uint16_t *ft, const uint16_t *fp, int64_t n, double delta, int b_low, int b_high,
                    void *state, void *workspace, hipStream_t stream) {
    int64_t blocks = (n / 8 + kThreads - 1) / kThreads;
    if (blocks < 1) blocks = 1;
    if (blocks > kMaxBlocks) blocks = kMaxBlocks;
    double *partial = static_cast<double *>(workspace);
    hipLaunchKernelGGL(gbs_partial_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, stream, ft, fp, n, partial);
    int rc = check_launch();
    if (rc != DVDQ_OK) return rc;
    hipLaunchKernelGGL(gbs_update_kernel, dim3(1), dim3(64), 0, stream, partial, (int)blocks, delta, b_low, b_high,
                       static_cast<GbsState *>(state));
    return check_launch();
}

}  // namespace dvdq

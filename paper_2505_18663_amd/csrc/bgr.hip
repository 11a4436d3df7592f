// Bounded-init Grid Refinement (Sec. 3.1, Alg. 1): the offline INT4 weight quantizer.
// For every weight row (output channel) it searches clipped MinMax starts, refines each
// start's grid (least-squares step size, relaxed zero-point, re-quantization) round after
// round, and keeps the grid with the smallest row error: either as Alg. 1 prints it (starts
// i = 1, 2, ..., a start's result is the grid of its last round) or as a superset search (i = 0,
// plain MinMax, is a start too and every grid evaluated competes).  Runs once per layer, off the
// inference path; everything is fp64 so that its decisions (roundings, comparisons) match a
// plain fp64 implementation up to summation order.
//
// One workgroup per row.  The row lives in LDS as fp32; one "evaluation" of a grid
// (Delta, z) is a pass over the row that quantizes every weight and accumulates, in fp64,
//   e2  = sum (w - Delta (q - z))^2        the squared row error
//   num = sum (q - z) w,  den = sum (q - z)^2,  sq = sum q
// i.e. also the sums the NEXT refinement round needs, so the codes are never stored until
// the best grid is known.  All threads then run the same scalar search logic on the reduced
// sums (uniform control flow, no divergence in the barriers).
#include "dvdq_internal.h"

#pragma clang fp contract(off)   // every product and sum rounded on its own, like a plain C loop

namespace dvdq {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr double kQmax = 15.0;   // INT4
constexpr size_t kMaxK = 32768;  // longest row (the row is kept in LDS); the C ABI checks it

struct Sums { double e2, num, den, sq; };

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) v += __shfl_xor(v, m, 64);
    return v;
}

// sum of `v` over the workgroup, returned to every thread; `slots` holds kWaves doubles
__device__ __forceinline__ double block_sum(double v, double *slots) {
    v = wave_sum(v);
    __syncthreads();   // the previous use of the slots is over
    if ((threadIdx.x & 63) == 0) slots[threadIdx.x >> 6] = v;
    __syncthreads();
    double s = 0.0;
#pragma unroll
    for (int i = 0; i < kWaves; ++i) s += slots[i];
    return s;
}

__device__ __forceinline__ double clamp_d(double v, double lo, double hi) { return v < lo ? lo : (v > hi ? hi : v); }

// quantize the row on the grid (delta, z) and reduce the four sums
__device__ __forceinline__ Sums evaluate(const float *row, int K, double delta, double z, double *slots) {
    Sums s = {0.0, 0.0, 0.0, 0.0};
    for (int k = threadIdx.x; k < K; k += kThreads) {
        const double w = (double)row[k];
        const double c = clamp_d(rint(w / delta) + z, 0.0, kQmax);   // rint: ties to even
        const double d = c - z;
        const double r = w - delta * d;
        s.e2 += r * r;
        s.num += d * w;
        s.den += d * d;
        s.sq += c;
    }
    s.e2 = block_sum(s.e2, slots);
    s.num = block_sum(s.num, slots);
    s.den = block_sum(s.den, slots);
    s.sq = block_sum(s.sq, slots);
    return s;
}

__global__ __launch_bounds__(kThreads) void bgr_kernel(const float *__restrict__ w, int K, int n_steps, int max_refine,
                                                       double eps, int search, uint8_t *__restrict__ w_packed,
                                                       float *__restrict__ w_scale, int8_t *__restrict__ w_zero,
                                                       double *__restrict__ row_error) {
    extern __shared__ __align__(16) uint8_t smem_raw[];
    double *slots = reinterpret_cast<double *>(smem_raw);            // kWaves doubles
    float *row = reinterpret_cast<float *>(smem_raw + kWaves * sizeof(double));
    const int64_t n = blockIdx.x;
    const float *src = w + n * K;

    // the row into LDS; its minimum, maximum and sum
    double lo0 = INFINITY, hi0 = -INFINITY, sw = 0.0;
    for (int k = threadIdx.x; k < K; k += kThreads) {
        const float v = src[k];
        row[k] = v;
        lo0 = fmin(lo0, (double)v);
        hi0 = fmax(hi0, (double)v);
        sw += (double)v;
    }
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
        lo0 = fmin(lo0, __shfl_xor(lo0, m, 64));
        hi0 = fmax(hi0, __shfl_xor(hi0, m, 64));
    }
    __shared__ double s_lo[kWaves], s_hi[kWaves];
    if ((threadIdx.x & 63) == 0) { s_lo[threadIdx.x >> 6] = lo0; s_hi[threadIdx.x >> 6] = hi0; }
    sw = block_sum(sw, slots);   // (its barriers also publish s_lo / s_hi and the row)
#pragma unroll
    for (int i = 0; i < kWaves; ++i) { lo0 = fmin(lo0, s_lo[i]); hi0 = fmax(hi0, s_hi[i]); }

    double best = INFINITY, best_delta = 1.0, best_z = 0.0;
    if (!(hi0 > lo0)) {
        // constant row c, represented exactly: Delta = |c| (1 if c = 0), z = (c < 0), q = (c > 0)
        best = 0.0;
        best_delta = lo0 == 0.0 ? 1.0 : fabs(lo0);
        best_z = lo0 < 0.0 ? 1.0 : 0.0;
    } else {
        const double step = (hi0 - lo0) / (double)n_steps;
        const bool all = search == DVDQ_BGR_BEST_OF_ALL;
        for (int i = all ? 0 : 1; i <= n_steps; ++i) {
            const double lo = lo0 + (double)i * step, hi = hi0 - (double)i * step;
            if (!(lo < hi)) break;   // the range has collapsed (from i = n_steps / 2 on)
            // clipped MinMax start
            double delta = (hi - lo) / kQmax;
            double z = clamp_d(rint(-(lo / delta)), 0.0, kQmax);
            Sums s = evaluate(row, K, delta, z, slots);
            double e = sqrt(s.e2);
            if (all && e < best) { best = e; best_delta = delta; best_z = z; }
            for (int j = 0; j < max_refine; ++j) {
                if (s.den == 0.0) break;
                const double dn = s.num / s.den;
                if (!(dn > 0.0)) break;
                const double zn = clamp_d(rint(s.sq / (double)K - (sw / (double)K) / dn), 0.0, kQmax);
                s = evaluate(row, K, dn, zn, slots);
                const double en = sqrt(s.e2);
                if (all && en < best) { best = en; best_delta = dn; best_z = zn; }
                const double gain = e - en;
                e = en; delta = dn; z = zn;   // the start's current (last) grid
                if (gain < eps) break;
            }
            // as printed in Alg. 1: only the grid of the start's last round competes
            if (!all && e < best) { best = e; best_delta = delta; best_z = z; }
        }
    }

    // the codes on the best grid, as signed nibbles (unsigned code - 8), two per byte
    const bool constant = !(hi0 > lo0);
    for (int p = threadIdx.x; p < K / 2; p += kThreads) {
        int c[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const double wv = (double)row[2 * p + h];
            const double q = constant ? (lo0 > 0.0 ? 1.0 : 0.0) : clamp_d(rint(wv / best_delta) + best_z, 0.0, kQmax);
            c[h] = (int)q - 8;
        }
        w_packed[n * (K / 2) + p] = (uint8_t)((c[0] & 0xF) | ((c[1] & 0xF) << 4));
    }
    if (threadIdx.x == 0) {
        w_scale[n] = (float)best_delta;
        w_zero[n] = (int8_t)((int)best_z - 8);
        if (row_error) row_error[n] = best;
    }
}

}  // namespace

int launch_bgr(const float *w, int64_t N, int64_t K, int n_steps, int max_refine, double eps, int search,
               uint8_t *w_packed, float *w_scale, int8_t *w_zero, double *row_error, hipStream_t stream) {
    const size_t smem = kWaves * sizeof(double) + (size_t)K * sizeof(float);
    static std::atomic<uint64_t> configured{0};
    allow_dynamic_lds(reinterpret_cast<const void *>(bgr_kernel), kWaves * sizeof(double) + kMaxK * sizeof(float),
                      configured);   // the limit for the longest row the API admits
    hipLaunchKernelGGL(bgr_kernel, dim3((unsigned)N), dim3(kThreads), smem, stream, w, (int)K, n_steps, max_refine, eps,
                       search, w_packed, w_scale, w_zero, row_error);
    return check_launch();
}

}  // namespace dvdq

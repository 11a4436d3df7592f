// W4Ax GEMM, generic path for weights in the canonical [N, K/2] layout: int8
// activation codes x packed INT4 weights on the INT8 matrix cores, exact int32
// accumulation, dequantizing epilogue to bf16 (Sec. 3.2: Y = X^ Lambda W^^T;
// Sec. 3.1 DeQuant with zero-point 0).  The fast path for pre-packed weights
// lives in w4ax_gemm.hip; this one trades speed for taking the weights as they
// come out of an offline quantizer.
//
// Weight nibbles are widened to int8 lanes holding 16*code (mask / shift-by-4 of the
// packed word: the nibble lands in the top half of its byte with the right sign), so
// the MFMA accumulates 16*acc exactly; the factor is removed by an arithmetic shift
// before the accumulator is exposed or scaled.  |16 * acc| <= 16 * 127 * 8 * K must
// stay below 2^31, which the API layer checks.
//
// Tiling: a workgroup of 4 waves (2 x 2) computes a BM x BN tile of Y; each wave a
// (BM/2) x (BN/2) sub-tile out of 32x32x32 MFMAs.  The weight tile is the MFMA's
// row operand and the code tile its column operand, so a lane ends up with 4
// consecutive output channels of one token: one 8-byte bf16 store.  K is consumed in
// slices of 64 through double-buffered LDS; global loads for slice t+1 are in flight
// while slice t is multiplied.  LDS rows are 64 bytes with the 16-byte chunk index
// xor-ed by (row >> 1) & 3 so that 8 consecutive rows hit distinct bank groups.
#include "dvdq_internal.h"

namespace dvdq {
namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kBK = 64;  // K slice per main-loop step (bytes of int8 codes)

// 64-byte rows: four rows share a quarter of the 64 LDS banks; a 16-byte read serves 16 rows at a time
__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ ((row >> 2) & 3); }

// 8 packed nibbles (nibble i = channel i) -> two dwords of int8 lanes (16*code),
// channels in natural order: interleave the bytes of the even and odd nibbles.
__device__ __forceinline__ void widen8(uint32_t p, uint32_t &d0, uint32_t &d1) {
    const uint32_t lo = (p << 4) & 0xF0F0F0F0u;  // nibbles 0,2,4,6
    const uint32_t hi = p & 0xF0F0F0F0u;         // nibbles 1,3,5,7
    d0 = __builtin_amdgcn_perm(hi, lo, 0x05010400u);
    d1 = __builtin_amdgcn_perm(hi, lo, 0x07030602u);
}

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
    typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
    v2bf p = {(__bf16)a, (__bf16)b};  // round-to-nearest-even conversions
    return __builtin_bit_cast(uint32_t, p);
}

template <int BM, int BN>
__global__ __launch_bounds__(256) void w4ax_gemm_canonical_kernel(
    const int8_t *__restrict__ codes, const float *__restrict__ x_scale, const uint8_t *__restrict__ w,
    const float *__restrict__ w_scale, const uint16_t *__restrict__ bias, int M, int N, int K,
    uint16_t *__restrict__ y, int32_t *__restrict__ acc_out, int tiles_m, int tiles_n) {
    constexpr int WM = BM / 2, WN = BN / 2;      // wave sub-tile
    constexpr int TM = WM / 32, TN = WN / 32;    // MFMA tiles per wave
    constexpr int A_LOADS = BM * kBK / 16 / 256; // 16-byte code loads per thread per slice
    constexpr int W_LOADS = BN * (kBK / 2) / 16 / 256;
    static_assert(A_LOADS >= 1 && W_LOADS >= 1, "tile too small for 256 threads");

    extern __shared__ __align__(16) uint8_t smem[];
    uint8_t *sA = smem;                       // [2][BM][64]
    uint8_t *sW = smem + 2 * BM * kBK;        // [2][BN][64]

    // XCD-aware tile order: consecutive workgroup ids land on different XCDs, so give
    // each XCD one contiguous range of tiles (they share code panels in that XCD's L2).
    const int total = tiles_m * tiles_n;
    int tile = blockIdx.x;
    const int per_xcd = total / 8;
    if (tile < per_xcd * 8) tile = (tile % 8) * per_xcd + tile / 8;
    const int tile_m = tile / tiles_n, tile_n = tile - tile_m * tiles_n;
    const int m0 = tile_m * BM, n0 = tile_n * BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = (wave & 1) * WM, wn = (wave >> 1) * WN;

    // global -> register staging
    uint4 ra[A_LOADS], rw[W_LOADS];
    // K is a multiple of 32: the last slice may be half a slice, whose missing channels are zero codes and
    // zero weights (they add nothing to the exact integer sums)
    const int KT = (K + kBK - 1) / kBK;
    auto load_slice = [&](int kt) {
#pragma unroll
        for (int i = 0; i < A_LOADS; ++i) {
            const int idx = tid + i * 256, row = idx >> 2, chunk = idx & 3;
            const int gm = min(m0 + row, M - 1);
            const int k = kt * kBK + chunk * 16;
            ra[i] = k < K ? *reinterpret_cast<const uint4 *>(codes + (int64_t)gm * K + k) : make_uint4(0, 0, 0, 0);
        }
#pragma unroll
        for (int i = 0; i < W_LOADS; ++i) {
            const int idx = tid + i * 256, row = idx >> 1, half = idx & 1;
            const int gn = min(n0 + row, N - 1);
            const int k = kt * kBK + half * 32;
            rw[i] = k < K ? *reinterpret_cast<const uint4 *>(w + (int64_t)gn * (K / 2) + k / 2) : make_uint4(0, 0, 0, 0);
        }
    };
    auto store_slice = [&](int buf) {
        uint8_t *a = sA + buf * BM * kBK, *b = sW + buf * BN * kBK;
#pragma unroll
        for (int i = 0; i < A_LOADS; ++i) {
            const int idx = tid + i * 256, row = idx >> 2, chunk = idx & 3;
            *reinterpret_cast<uint4 *>(a + row * kBK + swz(row, chunk) * 16) = ra[i];
        }
#pragma unroll
        for (int i = 0; i < W_LOADS; ++i) {
            const int idx = tid + i * 256, row = idx >> 1, half = idx & 1;
            uint4 c0, c1;
            widen8(rw[i].x, c0.x, c0.y);
            widen8(rw[i].y, c0.z, c0.w);
            widen8(rw[i].z, c1.x, c1.y);
            widen8(rw[i].w, c1.z, c1.w);
            *reinterpret_cast<uint4 *>(b + row * kBK + swz(row, 2 * half) * 16) = c0;
            *reinterpret_cast<uint4 *>(b + row * kBK + swz(row, 2 * half + 1) * 16) = c1;
        }
    };

    v16i acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    load_slice(0);
    store_slice(0);
    __syncthreads();

    const int frow = lane & 31, fchunk = lane >> 5;  // fragment row / 16-byte half within a K=32 step
    for (int kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < KT) load_slice(kt + 1);
        const uint8_t *a = sA + buf * BM * kBK, *b = sW + buf * BN * kBK;
#pragma unroll
        for (int ks = 0; ks < kBK / 32; ++ks) {
            v4i fa[TM], fw[TN];
#pragma unroll
            for (int j = 0; j < TM; ++j) {
                const int row = wm + j * 32 + frow;
                fa[j] = *reinterpret_cast<const v4i *>(a + row * kBK + swz(row, ks * 2 + fchunk) * 16);
            }
#pragma unroll
            for (int i = 0; i < TN; ++i) {
                const int row = wn + i * 32 + frow;
                fw[i] = *reinterpret_cast<const v4i *>(b + row * kBK + swz(row, ks * 2 + fchunk) * 16);
            }
#pragma unroll
            for (int i = 0; i < TN; ++i)
#pragma unroll
                for (int j = 0; j < TM; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fw[i], fa[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < KT) store_slice(buf ^ 1);
        __syncthreads();
    }

    // Epilogue.  Accumulator register r of MFMA tile (i, j) in lane l is
    //   n = n0 + wn + 32 i + 8 (r / 4) + 4 (l / 32) + (r % 4),   m = m0 + wm + 32 j + (l % 32).
    const bool vec_ok = (N & 3) == 0;
#pragma unroll
    for (int j = 0; j < TM; ++j) {
        const int m = m0 + wm + j * 32 + (lane & 31);
        if (m >= M) continue;
        const float xs = x_scale[m];
#pragma unroll
        for (int i = 0; i < TN; ++i) {
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const int n = n0 + wn + i * 32 + g * 8 + (lane >> 5) * 4;
                if (n >= N) continue;
                int a4[4];
#pragma unroll
                for (int r = 0; r < 4; ++r) a4[r] = acc[i][j][g * 4 + r] >> 4;  // exact: low 4 bits are zero
                if (vec_ok) {  // n + 3 < N because N % 4 == 0 and n % 4 == 0
                    const float4 ws = *reinterpret_cast<const float4 *>(w_scale + n);
                    float o[4] = {(float)a4[0] * xs * ws.x, (float)a4[1] * xs * ws.y, (float)a4[2] * xs * ws.z,
                                  (float)a4[3] * xs * ws.w};
                    if (bias) {
                        const uint2 bb = *reinterpret_cast<const uint2 *>(bias + n);
                        o[0] += __uint_as_float(bb.x << 16);
                        o[1] += __uint_as_float(bb.x & 0xFFFF0000u);
                        o[2] += __uint_as_float(bb.y << 16);
                        o[3] += __uint_as_float(bb.y & 0xFFFF0000u);
                    }
                    uint2 out;
                    out.x = pack_bf16x2(o[0], o[1]);
                    out.y = pack_bf16x2(o[2], o[3]);
                    *reinterpret_cast<uint2 *>(y + (int64_t)m * N + n) = out;
                    if (acc_out)
                        *reinterpret_cast<int4 *>(acc_out + (int64_t)m * N + n) = make_int4(a4[0], a4[1], a4[2], a4[3]);
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        if (n + r >= N) break;
                        float o = (float)a4[r] * xs * w_scale[n + r];
                        if (bias) o += __uint_as_float((uint32_t)bias[n + r] << 16);
                        y[(int64_t)m * N + n + r] = (uint16_t)(pack_bf16x2(o, 0.f) & 0xFFFFu);
                        if (acc_out) acc_out[(int64_t)m * N + n + r] = a4[r];
                    }
                }
            }
        }
    }
}

template <int BM, int BN>
int launch_tile(const int8_t *codes, const float *x_scale, const uint8_t *w, const float *w_scale,
                const uint16_t *bias, int M, int N, int K, uint16_t *y, int32_t *acc_out, hipStream_t stream) {
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const size_t smem = 2 * (size_t)(BM + BN) * kBK;
    const dim3 grid((unsigned)(tiles_m * tiles_n)), block(256);
    auto k = w4ax_gemm_canonical_kernel<BM, BN>;
    static std::atomic<uint64_t> configured{0};   // one per template instantiation
    allow_dynamic_lds(reinterpret_cast<const void *>(k), smem, configured);
    hipLaunchKernelGGL(k, grid, block, smem, stream, codes, x_scale, w, w_scale, bias, M, N, K, y, acc_out, tiles_m,
                       tiles_n);
    return check_launch();
}

}  // namespace

int launch_w4ax_gemm_canonical(const int8_t *codes, const float *x_scale, const uint8_t *w, const float *w_scale,
                               const uint16_t *bias, int64_t M, int64_t N, int64_t K, uint16_t *y, int32_t *acc_out,
                               hipStream_t stream) {
    return launch_tile<256, 256>(codes, x_scale, w, w_scale, bias, (int)M, (int)N, (int)K, y, acc_out, stream);
}

}  // namespace dvdq

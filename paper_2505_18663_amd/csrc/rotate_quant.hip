// Rotate + auto-scale + quantize for gfx950 (Sec. 3.2: X~ = XH by fast Hadamard
// transform; s = ||x~||_inf / qmax per token row; codes = round-half-even(x~ / s)).
//
// One pass over HBM: a token row is read once (bf16), kept in registers while the
// transform, the row abs-max and the quantizer run, and written once (int8 codes +
// one fp32 scale).  The kernel is bound by HBM only if the transform is cheap in
// VALU instructions, so the 9 butterfly stages of a 512-channel unit are split:
//
//   * channel-index bits 0..4 (strides 1..16) go through the matrix cores: the lane's
//     8 raw bf16 values are the B operand of two 16x16x32 bf16 MFMAs whose A operand
//     is a constant +-1 / 0 matrix (H_32, or I (x) H_2^b for smaller blocks).  The
//     products are exact and the sums are accumulated in fp32.  No bf16 -> fp32
//     unpacking is needed and the result lands in the same lane, same order.
//   * bits 5..8 (strides 32..256) are butterflies between lanes, on fp32 values, with
//     DPP row operations.  The 16-byte chunks of a unit are dealt to lanes so that
//     bits 5, 6, 7 pair lanes l ^ 1, l ^ 2, l ^ 8 (single DPP operations) and bit 8,
//     which only 512-blocks transform, pairs l ^ 4 (two masked row shifts).
//
// Chunk c (16 bytes = 8 channels) of a unit belongs to lane
//   l = (c & 3) << 4 | (c >> 2 & 1) | (c >> 3 & 1) << 1 | (c >> 5 & 1) << 2 | (c >> 4 & 1) << 3,
// i.e. lanes l, l+16, l+32, l+48 hold 64 contiguous bytes and a wave instruction still
// covers one contiguous kilobyte.  Rows longer than a few units are spread over the
// waves of a workgroup and the abs-max is combined through LDS.  The 1/sqrt(B)
// normalization is never applied to the data: it is folded into the scale and into
// the reciprocal the codes are taken with.
#include "dvdq_internal.h"

namespace dvdq {
namespace {

constexpr int kWave = 64;
constexpr int kUnit = 512;  // channels a wave handles per step (64 lanes x 8)

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));

template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

// value of lane (l ^ 4): rows shifted left by 4 for the lanes with bit 2 clear (banks 0 and 2),
// right by 4 for the others (banks 1 and 3)
__device__ __forceinline__ float dpp_xor4(float v) {
    const int x = __builtin_bit_cast(int, v);
    int t = __builtin_amdgcn_update_dpp(0, x, 0x104 /* row_shl:4 */, 0xF, 0x5, false);
    t = __builtin_amdgcn_update_dpp(t, x, 0x114 /* row_shr:4 */, 0xF, 0xA, false);
    return __builtin_bit_cast(float, t);
}

// entry (r, k) of the 32 x 32 matrix that applies H to the index bits in `mask` and the
// identity to the others, as a bf16 bit pattern (+1, -1 or 0)
__device__ __forceinline__ uint32_t had5_bf16(int r, int k, int mask) {
    if ((r ^ k) & ~mask & 31) return 0u;
    return (__builtin_popcount(r & k & mask) & 1) ? 0xBF80u : 0x3F80u;
}

// CPW = units per wave.  waves_per_row (W) waves share a row; unit u of the row
// belongs to wave (u % W) as its (u / W)-th unit.
template <int LOG2B, int CPW>
__global__ __launch_bounds__(1024) void rotate_quant_kernel(
    const uint16_t *__restrict__ x, int64_t M, int K, int waves_per_row, int rows_per_wg,
    double scale_mul,  // 1 / (sqrt(B) * qmax); fp64 so the fp32 scale is rounded once
    float recip_num,   // 1 / sqrt(B)
    int8_t *__restrict__ codes, float *__restrict__ x_scale) {
    extern __shared__ float s_amax[];  // [rows_per_wg * waves_per_row]
    constexpr int MASK5 = LOG2B >= 5 ? 31 : ((1 << LOG2B) - 1);
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int row_in_wg = wave / waves_per_row;
    const int wsub = wave - row_in_wg * waves_per_row;
    const int64_t row = (int64_t)blockIdx.x * rows_per_wg + row_in_wg;
    const bool row_ok = row < M;
    // this lane's 16-byte chunk within a unit
    const int chunk = ((lane >> 4) & 3) | ((lane & 1) << 2) | (((lane >> 1) & 1) << 3) | (((lane >> 3) & 1) << 4) |
                      (((lane >> 2) & 1) << 5);

    // constant MFMA operands: rows r = 8 (m / 4) + 4 h + (m % 4) of the 32 x 32 transform, m = lane % 16,
    // columns k = 8 (lane / 16) + t.  MFMA h then yields transformed channels 4h .. 4h+3 of this lane's chunk.
    bf16x8 tmat[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const int m = lane & 15, r = 8 * (m >> 2) + 4 * h + (m & 3);
        uint32_t w[4];
#pragma unroll
        for (int t = 0; t < 8; t += 2) {
            const int k = 8 * (lane >> 4) + t;
            w[t / 2] = had5_bf16(r, k, MASK5) | (had5_bf16(r, k + 1, MASK5) << 16);
        }
        tmat[h] = __builtin_bit_cast(bf16x8, make_uint4(w[0], w[1], w[2], w[3]));
    }
    // butterfly signs of the lane-pairing stages: the lane with the stage's bit set takes (partner - own)
    const float s1 = (lane & 1) ? -1.f : 1.f, s2 = (lane & 2) ? -1.f : 1.f;
    const float s8 = (lane & 8) ? -1.f : 1.f, s4 = (lane & 4) ? -1.f : 1.f;

    float v[CPW][8];
    float amax = 0.f;
#pragma unroll
    for (int c = 0; c < CPW; ++c) {
        const int k0 = (wsub + c * waves_per_row) * kUnit + chunk * 8;
        uint4 raw = make_uint4(0, 0, 0, 0);
        if (row_ok && k0 < K) raw = *reinterpret_cast<const uint4 *>(x + row * K + k0);
        if (LOG2B == 0) {
            const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                v[c][2 * i] = __uint_as_float(w[i] << 16);
                v[c][2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
            }
        } else {
            const bf16x8 data = __builtin_bit_cast(bf16x8, raw);
            const v4f zero = {0.f, 0.f, 0.f, 0.f};
            const v4f d0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(tmat[0], data, zero, 0, 0, 0);
            const v4f d1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(tmat[1], data, zero, 0, 0, 0);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                v[c][i] = d0[i];
                v[c][4 + i] = d1[i];
            }
        }
    }
#pragma unroll
    for (int c = 0; c < CPW; ++c) {
        if (LOG2B >= 6) {
#pragma unroll
            for (int i = 0; i < 8; ++i) v[c][i] = fmaf(v[c][i], s1, dpp_mov<0xB1>(v[c][i]));  // quad_perm [1,0,3,2]
        }
        if (LOG2B >= 7) {
#pragma unroll
            for (int i = 0; i < 8; ++i) v[c][i] = fmaf(v[c][i], s2, dpp_mov<0x4E>(v[c][i]));  // quad_perm [2,3,0,1]
        }
        if (LOG2B >= 8) {
#pragma unroll
            for (int i = 0; i < 8; ++i) v[c][i] = fmaf(v[c][i], s8, dpp_mov<0x128>(v[c][i]));  // row_ror:8
        }
        if (LOG2B >= 9) {
#pragma unroll
            for (int i = 0; i < 8; ++i) v[c][i] = fmaf(v[c][i], s4, dpp_xor4(v[c][i]));
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf(v[c][i]));
    }
#pragma unroll
    for (int m = 1; m < kWave; m <<= 1) amax = fmaxf(amax, __shfl_xor(amax, m, kWave));
    if (waves_per_row > 1) {
        if (lane == 0) s_amax[wave] = amax;
        __syncthreads();
        amax = 0.f;
        for (int i = 0; i < waves_per_row; ++i) amax = fmaxf(amax, s_amax[row_in_wg * waves_per_row + i]);
    }
    // scale handed on = amax / (sqrt(B) * qmax); codes = rne(v * (1/sqrt(B)) / scale)
    const float scale = (float)((double)amax * scale_mul);
    const float r = scale > 0.f ? recip_num / scale : 0.f;
    if (row_ok && wsub == 0 && lane == 0) x_scale[row] = scale;

    const float magic = 12582912.f;  // 1.5 * 2^23: adding it rounds to integer, ties to even
#pragma unroll
    for (int c = 0; c < CPW; ++c) {
        const int k0 = (wsub + c * waves_per_row) * kUnit + chunk * 8;
        uint32_t b[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) b[i] = __float_as_uint(fmaf(v[c][i], r, magic));
        // low bytes of b[0..3] / b[4..7] -> one dword each
        uint2 out;
        out.x = __builtin_amdgcn_perm(__builtin_amdgcn_perm(b[3], b[2], 0x0c0c0400u),
                                      __builtin_amdgcn_perm(b[1], b[0], 0x0c0c0400u), 0x05040100u);
        out.y = __builtin_amdgcn_perm(__builtin_amdgcn_perm(b[7], b[6], 0x0c0c0400u),
                                      __builtin_amdgcn_perm(b[5], b[4], 0x0c0c0400u), 0x05040100u);
        if (row_ok && k0 < K) *reinterpret_cast<uint2 *>(codes + row * K + k0) = out;
    }
}

template <int LOG2B>
int launch_cpw(int cpw, dim3 grid, dim3 block, size_t smem, hipStream_t stream, const uint16_t *x, int64_t M,
               int K, int W, int rpw, double scale_mul, float recip_num, int8_t *codes, float *x_scale) {
#define DVDQ_RQ_CASE(C)                                                                                   \
    case C:                                                                                               \
        hipLaunchKernelGGL((rotate_quant_kernel<LOG2B, C>), grid, block, smem, stream, x, M, K, W, rpw,   \
                           scale_mul, recip_num, codes, x_scale);                                         \
        break;
    switch (cpw) {
        DVDQ_RQ_CASE(1) DVDQ_RQ_CASE(2) DVDQ_RQ_CASE(3) DVDQ_RQ_CASE(4)
        DVDQ_RQ_CASE(5) DVDQ_RQ_CASE(6) DVDQ_RQ_CASE(7) DVDQ_RQ_CASE(8)
        default: return DVDQ_ERR_UNSUPPORTED;
    }
#undef DVDQ_RQ_CASE
    return check_launch();
}

}  // namespace

int launch_rotate_quant(const uint16_t *x, int64_t M, int64_t K, int log2_block, int act_bits, int8_t *codes,
                        float *x_scale, hipStream_t stream) {
    const int units = (int)((K + kUnit - 1) / kUnit);
    // waves per row: at most 4 units (32 fp32 values per lane) in registers per wave, at most 16 waves
    int W = (units + 3) / 4;
    if (W > 16) W = 16;
    const int cpw = (units + W - 1) / W;
    if (cpw > 8) return DVDQ_ERR_UNSUPPORTED;
    const int rows_per_wg = W >= 4 ? 1 : 4 / W;
    const dim3 block(kWave * W * rows_per_wg);
    const dim3 grid((unsigned)((M + rows_per_wg - 1) / rows_per_wg));
    const size_t smem = sizeof(float) * W * rows_per_wg;
    const double qmax = (double)((1 << (act_bits - 1)) - 1);
    const double norm = 1.0 / sqrt((double)(1 << log2_block));
    const double scale_mul = norm / qmax;
    const float recip_num = (float)norm;
#define DVDQ_RQ_B(L)                                                                                        \
    case L:                                                                                                 \
        return launch_cpw<L>(cpw, grid, block, smem, stream, x, M, (int)K, W, rows_per_wg, scale_mul,       \
                             recip_num, codes, x_scale);
    switch (log2_block) {
        DVDQ_RQ_B(0) DVDQ_RQ_B(1) DVDQ_RQ_B(2) DVDQ_RQ_B(3) DVDQ_RQ_B(4)
        DVDQ_RQ_B(5) DVDQ_RQ_B(6) DVDQ_RQ_B(7) DVDQ_RQ_B(8) DVDQ_RQ_B(9)
    }
#undef DVDQ_RQ_B
    return DVDQ_ERR_UNSUPPORTED;
}

}  // namespace dvdq

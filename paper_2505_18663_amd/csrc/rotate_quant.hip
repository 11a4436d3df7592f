// Rotate + auto-scale + quantize for gfx950 (Sec. 3.2: X~ = XH by fast Hadamard
// transform; s = ||x~||_inf / qmax per token row; codes = round-half-even(x~ / s)).
//
// One pass over HBM: a token row is read once (bf16), kept in registers while the
// butterfly, the row abs-max and the quantizer run, and written once (int8 codes +
// one fp32 scale).  A wave owns 512-channel "units" of a row: lane l holds channels
// 8l..8l+7 of the unit (one 16-byte load), so butterfly strides 1,2,4 are in-lane and
// strides 8..256 pair lane l with lane l ^ (stride/8).  Rows longer than one unit
// per wave are spread over the waves of a workgroup and the abs-max is combined
// through LDS.  The 1/sqrt(B) normalization is never applied to the data: it is
// folded into the scale and into the reciprocal the codes are taken with.
#include "dvdq_internal.h"

namespace dvdq {
namespace {

constexpr int kWave = 64;
constexpr int kUnit = 512;  // channels a wave handles per step (64 lanes x 8)

__device__ __forceinline__ float lane_xor(float v, int lane_mask) {
    return __shfl_xor(v, lane_mask, kWave);
}

template <int LOG2B>
__device__ __forceinline__ void hadamard_unit(float (&v)[8], int lane) {
    // in-lane stages: strides 1, 2, 4
    if (LOG2B >= 1) {
#pragma unroll
        for (int i = 0; i < 8; i += 2) { float a = v[i], b = v[i + 1]; v[i] = a + b; v[i + 1] = a - b; }
    }
    if (LOG2B >= 2) {
#pragma unroll
        for (int i = 0; i < 8; i += 4)
#pragma unroll
            for (int j = 0; j < 2; ++j) { float a = v[i + j], b = v[i + j + 2]; v[i + j] = a + b; v[i + j + 2] = a - b; }
    }
    if (LOG2B >= 3) {
#pragma unroll
        for (int j = 0; j < 4; ++j) { float a = v[j], b = v[j + 4]; v[j] = a + b; v[j + 4] = a - b; }
    }
    // cross-lane stages: channel stride 8 << s  <=>  lane stride 1 << s
#pragma unroll
    for (int s = 0; s < LOG2B - 3; ++s) {
        const int m = 1 << s;
        const bool upper = (lane & m) != 0;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            float p = lane_xor(v[i], m);
            v[i] = upper ? (p - v[i]) : (v[i] + p);
        }
    }
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
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int row_in_wg = wave / waves_per_row;
    const int wsub = wave - row_in_wg * waves_per_row;
    const int64_t row = (int64_t)blockIdx.x * rows_per_wg + row_in_wg;
    const bool row_ok = row < M;

    float v[CPW][8];
    float amax = 0.f;
#pragma unroll
    for (int c = 0; c < CPW; ++c) {
        const int k0 = (wsub + c * waves_per_row) * kUnit + lane * 8;
        uint4 raw = make_uint4(0, 0, 0, 0);
        if (row_ok && k0 < K) raw = *reinterpret_cast<const uint4 *>(x + row * K + k0);
        const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[c][2 * i] = __uint_as_float(w[i] << 16);
            v[c][2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
        }
        hadamard_unit<LOG2B>(v[c], lane);
#pragma unroll
        for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf(v[c][i]));
    }
#pragma unroll
    for (int m = 1; m < kWave; m <<= 1) amax = fmaxf(amax, lane_xor(amax, m));
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
        const int k0 = (wsub + c * waves_per_row) * kUnit + lane * 8;
        uint32_t b[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) b[i] = __float_as_uint(fmaf(v[c][i], r, magic)) & 0xFFu;
        uint2 out;
        out.x = b[0] | (b[1] << 8) | (b[2] << 16) | (b[3] << 24);
        out.y = b[4] | (b[5] << 8) | (b[6] << 16) | (b[7] << 24);
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
    // fewest waves per row that keep at most 4 units (32 fp32 values per lane) in registers
    int W = 1;
    while ((units + W - 1) / W > 4 && W < 16) W *= 2;
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

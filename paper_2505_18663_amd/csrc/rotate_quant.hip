// Rotate + auto-scale + quantize for gfx950 (Sec. 3.2: X~ = XH by fast Hadamard
// transform; s = ||x~||_inf / qmax per token row; codes = round-half-even(x~ / s)).
//
// One pass over HBM: a token row is read once (bf16), kept in registers while the
// transform, the row abs-max and the quantizer run, and written once (int8 codes,
// 4-bit codes packed two per byte, or 4-bit codes as 6-bit E2M3 patterns for the FP6 matrix
// path; one fp32 scale; optionally the row's code sum for weights with zero-points).  A block-wise scaled mode gives every channel group its own
// power-of-two fraction of the token's step and folds it into the int8 value (see the
// quantizer section of the kernel).  The kernel is bound by HBM only if the transform is
// cheap in VALU instructions, so the 9 butterfly stages of a 512-channel unit are split:
//
//   * channel-index bits 0..4 (strides 1..16) go through the matrix cores: the lane's
//     8 raw bf16 values are the B operand of two 16x16x32 bf16 MFMAs whose A operand
//     is a constant +-1 / 0 matrix (H_32, or I (x) H_2^b for smaller blocks).  The
//     products are exact and the sums are accumulated in fp32.  No bf16 -> fp32
//     unpacking is needed and the result lands in the same lane, same order.
//   * bits 5..8 (strides 32..256) are butterflies between lanes, on fp32 values, with
//     DPP row operations: one fused multiply-add with a DPP operand per value and stage.  A 16-lane row
//     has single-operation pairings l ^ 1, l ^ 2 (quad permutes), l ^ 8 (row rotate) and l ^ 7 (half-row
//     mirror), but none for l ^ 4; 1, 2, 8, 7 is a basis of the row's 16 lane numbers all the same, and a
//     transform whose stages pair along a basis is the Hadamard transform in the coordinates over that
//     basis.  So the 16-byte chunks of a unit are dealt to lanes by those coordinates: the lane whose
//     number is u5 * 1 ^ u6 * 2 ^ u7 * 8 ^ u8 * 7 takes the chunk whose channel-index bits 5..8 are
//     u5 .. u8, and the result lands in place.
//
// Chunk c (16 bytes = 8 channels) of a unit belongs to lane
//   l = (c & 3) << 4 | ((c >> 2 & 1) * 1 ^ (c >> 3 & 1) * 2 ^ (c >> 4 & 1) * 8 ^ (c >> 5 & 1) * 7),
// i.e. lanes l, l+16, l+32, l+48 hold 64 contiguous bytes and a wave instruction still
// covers one contiguous kilobyte.  Rows longer than a few units are spread over the
// waves of a workgroup and the abs-max is combined through LDS.  Workgroups stay
// resident and stride over the rows, prefetching the next row while one is processed.
// The 1/sqrt(B) normalization is never applied to the data: it is folded into the
// scale and into the reciprocal the codes are taken with.
#include "dvdq_internal.h"

namespace dvdq {
namespace {

constexpr int kWave = 64;
constexpr int kUnit = 512;  // channels a wave handles per step (64 lanes x 8)
constexpr size_t kLdsPerCu = 160 * 1024;

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float v4f __attribute__((ext_vector_type(4)));

template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v) {
    return __builtin_bit_cast(float, __builtin_amdgcn_mov_dpp(__builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}

// One butterfly stage over a lane pairing with a single DPP operand, 8 values, one
// instruction per value: v = own + sign * partner, sign = +1 in the lane whose stage bit
// is clear and -1 in the other.  The lane with the bit set therefore holds MINUS the
// butterfly's difference; the caller tracks that sign and folds it into the quantizer.
// (The compiler does not fuse a DPP move into an fma, so this is inline assembly.  The
// leading s_nop covers the 2 wait states a DPP read needs after a VALU write of the same
// register.  PRE is put in front of that: the first stage reads registers that an MFMA may have written
// directly, whose longer read-after-write distance the compiler does not see through inline assembly.)
#define DVDQ_FMAC_DPP8(PRE, CTRL)                                                                              \
    asm volatile(PRE "s_nop 1\n\t"                                                                             \
                 "v_fmac_f32_dpp %0, %0, %8 " CTRL " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"              \
                 "v_fmac_f32_dpp %1, %1, %8 " CTRL " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"              \
                 "v_fmac_f32_dpp %2, %2, %8 " CTRL " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"              \
                 "v_fmac_f32_dpp %3, %3, %8 " CTRL " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"              \
                 "v_fmac_f32_dpp %4, %4, %8 " CTRL " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"              \
                 "v_fmac_f32_dpp %5, %5, %8 " CTRL " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"              \
                 "v_fmac_f32_dpp %6, %6, %8 " CTRL " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"              \
                 "v_fmac_f32_dpp %7, %7, %8 " CTRL " row_mask:0xf bank_mask:0xf bound_ctrl:1"                  \
                 : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]), "+v"(v[4]), "+v"(v[5]), "+v"(v[6]), "+v"(v[7]) \
                 : "v"(sign))

// (first of the lane-pairing stages: its values come straight from the 8-pass MFMAs, whose results a vector
// instruction may read 12 wait states after the MFMA issued; 20 are kept)
__device__ __forceinline__ void stage_xor1(float (&v)[8], float sign) { DVDQ_FMAC_DPP8("s_nop 15\n\ts_nop 1\n\t", "quad_perm:[1,0,3,2]"); }
__device__ __forceinline__ void stage_xor2(float (&v)[8], float sign) { DVDQ_FMAC_DPP8("", "quad_perm:[2,3,0,1]"); }
__device__ __forceinline__ void stage_xor8(float (&v)[8], float sign) { DVDQ_FMAC_DPP8("", "row_ror:8"); }

__device__ __forceinline__ void stage_xor7(float (&v)[8], float sign) { DVDQ_FMAC_DPP8("", "row_half_mirror"); }

// Maximum of a non-negative value over the wave, the same in every lane: two quad permutes and two row
// mirrors leave each 16-lane row's maximum in all its lanes, two row broadcasts carry it on into lane 63.
// (Inline assembly: the compiler keeps a move, two canonicalizing maxima and the maximum per step instead of one
// maximum with a DPP operand.  s_nop 1: the 2 wait states between a vector write and a DPP read of a register.)
__device__ __forceinline__ float wave_max(float a) {
    asm volatile("s_nop 1\n\t"
                 "v_max_f32_dpp %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
                 "s_nop 1\n\t"
                 "v_max_f32_dpp %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
                 "s_nop 1\n\t"
                 "v_max_f32_dpp %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0xf\n\t"
                 "s_nop 1\n\t"
                 "v_max_f32_dpp %0, %0, %0 row_mirror row_mask:0xf bank_mask:0xf\n\t"
                 "s_nop 1\n\t"
                 "v_max_f32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"   // into rows 1, 3
                 "s_nop 1\n\t"
                 "v_max_f32_dpp %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf"          // into rows 2, 3
                 : "+v"(a));
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, a), 63));
}

// entry (r, k) of the 32 x 32 matrix that applies H to the index bits in `mask` and the
// identity to the others, as a bf16 bit pattern (+1, -1 or 0)
__device__ __forceinline__ uint32_t had5_bf16(int r, int k, int mask) {
    if ((r ^ k) & ~mask & 31) return 0u;
    return (__builtin_popcount(r & k & mask) & 1) ? 0xBF80u : 0x3F80u;
}

// CPW = units per wave.  waves_per_row (W) waves share a row; unit u of the row
// belongs to wave (u % W) as its (u / W)-th unit.
// FMT: container of the codes: 0 int8, 1 two 4-bit codes per byte, 2 FP6 (E2M3 patterns, block layout).
template <int LOG2B, int CPW, int FMT>
__global__ __launch_bounds__(1024) void rotate_quant_kernel(
    const uint16_t *__restrict__ x, int64_t M, int K, int waves_per_row, int rows_per_wg,
    double scale_mul,  // 1 / (sqrt(B) * qmax); fp64 so the fp32 scale is rounded once
    float recip_num,   // 1 / sqrt(B)
    int via_lds,       // FMT 1: gather the packed codes through LDS into 16-byte stores (K % 32 == 0);
                       // FMT 2: consecutive rows a wave takes in turn before it strides on (8, 4, 2 or 1)
    int group_log2,    // int8 container only: 0, or log2 of the channel group (7, 8, 9) of block-wise scaling
    int emax,          // block-wise scaling: largest power-of-two refinement of a group's step (8 - act_bits)
    int8_t *__restrict__ codes, float *__restrict__ x_scale,
    int32_t *__restrict__ code_rowsum,    // NULL, or [M]: sum of the row's codes (for weight zero-points)
    unsigned *__restrict__ clear_words) { // NULL, or 16 words to zero: the tile counters of the GEMM that follows on the stream
    if (clear_words && blockIdx.x == 0 && threadIdx.x < 16) clear_words[threadIdx.x] = 0u;
    extern __shared__ float s_amax[];  // [2][rows_per_wg * waves_per_row], slots alternate per iteration
    // then [2][rows_per_wg * waves_per_row] per-wave code sums, then, 16-byte aligned,
    // [waves][CPW][64] dwords for gathering packed codes (via_lds), or [waves][rows in turn][CPW * 384 + 16] bytes for FP6
    int32_t *s_sum = reinterpret_cast<int32_t *>(s_amax) + 2 * rows_per_wg * waves_per_row;
    uint32_t *s_pack = reinterpret_cast<uint32_t *>(s_amax) + (4 * rows_per_wg * waves_per_row + 3) / 4 * 4;
    constexpr bool PACK4 = FMT == 1;
    constexpr int MASK5 = LOG2B >= 5 ? 31 : ((1 << LOG2B) - 1);
    const int lane = threadIdx.x & (kWave - 1);
    // (provably wave-uniform, so that row numbers and row base addresses live in scalar registers)
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int row_in_wg = wave / waves_per_row;
    const int wsub = wave - row_in_wg * waves_per_row;
    // this lane's 16-byte chunk within a unit
    // (u5 .. u8: the lane's coordinates over the pairings 1, 2, 8, 7 = channel-index bits 5 .. 8 of its chunk)
    const int u8 = (lane >> 2) & 1, u7 = (lane >> 3) & 1, u6 = ((lane >> 1) & 1) ^ u8, u5 = (lane & 1) ^ u8;
    const int chunk = ((lane >> 4) & 3) | (u5 << 2) | (u6 << 3) | (u7 << 4) | (u8 << 5);

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
    // butterfly signs of the lane-pairing stages (the lane with the stage's bit set takes the difference)
    const float s1 = u5 ? -1.f : 1.f, s2 = u6 ? -1.f : 1.f, s8 = u7 ? -1.f : 1.f, s7 = u8 ? -1.f : 1.f;
    // every stage leaves MINUS the difference in the lane whose coordinate is set
    const float flip = (((LOG2B >= 6) & u5) ^ ((LOG2B >= 7) & u6) ^ ((LOG2B >= 8) & u7) ^ ((LOG2B >= 9) & u8)) ? -1.f : 1.f;

    // channel offsets of this lane's chunks; chunks at or past K are padding (zero in, nothing out)
    int k0[CPW];
#pragma unroll
    for (int c = 0; c < CPW; ++c) k0[c] = (wsub + c * waves_per_row) * kUnit + chunk * 8;

    // Unit c of this wave is unit wsub + c * waves_per_row of the row; only the last one can lie past the row's
    // end (the launcher gives every wave ceil(units / waves) slots).  Wave-uniform: such a wave branches around
    // the slot's work, which keeps the vector work of the SIMDs of a workgroup even when units do not divide.
    const bool last_unit_present = (wsub + (CPW - 1) * waves_per_row) * kUnit < K;
    auto present = [&] __device__(int c) { return c < CPW - 1 || last_unit_present; };

    // A row is read through a buffer descriptor of its own (base = the row, extent = its K bf16 values, or
    // nothing for rows past M): chunks past the end come back as zeros with no branch around the loads, so the
    // compiler can count the loads in flight and wait only for the row it needs while the next one is on its way.
    // X is read exactly once: streaming loads keep it from displacing the codes this kernel writes (and the
    // weights) from the caches the GEMM is about to read them from.
    auto load_row = [&] __device__(uint4 (&raw)[CPW], int64_t row) {
        const bool ok = row < M;
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint16_t *>(x) + (ok ? row : 0) * K, 0, ok ? K * 2 : 0, 0x00020000);
#pragma unroll
        for (int c = 0; c < CPW; ++c) {
            typedef uint32_t v4u __attribute__((ext_vector_type(4)));
            const v4u t = __builtin_amdgcn_raw_buffer_load_b128(rsrc, k0[c] * 2, 0, 2 /* nt */);
            raw[c] = make_uint4(t[0], t[1], t[2], t[3]);
        }
    };

    // Workgroups stride over groups of rows; the next row's loads are in flight while this one is
    // processed.  A group is rows_per_wg rows handled at once, except for the FP6 container: there the
    // waves of a row take `run` consecutive rows in turn (a group is rows_per_wg runs), because the
    // 16-byte chunks of 8 neighbouring rows make up one 128-byte line of that layout; a wave collects
    // its chunks of a run in LDS and writes them as whole lines (16-byte stores scattered over 64 lines
    // per instruction make the whole kernel take twice as long).
    const int run = FMT == 2 ? via_lds : 1;
    // FP6 write-back of a unit's 24 chunks x run rows: item t * 64 + lane is row (lane % run) of the run and
    // chunk part = (t * 64 + lane) / run of the unit, i.e. slice part / 6, piece part % 6; parts >= 24 are idle
    int wb_in[3], wb_out[3], wb_slice[3];
    const int wb_rr = lane & (run - 1);
#pragma unroll
    for (int t = 0; t < 3; ++t) {
        const int part = (t * kWave + lane) >> __builtin_ctz(run);
        wb_slice[t] = part < 24 ? part / 6 : (1 << 30);   // idle: past every row's slices
        wb_in[t] = wb_rr * (CPW * 384 + 16) + part * 16;
        wb_out[t] = (part / 6) * 3072 + (part % 6) * 512 + wb_rr * 16;
    }
    // The workgroup's iterations are numbered (g, turn): turn counts 0 .. run - 1 within group g, and wave row 0
    // takes row (blockIdx.x + g * gridDim.x) * run * rows_per_wg + turn; wave row r is r * run rows further on.
    // (Counted up by hand: a 64-bit division per iteration costs more than a hundred scalar instructions.)
    const int64_t group_stride = (int64_t)gridDim.x * (run * rows_per_wg);
    int64_t group_row = (int64_t)blockIdx.x * (run * rows_per_wg);   // first row of the current group
    int turn = 0;                                                    // turn of the row being processed
    int64_t row = group_row + row_in_wg * run;
    uint4 raw[CPW];
    load_row(raw, row);
    int slot = 0;
    for (int64_t base = group_row; base < M; slot ^= 1) {
        const bool last_turn = turn == run - 1;
        const int64_t next_group_row = last_turn ? group_row + group_stride : group_row;
        const int next_turn = last_turn ? 0 : turn + 1;
        const int64_t next_base = next_group_row + next_turn;
        uint4 nxt[CPW];
        load_row(nxt, next_base + row_in_wg * run);
        const bool row_ok = row < M;

        float v[CPW][8];
        float amax = 0.f;
#pragma unroll
        for (int c = 0; c < CPW; ++c) {
            if (!present(c)) continue;   // (its values are never read)
            if (LOG2B == 0) {
                const uint32_t w[4] = {raw[c].x, raw[c].y, raw[c].z, raw[c].w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    v[c][2 * i] = __uint_as_float(w[i] << 16);
                    v[c][2 * i + 1] = __uint_as_float(w[i] & 0xFFFF0000u);
                }
            } else {
                const bf16x8 data = __builtin_bit_cast(bf16x8, raw[c]);
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
            if (!present(c)) continue;
            if (LOG2B >= 6) stage_xor1(v[c], s1);
            if (LOG2B >= 7) stage_xor2(v[c], s2);
            if (LOG2B >= 8) stage_xor8(v[c], s8);
            if (LOG2B >= 9) stage_xor7(v[c], s7);
#pragma unroll
            for (int i = 0; i < 8; ++i) amax = fmaxf(amax, fabsf(v[c][i]));
        }
        amax = wave_max(amax);
        if (waves_per_row > 1) {
            float *slots = s_amax + slot * (rows_per_wg * waves_per_row);
            if (lane == 0) slots[wave] = amax;
            __syncthreads();
            amax = 0.f;
            for (int i = 0; i < waves_per_row; ++i) amax = fmaxf(amax, slots[row_in_wg * waves_per_row + i]);
        }
        // scale handed on = amax / (sqrt(B) * qmax); codes = rne(v * (1/sqrt(B)) / scale)
        const float scale = (float)((double)amax * scale_mul);
        const float r = scale > 0.f ? flip * (recip_num / scale) : 0.f;
        // (block-wise scaling stores values that carry a factor 2^emax, see below)
        if (row_ok && wsub == 0 && lane == 0) x_scale[row] = group_log2 ? ldexpf(scale, -emax) : scale;

        const float magic = 12582912.f;  // 1.5 * 2^23: adding it rounds to integer, ties to even
        int csum = 0;                    // this lane's share of the row's code sum (padding chunks hold zeros)
        if (FMT == 2) {
            // FP6 container: code c as the E2M3 pattern (c < 0) << 5 | |c|, a lane's 8 fields = 48 bits, made by
            // the chip's packed f32 -> FP6 conversion.  The bytes of the group's rows are put together in LDS in
            // channel order.
            constexpr int TURN_BYTES = CPW * 384 + 16;   // + 16: the 8 turns a quarter-wave reads back sit in different banks
            uint8_t *stage = reinterpret_cast<uint8_t *>(s_pack) + wave * (run * TURN_BYTES);
            uint8_t *sp = stage + turn * TURN_BYTES;
            // q_i = rne(v_i * r) as a float, by the same single-rounding fused multiply-add as the other
            // containers (so that all containers carry identical codes), then the packed conversion: exact
            // integers -7 .. 7 divided by 8 (its scale operand) are E2M3 subnormals m / 8, whose patterns
            // sign << 5 | m are the container's fields.  One conversion takes 32 values, field 2 i from element i
            // of its first source and field 2 i + 1 from element i of its second: four chunks of this lane at a
            // time, chunk g's even channels in elements 4 g .. 4 g + 3 of the first source and its odd channels
            // in those of the second, so that chunk g comes out as bits 48 g .. 48 g + 47.  The instruction
            // reads its sources while it writes its result, so the result must not share registers with them
            // (the early-clobber output; the compiler's own builtin does not keep them apart).
            typedef float v16f __attribute__((ext_vector_type(16)));
            typedef uint32_t v6u __attribute__((ext_vector_type(6)));
            // even chunks sit 4-byte aligned in the turn's bytes and store bytes 0-3 and 4-5, odd chunks (2 mod 4)
            // store bytes 0-1 and 2-5
            uint8_t *d = sp + chunk * 6;
            uint32_t *d_word = reinterpret_cast<uint32_t *>(d + ((chunk & 1) ? 2 : 0));
            uint16_t *d_half = reinterpret_cast<uint16_t *>(d + ((chunk & 1) ? 0 : 4));
            const bool odd = chunk & 1;
            float fsum = 0.f;   // code sums stay exact in fp32: at most 8 * CPW values of magnitude <= 127
#pragma unroll
            for (int c0 = 0; c0 < CPW; c0 += 4) {
                // (elements past the lane's last chunk are don't-cares: left undefined, they cost no instruction)
                const v4f none = {0.f, 0.f, 0.f, 0.f};
                v16f qa = __builtin_shufflevector(none, none, -1, -1, -1, -1, -1, -1, -1, -1, -1, -1, -1, -1, -1, -1, -1, -1);
                v16f qb = qa;
#pragma unroll
                for (int g = 0; g < 4 && c0 + g < CPW; ++g) {
                    if (!present(c0 + g)) continue;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        qa[4 * g + i] = fmaf(v[c0 + g][2 * i], r, magic) - magic;
                        qb[4 * g + i] = fmaf(v[c0 + g][2 * i + 1], r, magic) - magic;
                    }
                }
                if (code_rowsum) {
                    // (the empty volatile statement keeps the additions inside this branch: without it the
                    // compiler adds in every launch and selects afterwards, a tenth of the loop's vector work)
                    asm volatile("" : "+v"(fsum));
#pragma unroll
                    for (int g = 0; g < 4 && c0 + g < CPW; ++g) {
                        if (!present(c0 + g)) continue;
#pragma unroll
                        for (int i = 0; i < 4; ++i) fsum += qa[4 * g + i] + qb[4 * g + i];
                    }
                }
                v6u pk;
                asm volatile("v_cvt_scalef32_2xpk16_fp6_f32 %0, %1, %2, %3\n\ts_nop 1" : "=&v"(pk) : "v"(qa), "v"(qb), "v"(8.0f));
#pragma unroll
                for (int g = 0; g < 4 && c0 + g < CPW; ++g) {
                    if (!present(c0 + g)) continue;
                    // the chunk's three 16-bit pieces h0 h1 h2: an even chunk stores (h0 h1) and h2, an odd one h0 and (h1 h2)
                    const uint32_t w0 = pk[3 * (g / 2) + (g & 1)], w1 = pk[3 * (g / 2) + (g & 1) + 1];
                    uint32_t h01, h12, h0, h2;
                    if (g & 1) {   // bits 16 .. 63 of (w0, w1)
                        h01 = __builtin_amdgcn_alignbit(w1, w0, 16); h12 = w1; h0 = w0 >> 16; h2 = w1 >> 16;
                    } else {       // bits 0 .. 47
                        h01 = w0; h12 = __builtin_amdgcn_alignbit(w1, w0, 16); h0 = w0; h2 = w1;
                    }
                    d_word[(c0 + g) * 96] = odd ? h12 : h01;
                    d_half[(c0 + g) * 192] = (uint16_t)(odd ? h0 : h2);
                }
            }
            if (code_rowsum) csum = (int)fsum;
            if (turn == run - 1 || next_base >= M) {
                // the run is complete (or the rows are): chunk j of slice s of rows row0 .. row0 + run - 1 is the
                // line [row / 32][s][j][row % 32][16 B]; neighbouring lanes take neighbouring rows.  Wave-private
                // LDS, in order: no workgroup barrier.
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                // (row0 is a multiple of `run`, a power of two <= 8: the run lies inside one 32-row block, so a
                // unit's address splits into a wave-uniform 64-bit base and the lane's fixed offsets wb_out[])
                const int64_t row0 = row - turn;
                const int slices = K >> 7;
                uint8_t *run_base = reinterpret_cast<uint8_t *>(codes) + ((row0 >> 5) * slices) * 3072 + (row0 & 31) * 16;
                const int rows_left = (int)min((int64_t)turn, M - 1 - row0);   // rows row0 .. row0 + rows_left exist
                const bool rr_ok = wb_rr <= rows_left;
#pragma unroll
                for (int c = 0; c < CPW; ++c) {
                    if (!present(c)) continue;
                    const int unit = wsub + c * waves_per_row;
                    uint8_t *unit_base = run_base + (int64_t)unit * (4 * 3072);
                    const int slices_here = slices - 4 * unit;   // a row's last unit may hold fewer than 4 slices
#pragma unroll
                    for (int t = 0; t < 3; ++t) {
                        if (t * kWave >= 24 * run) break;
                        if (rr_ok && wb_slice[t] < slices_here)
                            *reinterpret_cast<uint4 *>(unit_base + wb_out[t]) =
                                *reinterpret_cast<const uint4 *>(stage + wb_in[t] + c * 384);
                    }
                }
                __builtin_amdgcn_wave_barrier();   // the next run's LDS writes stay behind these reads
            }
        } else if (PACK4) {
            // two codes per byte, in the nibble order the GEMM widens with two masks: byte b of a
            // chunk's dword = code[b] (bits 0-3) | code[b + 4] (bits 4-7), two's complement
            uint32_t p[CPW];
#pragma unroll
            for (int c = 0; c < CPW; ++c) {
                p[c] = 0;
                if (!present(c)) continue;
                uint32_t b[8], u[4];
#pragma unroll
                for (int i = 0; i < 8; ++i) b[i] = __float_as_uint(fmaf(v[c][i], r, magic));
#pragma unroll
                for (int i = 0; i < 4; ++i) u[i] = (b[i] & 0xFu) | (b[i + 4] << 4);
                p[c] = __builtin_amdgcn_perm(__builtin_amdgcn_perm(u[3], u[2], 0x0c0c0400u),
                                             __builtin_amdgcn_perm(u[1], u[0], 0x0c0c0400u), 0x05040100u);
                if (code_rowsum) csum = __builtin_amdgcn_sdot8((int)p[c], 0x11111111, csum, false);  // 8 signed nibbles
            }
            if (via_lds) {
                // K % 32 == 0: a unit's 64 dwords (one per lane, in chunk order) are gathered through
                // LDS so that 16 lanes store the unit as 16-byte pieces; wave-private LDS, in-order
                uint32_t *sp = s_pack + wave * (CPW * 64);
#pragma unroll
                for (int c = 0; c < CPW; ++c) sp[c * 64 + chunk] = p[c];
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
                for (int idx0 = 0; idx0 < CPW * 16; idx0 += kWave) {
                    const int idx = idx0 + lane, c = idx >> 4, part = idx & 15;
                    const int k = (wsub + c * waves_per_row) * kUnit + part * 32;  // first channel of the piece
                    if (idx < CPW * 16 && row_ok && k < K)
                        *reinterpret_cast<uint4 *>(codes + (row * K + k) / 2) =
                            *reinterpret_cast<const uint4 *>(sp + c * 64 + part * 4);
                }
                __builtin_amdgcn_wave_barrier();   // the next row's LDS writes stay behind these reads
            } else {
#pragma unroll
                for (int c = 0; c < CPW; ++c)
                    if (row_ok && k0[c] < K) *reinterpret_cast<uint32_t *>(codes + (row * K + k0[c]) / 2) = p[c];
            }
        } else {
#pragma unroll
            for (int c = 0; c < CPW; ++c) {
                if (!present(c)) continue;
                uint32_t b[8];
                if (group_log2) {
                    // Block-wise scaling (a reading of the block-wise variant of Sec. 3.2): a channel group
                    // whose maximum a satisfies a * 2^e <= row maximum is quantized with the step scale / 2^e
                    // (e <= emax, the largest such e) and stored as code * 2^(emax - e), so that one token
                    // scale, scale / 2^emax, dequantizes every group and the GEMM is unchanged.  The lanes of
                    // a group are those that agree in lane bits 2, 3 (128 channels), bit 2 (256), none (512).
                    float a = 0.f;
#pragma unroll
                    for (int i = 0; i < 8; ++i) a = fmaxf(a, fabsf(v[c][i]));
                    a = fmaxf(a, __shfl_xor(a, 1, kWave));
                    a = fmaxf(a, __shfl_xor(a, 2, kWave));
                    a = fmaxf(a, __shfl_xor(a, 16, kWave));
                    a = fmaxf(a, __shfl_xor(a, 32, kWave));
                    if (group_log2 >= 8) a = fmaxf(a, __shfl_xor(a, 8, kWave));
                    if (group_log2 >= 9) a = fmaxf(a, __shfl_xor(a, 4, kWave));
                    int e = 0;
                    for (int t = 1; t <= emax; ++t)
                        if (ldexpf(a, t) <= amax) e = t;
                    const float rg = ldexpf(r, e);
                    const int sh = emax - e;
#pragma unroll
                    for (int i = 0; i < 8; ++i) b[i] = __float_as_uint(fmaf(v[c][i], rg, magic)) << sh;
                } else {
#pragma unroll
                    for (int i = 0; i < 8; ++i) b[i] = __float_as_uint(fmaf(v[c][i], r, magic));
                }
                // low bytes of b[0..3] / b[4..7] -> one dword each
                uint2 out;
                out.x = __builtin_amdgcn_perm(__builtin_amdgcn_perm(b[3], b[2], 0x0c0c0400u),
                                              __builtin_amdgcn_perm(b[1], b[0], 0x0c0c0400u), 0x05040100u);
                out.y = __builtin_amdgcn_perm(__builtin_amdgcn_perm(b[7], b[6], 0x0c0c0400u),
                                              __builtin_amdgcn_perm(b[5], b[4], 0x0c0c0400u), 0x05040100u);
                if (row_ok && k0[c] < K) *reinterpret_cast<uint2 *>(codes + row * K + k0[c]) = out;
                if (code_rowsum) {
                    csum = __builtin_amdgcn_sdot4((int)out.x, 0x01010101, csum, false);  // 4 signed bytes
                    csum = __builtin_amdgcn_sdot4((int)out.y, 0x01010101, csum, false);
                }
            }
        }
        if (code_rowsum) {   // (kernel argument: the whole workgroup takes the same path)
#pragma unroll
            for (int m = 1; m < kWave; m <<= 1) csum += __shfl_xor(csum, m, kWave);
            if (waves_per_row > 1) {
                int32_t *slots = s_sum + slot * (rows_per_wg * waves_per_row);
                if (lane == 0) slots[wave] = csum;
                __syncthreads();
                csum = 0;
                for (int i = 0; i < waves_per_row; ++i) csum += slots[row_in_wg * waves_per_row + i];
            }
            if (row_ok && wsub == 0 && lane == 0) code_rowsum[row] = csum;
        }
#pragma unroll
        for (int c = 0; c < CPW; ++c) raw[c] = nxt[c];
        base = next_base;
        row = next_base + row_in_wg * run;
        group_row = next_group_row;
        turn = next_turn;
    }
}

template <int LOG2B>
int launch_cpw(int cpw, dim3 grid, dim3 block, size_t smem, hipStream_t stream, const uint16_t *x, int64_t M,
               int K, int W, int rpw, double scale_mul, float recip_num, int pack4, int group_log2, int emax,
               int8_t *codes, float *x_scale, int32_t *code_rowsum, unsigned *clear_words) {
#define DVDQ_RQ_CASE(C)                                                                                   \
    case C:                                                                                               \
        if (pack4 == 3) {                                                                                 \
            static std::atomic<uint64_t> lds_allowed{0};                                                  \
            allow_dynamic_lds(reinterpret_cast<const void *>(&rotate_quant_kernel<LOG2B, C, 2>),          \
                              kLdsPerCu, lds_allowed);                                                    \
            hipLaunchKernelGGL((rotate_quant_kernel<LOG2B, C, 2>), grid, block, smem, stream, x, M, K, W, \
                               rpw, scale_mul, recip_num, group_log2, 0, 0, codes, x_scale, code_rowsum, clear_words); \
        } else if (pack4)                                                                                   \
            hipLaunchKernelGGL((rotate_quant_kernel<LOG2B, C, 1>), grid, block, smem, stream, x, M, K, W, \
                               rpw, scale_mul, recip_num, pack4 == 2, 0, 0, codes, x_scale, code_rowsum, clear_words); \
        else                                                                                              \
            hipLaunchKernelGGL((rotate_quant_kernel<LOG2B, C, 0>), grid, block, smem, stream, x, M, K, W, \
                               rpw, scale_mul, recip_num, 0, group_log2, emax, codes, x_scale,            \
                               code_rowsum, clear_words);                                                 \
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

int launch_rotate_quant(const uint16_t *x, int64_t M, int64_t K, int log2_block, int act_bits, int codes_format,
                        int group_log2, int8_t *codes, float *x_scale, int32_t *code_rowsum, hipStream_t stream) {
    // the kernel also zeroes the tile counters of the stream: a GEMM enqueued next needs no clearing kernel of its own
    unsigned *clear_words = sched_slot_to_clear(stream);
    const int emax = group_log2 ? 8 - act_bits : 0;
    // 0: int8; 1 / 2: packed nibbles stored per lane / gathered through LDS; 3: FP6 container
    const int pack4 = codes_format == DVDQ_CODES_FP6 ? 3 : (codes_format != DVDQ_CODES_PACKED4 ? 0 : ((K % 32) == 0 ? 2 : 1));
    const int units = (int)((K + kUnit - 1) / kUnit);
    // Waves per row: at most 4 units (32 fp32 values per lane) in registers per wave, never 3 waves, whole waves
    // per SIMD beyond 4, at most 16.  Workgroups of 8 waves, of 16 once a row takes 8 (two such rows then share a
    // workgroup and its barrier), 16 waves resident per compute unit (256 of them), every workgroup striding over
    // the rows.  Swept with the kernel timed where the layer runs it, between two GEMMs, over units per wave
    // (3 .. 8) and workgroups of 8 and 16 waves, rows of 2048 .. 16384 channels, both containers: rows of 4, 8 and
    // 16 units are 6-17 % faster as one, two and four waves of 4 units than in waves of 3 or fewer; 12 units are
    // 4 % slower as three waves of 4 than as four of 3; a 13824-channel row (27 units) takes 225 us per launch as
    // eight waves of 3-4 units in 16-wave workgroups, 238 in 8-wave workgroups, 252 as twelve waves of 2-3 units
    // (an earlier state of this rule, chosen from launches timed back to back).  Resident waves (8 .. 28) and
    // smaller workgroups stay within 2 % of this on the video-DiT shapes.
    int W = (units + 3) / 4;
    if (W == 3) W = 4;
    if (W > 4) W = (W + 3) / 4 * 4;   // whole waves per SIMD
    if (W > 16) W = 16;
    const int cpw = (units + W - 1) / W;
    if (cpw > 8) return DVDQ_ERR_UNSUPPORTED;
    const int wg_waves = W >= 8 ? 16 : 8;
    const int rows_per_wg = W >= wg_waves ? 1 : wg_waves / W;
    const dim3 block(kWave * W * rows_per_wg);
    int wgs_per_cu = 16 / (W * rows_per_wg);
    if (wgs_per_cu < 1) wgs_per_cu = 1;
    // FP6: consecutive rows a wave takes in turn (see the kernel): 8 if the LDS for collecting them allows
    int run = 1;
    if (pack4 == 3) {
        const size_t budget = (kLdsPerCu - 8192) / wgs_per_cu;
        for (run = 8; run > 1 && (size_t)W * rows_per_wg * run * (cpw * 384 + 16) > budget;) run /= 2;
    }
    const int group_rows = rows_per_wg * run;
    const int64_t wgs_needed = (M + group_rows - 1) / group_rows;
    const int64_t wgs_resident = 256 * (int64_t)wgs_per_cu;
    const dim3 grid((unsigned)(wgs_needed < wgs_resident ? wgs_needed : wgs_resident));
    size_t smem = 4 * sizeof(float) * W * rows_per_wg;   // abs-max slots, then code-sum slots
    if (pack4 == 2) smem = (smem + 15) / 16 * 16 + (size_t)W * rows_per_wg * cpw * 256;
    if (pack4 == 3) smem = (smem + 15) / 16 * 16 + (size_t)W * rows_per_wg * run * (cpw * 384 + 16);
    const double qmax = (double)((1 << (act_bits - 1)) - 1);
    const double norm = 1.0 / sqrt((double)(1 << log2_block));
    const double scale_mul = norm / qmax;
    const float recip_num = (float)norm;
    int rc = DVDQ_ERR_UNSUPPORTED;
#define DVDQ_RQ_B(L)                                                                                        \
    case L:                                                                                                 \
        rc = launch_cpw<L>(cpw, grid, block, smem, stream, x, M, (int)K, W, rows_per_wg, scale_mul,       \
                             recip_num, pack4, pack4 == 3 ? run : group_log2, emax, codes, x_scale, code_rowsum, clear_words); \
        break;
    switch (log2_block) {
        DVDQ_RQ_B(0) DVDQ_RQ_B(1) DVDQ_RQ_B(2) DVDQ_RQ_B(3) DVDQ_RQ_B(4)
        DVDQ_RQ_B(5) DVDQ_RQ_B(6) DVDQ_RQ_B(7) DVDQ_RQ_B(8) DVDQ_RQ_B(9)
    }
#undef DVDQ_RQ_B
    if (rc == DVDQ_OK && clear_words) sched_slot_cleared(stream);
    return rc;
}

}  // namespace dvdq

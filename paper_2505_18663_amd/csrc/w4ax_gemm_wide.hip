// W4Ax GEMM for gfx950, one 4-wave workgroup per compute unit with 128 x 128 wave tiles (Sec. 3.2:
// Y = X^ Lambda W^^T, exact integer accumulation; Sec. 3.1 DeQuant in the epilogue).  Two operand paths:
//   INT8 matrix path: int8 codes [M, K] x packed INT4 weights in the native layout of w4ax_gemm.hip,
//                     v_mfma_i32_32x32x32_i8, weights widened to int8 lanes of 16 * code in registers;
//   FP6 matrix path:  4-bit codes and weights as E2M3 patterns in the block-slice layout of
//                     w4a4_fp6_gemm.hip, v_mfma_f32_32x32x64_f8f6f4 (value = code / 8, sums exact in fp32).
//
// Why this shape.  With two waves per SIMD (the kernels in the two files named above) a wave can hold a
// 64 x 128 tile in 128 accumulator registers, and every MFMA then needs 6 bytes per lane of LDS fragment
// reads; LDS traffic (fragment reads plus the LDS-direct writes of the operand ring) is what those K loops
// are short of.  One wave per SIMD may use 512 registers: the 256 accumulators of a 128 x 128 tile live in
// AGPRs (the MFMAs are written as inline assembly so that they stay there), which cuts the fragment bytes per
// MFMA by a third and the LDS-direct bytes per MFMA by a quarter to a third, and leaves 256 VGPRs for two
// sets of operand fragments.  With only one wave per SIMD nothing else hides LDS latency, so the loop is
// skewed by one step: the fragments of step s+1 are requested before the MFMAs of step s are issued, also
// across the workgroup barrier that publishes the next K slice (the barrier sits before a slice's LAST
// step, whose fragments are already in registers).
//
// Ring: three buffers of one 128-channel slice of both operands (48 KB).  In iteration q the waves multiply
// slice q, slice q+1 is landing and the loads of slice q+2 are dealt out between the MFMA groups; the
// barrier of iteration q publishes slice q+1 and frees buffer q % 3 for slice q+3.  Everything else --
// LDS-direct loads with hand-kept vmcnt, persistent workgroups drawing tiles per XCD, tile scales staged in
// LDS, whole-line epilogue through the ring buffer that was consumed last -- follows w4ax_gemm.hip.
#include <type_traits>

#include "gemm_common.h"

namespace dvdq {

namespace {

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v6i __attribute__((ext_vector_type(6)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kFp6Block = kGroup * kBK * 6 / 8;   // 3072: 32 rows of one K slice as E2M3 patterns

// One group of four MFMAs that share the row operand `w` (output channels) against four column operands
// (tokens).  Inline assembly with the accumulators constrained to AGPRs; the leading s_nop covers the two
// wait states an MFMA needs after a VALU write of one of its operand registers (the widening), which the
// compiler cannot insert for an instruction it does not see.
__device__ __forceinline__ void mfma4_i8(v16i &c0, v16i &c1, v16i &c2, v16i &c3, v4i w, v4i a0, v4i a1, v4i a2, v4i a3) {
    asm volatile("s_nop 1\n\t"
                 "v_mfma_i32_32x32x32_i8 %0, %4, %5, %0\n\t"
                 "v_mfma_i32_32x32x32_i8 %1, %4, %6, %1\n\t"
                 "v_mfma_i32_32x32x32_i8 %2, %4, %7, %2\n\t"
                 "v_mfma_i32_32x32x32_i8 %3, %4, %8, %3"
                 : "+a"(c0), "+a"(c1), "+a"(c2), "+a"(c3)
                 : "v"(w), "v"(a0), "v"(a1), "v"(a2), "v"(a3));
}
__device__ __forceinline__ void mfma4_fp6(v16f &c0, v16f &c1, v16f &c2, v16f &c3, v6i w, v6i a0, v6i a1, v6i a2, v6i a3) {
    asm volatile("v_mfma_f32_32x32x64_f8f6f4 %0, %4, %5, %0 cbsz:2 blgp:2\n\t"
                 "v_mfma_f32_32x32x64_f8f6f4 %1, %4, %6, %1 cbsz:2 blgp:2\n\t"
                 "v_mfma_f32_32x32x64_f8f6f4 %2, %4, %7, %2 cbsz:2 blgp:2\n\t"
                 "v_mfma_f32_32x32x64_f8f6f4 %3, %4, %8, %3 cbsz:2 blgp:2"
                 : "+a"(c0), "+a"(c1), "+a"(c2), "+a"(c3)
                 : "v"(w), "v"(a0), "v"(a1), "v"(a2), "v"(a3));
}

}  // namespace

template <bool FP6>
__global__ __launch_bounds__(256, 1) void w4ax_gemm_wide_kernel(
    const uint8_t *__restrict__ codes, const float *__restrict__ x_scale, const uint8_t *__restrict__ w,
    const float *__restrict__ w_scale, const int8_t *__restrict__ w_zero, const int32_t *__restrict__ code_rowsum,
    const uint16_t *__restrict__ bias, int M, int N, int K, uint16_t *__restrict__ y, int32_t *__restrict__ acc_out,
    int tiles_m, int tiles_n, int group_n, unsigned *__restrict__ sched) {
    constexpr int BM = 256, BN = 256, NW = 4, WM = 128, WN = 128, TM = 4, TN = 4, STAGES = 3;
    constexpr int STEPS = FP6 ? 2 : 4;                       // pipeline steps per slice: 64 resp. 32 channels
    constexpr int A_ROW = kBK;                               // INT8 path: bytes of one code row per slice
    constexpr int A_STAGE = FP6 ? BM / 32 * kFp6Block : BM * A_ROW;
    constexpr int W_STAGE = FP6 ? BN / 32 * kFp6Block : BN * kBK / 2;
    constexpr int STAGE = A_STAGE + W_STAGE;                 // 48 KB on both paths
    constexpr int A_DMA = A_STAGE / 1024 / NW, W_DMA = W_STAGE / 1024 / NW, DMA = A_DMA + W_DMA;   // 12 per wave and slice
    constexpr int GROUPS = (STEPS - 1) * TN;                 // MFMA groups of a slice's steps before its barrier
    constexpr int DMA_PER_GROUP = (DMA + GROUPS - 1) / GROUPS;
    constexpr int OFF_BIAS = (BM + BN) * 4, OFF_RSUM = OFF_BIAS + BN * 2, OFF_ZERO = OFF_RSUM + BM * 4;
    constexpr int SCALES = OFF_ZERO + BN;
    constexpr int SHIFT = 4;                                 // INT8 path: the widened weights carry a factor 16
    constexpr float kFp6Unit = 64.f;                         // FP6 path: accumulator * 64 = integer sum
    constexpr int STORES = TM * TN * 2;                      // 16-byte store instructions per wave per full tile
    static_assert(STAGE == 48 * 1024 && DMA == 12, "ring geometry");
    static_assert(DMA + STORES < 64 && (STAGES - 1) * DMA + 8 < 64, "vmcnt is 6 bits");
    static_assert(NW * 4096 <= STAGE, "the epilogue stages 4 KB per wave in one ring buffer");
    using Acc = std::conditional_t<FP6, v16f, v16i>;

    extern __shared__ __align__(16) uint8_t smem[];
    const uint32_t smem_base = lds_address(smem);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = (wave & 1) * WM, wn = (wave >> 1) * WN;
    const int KT = K / kBK;
    const int G = ((N + kNPad - 1) / kNPad) * (kNPad / kGroup);   // 32-row groups in the padded weight buffer
    const int64_t w_slice_stride = (int64_t)G * (FP6 ? kFp6Block : kGroupBytes);
    const int last_block = (M - 1) / 32;                          // FP6 codes: row blocks past it do not exist

    // ---- tiles: persistent workgroups, per-XCD runs of tile numbers drawn through counters (sched) or dealt
    // in fixed shares (sched == nullptr); numbers travel through an 8-entry ring in LDS.  See w4ax_gemm.hip.
    const int total = tiles_m * tiles_n;
    const int grid = gridDim.x;  // multiple of 8
    const int xcd = blockIdx.x % 8;
    const int first_tile = xcd * (grid / 8) + blockIdx.x / 8;
    const int run_lo = (int)((int64_t)xcd * total / 8);
    const unsigned run_len = (unsigned)((int64_t)(xcd + 1) * total / 8) - (unsigned)run_lo;
    typedef volatile __attribute__((address_space(3))) int lds_int;
    lds_int *s_tiles = (lds_int *)DVDQ_LDS(smem + STAGES * STAGE + 3 * SCALES);
    // A tile number drawn while slice `draw_kt` of tile n is issued belongs to tile n + 2.  It is written into the
    // ring before a later barrier: the barrier after next when it comes from an atomic (by then the loads issued
    // around the atomic have been awaited, so its reply is there), the next barrier with fixed shares.  Draws follow
    // each other by K / 128 issue steps, and the prologue issues two steps at once, so up to three can be pending.
    int draws = 0, published = 2;          // tiles drawn / tile numbers written into the ring
    unsigned pend_v0 = 0, pend_v1 = 0, pend_v2 = 0;   // wave 0, lane 0: replies not yet written, oldest first
    int pend_a0 = 0, pend_a1 = 0, pend_a2 = 0, pend_n = 0;   // barriers they have seen
    const int publish_age = sched ? 2 : 1;
    auto tile_of_draw = [&] __device__(unsigned i, int ordinal) {
        if (sched) return i < run_len ? run_lo + (int)i : -1;
        const int t = first_tile + ordinal * grid;
        return t < total ? t : -1;
    };
    auto draw = [&] __device__() {
        unsigned v = 0;
        if (wave == 0 && sched && lane == 0) v = atomicAdd(sched + xcd, 1u);
        if (pend_n == 0) { pend_v0 = v; pend_a0 = 0; }
        else if (pend_n == 1) { pend_v1 = v; pend_a1 = 0; }
        else { pend_v2 = v; pend_a2 = 0; }
        ++pend_n;
        ++draws;
    };
    auto before_barrier = [&] __device__() {   // every wave, before each workgroup barrier of the pipeline
        ++pend_a0; ++pend_a1; ++pend_a2;
        while (pend_n > 0 && pend_a0 >= publish_age) {
            if (wave == 0) {
                if (lane == 0) s_tiles[published & 7] = tile_of_draw(pend_v0, published);
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            }
            ++published;
            pend_v0 = pend_v1; pend_a0 = pend_a1;
            pend_v1 = pend_v2; pend_a1 = pend_a2;
            --pend_n;
        }
    };
    auto leave = [&] __device__() {
        if (sched && tid == 0) {
            if (atomicAdd(sched + 8, 1u) == (unsigned)grid - 1) {
#pragma unroll
                for (int i = 0; i < 9; ++i) __hip_atomic_store(sched + i, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
        }
    };
    if (wave == 0) {
        unsigned i = 0;
        if (sched && lane == 0) i = atomicAdd(sched + xcd, 2u);
        if (lane == 0) {
            s_tiles[0] = tile_of_draw(i, 0);
            s_tiles[1] = tile_of_draw(i + 1, 1);
        } else if (lane >= 2 && lane < 8) {
            s_tiles[lane] = -1;   // a ring entry read before it was written would end the workgroup's work, not misdirect it
        }
    }
    draws = 2;
    __syncthreads();
    int comp_tile = __builtin_amdgcn_readfirstlane(s_tiles[0]);
    if (comp_tile < 0) {   // (whole workgroup: nothing below is reached, no barrier is missed)
        leave();
        return;
    }

    // ---- LDS-direct loads of one slice: 12 pieces of 1 KB per wave.
    // INT8 path, codes: piece i of wave v fills 8 consecutive LDS rows (128 B each) of the stage; LDS position p
    // of a row holds the row's 16-byte chunk p ^ swz(row) (see swz_bk); rows past M re-read the last valid row.
    // Weights: the tile's slice is one linear run of the native buffer (16 KB).
    // FP6 path: a 32-row block of codes of one slice is 3 KB contiguous in memory and in LDS (blocks past the last
    // one repeat it; their rows are never stored); the tile's weight slice is one 24 KB run.
    const uint32_t lane16 = lane * 16;
    int a_row[FP6 ? 1 : A_DMA];
    uint32_t a_voff[FP6 ? 1 : A_DMA];
    if constexpr (!FP6) {
#pragma unroll
        for (int i = 0; i < A_DMA; ++i) a_row[i] = (wave * A_DMA + i) * 8 + lane / 8;
    }
    const uint8_t *a_base = codes, *a_base2 = codes;   // FP6: the wave's two code blocks of the slice being issued
    const uint8_t *w_base = w;
    int issue_tile = 0, issue_kt = 0;
    bool issue_live = true;
    const int draw_kt = KT > 1 ? 1 : 0;
    uint32_t issue_sa = 0;
    auto issue_prepare = [&] __device__(int buf) {
        int issue_no = -1;
        if (issue_live && issue_kt == 0) {
            issue_no = __builtin_amdgcn_readfirstlane(s_tiles[issue_tile & 7]);
            issue_live = issue_no >= 0;
        }
        if (issue_live && issue_kt == draw_kt) draw();
        if (issue_no >= 0) {
            int m0, n0;
            tile_origin(issue_no, tiles_m, tiles_n, group_n, BM, BN, m0, n0);
            if constexpr (FP6) {
                a_base = uniform_ptr(codes + (int64_t)min(m0 / 32 + 2 * wave, last_block) * KT * kFp6Block);
                a_base2 = uniform_ptr(codes + (int64_t)min(m0 / 32 + 2 * wave + 1, last_block) * KT * kFp6Block);
                w_base = uniform_ptr(w + (int64_t)(n0 / kGroup) * kFp6Block);
            } else {
                a_base = uniform_ptr(codes + (int64_t)m0 * K);
                w_base = uniform_ptr(w + (int64_t)(n0 / kGroup) * kGroupBytes);
#pragma unroll
                for (int i = 0; i < A_DMA; ++i) {
                    const int row = min(a_row[i], M - 1 - m0);
                    a_voff[i] = (uint32_t)row * K + (((lane & 7) ^ swz_bk<A_ROW>(a_row[i])) << 4);
                }
            }
            // the tile's epilogue vectors: token scales, channel scales, bias, code sums, zero-points.  Three tiles
            // deep: loads run two slices ahead, so with one slice per tile the tile after next is issued before
            // this tile's epilogue has read its own
            const uint32_t sc = smem_base + STAGES * STAGE + (issue_tile % 3) * SCALES;
#pragma unroll
            for (int j = 0; j < (BM + BN) / 64; ++j) {
                if (j % NW != wave) continue;
                if (j < BM / 64)
                    lds_direct_load4(x_scale, (uint32_t)min(m0 + j * 64 + lane, M - 1) * 4, sc + j * 256);
                else
                    lds_direct_load4(w_scale, (uint32_t)min(n0 + (j - BM / 64) * 64 + lane, N - 1) * 4, sc + j * 256);
            }
            if (bias && n0 + BN <= N) {
#pragma unroll
                for (int j = 0; j < BN / 128; ++j)
                    if (j % NW == wave)
                        lds_direct_load4(bias + n0, (uint32_t)(j * 64 + lane) * 4, sc + OFF_BIAS + j * 256);
            }
            if (w_zero) {
#pragma unroll
                for (int j = 0; j < BM / 64; ++j)
                    if (j % NW == wave)
                        lds_direct_load4(code_rowsum, (uint32_t)min(m0 + j * 64 + lane, M - 1) * 4, sc + OFF_RSUM + j * 256);
                if (n0 + BN <= N) {
#pragma unroll
                    for (int j = 0; j < BN / 256; ++j)
                        if (j % NW == wave)
                            lds_direct_load4(w_zero + n0, (uint32_t)(j * 64 + lane) * 4, sc + OFF_ZERO + j * 256);
                }
            }
        }
        issue_sa = smem_base + buf * STAGE;
    };
    auto issue_one = [&] __device__(int idx) {
        if constexpr (FP6) {
            if (idx < 3)
                lds_direct_load16(a_base + idx * 1024, lane16, issue_sa + (wave * A_DMA + idx) * 1024);
            else if (idx < A_DMA)
                lds_direct_load16(a_base2 + (idx - 3) * 1024, lane16, issue_sa + (wave * A_DMA + idx) * 1024);
            else
                lds_direct_load16(w_base + (wave * W_DMA + idx - A_DMA) * 1024, lane16,
                                  issue_sa + A_STAGE + (wave * W_DMA + idx - A_DMA) * 1024);
        } else {
            if (idx < A_DMA)
                lds_direct_load16(a_base, a_voff[idx], issue_sa + (wave * A_DMA + idx) * 1024);
            else
                lds_direct_load16(w_base + (wave * W_DMA + idx - A_DMA) * 1024, lane16,
                                  issue_sa + A_STAGE + (wave * W_DMA + idx - A_DMA) * 1024);
        }
    };
    auto issue_advance = [&] __device__() {
        if (!issue_live) return;
        if (issue_kt + 1 < KT) {
            if constexpr (FP6) {
                a_base += kFp6Block;
                a_base2 += kFp6Block;
            } else {
                a_base += A_ROW;
            }
            w_base += w_slice_stride;
            ++issue_kt;
        } else {   // next: slice 0 of the next tile, whose addresses issue_prepare sets (or none: stay on this slice)
            issue_kt = 0;
            ++issue_tile;
        }
    };

    // ---- fragments.  MFMA operand row = lane % 32, K half = lane / 32.
    const int frow = lane & 31, fhalf = lane >> 5;
    // INT8 path: a step is 32 channels.  Code fragment: 16-byte chunk 2 s + fhalf of the row (xor swizzle);
    // weight fragment: 8 bytes at [32-row group][k32 step s][k16 half fhalf][row], widened to int8 lanes of 16 * code.
    // FP6 path: a step is 64 channels.  The 24-byte fragment 2 fhalf + s of a row is bytes 24 f .. 24 f + 23 of its
    // 96: step 0 takes chunk 3 fhalf whole and the lower half of chunk 3 fhalf + 1, step 1 the upper half of
    // that chunk and chunk 3 fhalf + 2 whole (a 16-byte and an 8-byte read per fragment and step).
    struct FragsI8 { v4i a[TM]; v2i w[TN]; };
    struct FragsF6 { v6i a[TM]; v6i w[TN]; };
    using Frags = std::conditional_t<FP6, FragsF6, FragsI8>;
    const int a_frag_off = FP6 ? (wm / 32) * kFp6Block + fhalf * 1536 + frow * 16 : (wm + frow) * A_ROW;
    const int w_frag_off = FP6 ? A_STAGE + (wn / 32) * kFp6Block + fhalf * 1536 + frow * 16
                               : A_STAGE + (wn / kGroup) * kGroupBytes + frow * 8 + fhalf * 256;
    const int a_xor = swz_bk<A_ROW>(frow);
    auto load_frags = [&] __device__(Frags &f, int buf, int s) {
        const uint8_t *st = smem + buf * STAGE;
        if constexpr (FP6) {
#pragma unroll
            for (int j = 0; j < TM; ++j) {
                const uint8_t *p = st + a_frag_off + j * kFp6Block;
                if (s == 0) {
                    const v4i h = *reinterpret_cast<const v4i *>(p);
                    const v2i t = *reinterpret_cast<const v2i *>(p + 512);
                    f.a[j] = v6i{h[0], h[1], h[2], h[3], t[0], t[1]};
                } else {
                    const v2i t = *reinterpret_cast<const v2i *>(p + 512 + 8);
                    const v4i h = *reinterpret_cast<const v4i *>(p + 1024);
                    f.a[j] = v6i{t[0], t[1], h[0], h[1], h[2], h[3]};
                }
            }
#pragma unroll
            for (int i = 0; i < TN; ++i) {
                const uint8_t *p = st + w_frag_off + i * kFp6Block;
                if (s == 0) {
                    const v4i h = *reinterpret_cast<const v4i *>(p);
                    const v2i t = *reinterpret_cast<const v2i *>(p + 512);
                    f.w[i] = v6i{h[0], h[1], h[2], h[3], t[0], t[1]};
                } else {
                    const v2i t = *reinterpret_cast<const v2i *>(p + 512 + 8);
                    const v4i h = *reinterpret_cast<const v4i *>(p + 1024);
                    f.w[i] = v6i{t[0], t[1], h[0], h[1], h[2], h[3]};
                }
            }
        } else {
#pragma unroll
            for (int j = 0; j < TM; ++j)
                f.a[j] = *reinterpret_cast<const v4i *>(st + a_frag_off + j * 32 * A_ROW + (((s * 2 + fhalf) ^ a_xor) << 4));
#pragma unroll
            for (int i = 0; i < TN; ++i)
                f.w[i] = *reinterpret_cast<const v2i *>(st + w_frag_off + i * kGroupBytes + s * 512);
        }
    };

    Acc acc[TN][TM];
    auto clear_acc = [&] __device__() {
#pragma unroll
        for (int i = 0; i < TN; ++i)
#pragma unroll
            for (int j = 0; j < TM; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;
    };
    // the MFMAs of one step; `first_load` .. : LDS-direct loads dealt out behind the groups (none when < 0)
    auto mfma_step = [&] __device__(const Frags &f, int group0) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < TN; ++i) {
            if constexpr (FP6) {
                mfma4_fp6(acc[i][0], acc[i][1], acc[i][2], acc[i][3], f.w[i], f.a[0], f.a[1], f.a[2], f.a[3]);
            } else {
                const uint32_t lo = (uint32_t)f.w[i][0], hi = (uint32_t)f.w[i][1];
                const v4i fw = {(int)((lo << 4) & 0xF0F0F0F0u), (int)(lo & 0xF0F0F0F0u), (int)((hi << 4) & 0xF0F0F0F0u),
                                (int)(hi & 0xF0F0F0F0u)};
                mfma4_i8(acc[i][0], acc[i][1], acc[i][2], acc[i][3], fw, f.a[0], f.a[1], f.a[2], f.a[3]);
            }
            if (group0 >= 0) {
#pragma unroll
                for (int d = (group0 + i) * DMA_PER_GROUP; d < DMA && d < (group0 + i + 1) * DMA_PER_GROUP; ++d) issue_one(d);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // ---- prologue: slices 0 and 1 on their way, slice 0 published, its first fragments requested
#pragma unroll
    for (int st = 0; st < STAGES - 1; ++st) {
        issue_prepare(st);
#pragma unroll
        for (int d = 0; d < DMA; ++d) issue_one(d);
        issue_advance();
    }
    wait_vmcnt<DMA>();
    before_barrier();
    __builtin_amdgcn_s_barrier();
    Frags f0, f1;
    load_frags(f0, 0, 0);
    clear_acc();

    int store_credit = 0, tile_j = 0;
    for (int q = 0;;) {
        for (int kt = 0; kt < KT; ++kt, ++q) {
            const int buf = q % STAGES;
            issue_prepare((q + STAGES - 1) % STAGES);   // slice q + 2 goes where slice q - 1 was
            // steps 0 .. STEPS - 2 of slice q; step s + 1's fragments are requested before step s multiplies
#pragma unroll
            for (int s = 0; s < STEPS - 1; ++s) {
                load_frags((s & 1) ? f0 : f1, buf, s + 1);
                __builtin_amdgcn_sched_barrier(0);
                mfma_step((s & 1) ? f1 : f0, s * TN);
            }
            issue_advance();
            // Publish slice q + 1: it has landed once at most the loads of slice q + 2 (just issued) are
            // outstanding, plus, right after a full tile's epilogue, that tile's stores.  Every fragment read of
            // slice q has been issued; once they are back (lgkmcnt) and everyone is here, buffer q % 3 is free.
            if (store_credit > 0) {
                wait_vmcnt<DMA + STORES>();
                store_credit = 0;
            } else {
                wait_vmcnt<DMA>();
            }
            before_barrier();
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            __builtin_amdgcn_s_barrier();
            // the last step of slice q multiplies while step 0 of slice q + 1 is fetched (past the workgroup's
            // last slice: a stale but in-bounds buffer, never used)
            load_frags(f0, (q + 1) % STAGES, 0);
            __builtin_amdgcn_sched_barrier(0);
            mfma_step(f1, -1);
        }

        // ---- epilogue of tile comp_tile.  Accumulator register r = 4 g + e of MFMA tile (i, j) in lane l is
        //   n = n0 + wn + 32 i + 8 g + 4 (l / 32) + e,   m = m0 + wm + 32 j + (l % 32);
        //   INT8 path: 16 * sum, FP6 path: sum / 64.
        // (The MFMAs are invisible to the compiler: the wait states between an MFMA's write and a read of its
        // result are put here by hand, generously.)
        asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
        int m0, n0;
        tile_origin(comp_tile, tiles_m, tiles_n, group_n, BM, BN, m0, n0);
        ++tile_j;
        comp_tile = __builtin_amdgcn_readfirstlane(s_tiles[tile_j & 7]);   // the next one (its loads are under way)
        const bool vec8 = (N & 7) == 0;
        const uint8_t *s_tile = smem + STAGES * STAGE + ((tile_j - 1) % 3) * SCALES;
        const float *s_xs = reinterpret_cast<const float *>(s_tile);
        const float *s_ws = s_xs + BM;
        const int32_t *s_rsum = reinterpret_cast<const int32_t *>(s_tile + OFF_RSUM);
        // the integer accumulator, and sum q (c - z) = acc - z * rs with a 24-bit multiply (ranges: C ABI)
        auto acc_int = [] __device__(auto a) {
            if constexpr (FP6) return (int)(a * kFp6Unit);
            else return (int)a >> SHIFT;
        };
        auto unzero = [] __device__(int a, int z, int rs) { return a - __mul24(z, rs); };
        uint8_t *stg = smem + ((q - 1) % STAGES) * STAGE + wave * 4096;   // the buffer of the slice consumed last
        if (vec8 && !acc_out && m0 + BM <= M && n0 + BN <= N) {
            // ---- interior tile: no predicates; channel vectors fetched one register group ahead; the bf16 tile
            // is transposed through LDS, 32 tokens x 64 channels at a time, into whole-line streaming stores
            if (KT >= 2) store_credit = 1;
            auto interior = [&] __device__(auto has_zero) __attribute__((always_inline)) {
                constexpr bool ZP = decltype(has_zero)::value;
                int lane_e = lane;   // (keeps the epilogue's lane-dependent addresses out of the K loop's registers)
                asm volatile("" : "+v"(lane_e));
                const int frow = lane_e & 31, fhalf = lane_e >> 5;
                const float *ws_l = s_ws + wn + fhalf * 4;
                const uint32_t *bias_l = reinterpret_cast<const uint32_t *>(s_tile + OFF_BIAS) + (wn + fhalf * 4) / 2;
                const uint32_t *zero_l = reinterpret_cast<const uint32_t *>(s_tile + OFF_ZERO) + (wn + fhalf * 4) / 4;
                // token scale folded with the accumulator's power-of-two unit (exact); with zero-points the
                // integer accumulator is formed first
                float xs_l[TM];
                int rsum[TM];
#pragma unroll
                for (int j = 0; j < TM; ++j) {
                    const float xs = s_xs[wm + j * 32 + frow];
                    if constexpr (FP6) xs_l[j] = ZP ? xs : xs * kFp6Unit;
                    else xs_l[j] = xs * (1.f / (float)(1 << SHIFT));
                    rsum[j] = ZP ? s_rsum[wm + j * 32 + frow] : 0;
                }
                const int rd_row = lane_e >> 3, rd_piece = lane_e & 7;
                struct ChannelVec { float4 ws; uint2 bb; uint32_t zq; };
                auto fetch = [&] __device__(ChannelVec &cv, int i, int g) {
                    const int c = i * 32 + g * 8;
                    cv.ws = *reinterpret_cast<const float4 *>(ws_l + c);
                    if (bias) cv.bb = *reinterpret_cast<const uint2 *>(bias_l + c / 2);
                    if constexpr (ZP) cv.zq = zero_l[c / 4];
                };
                ChannelVec cv[2];
                fetch(cv[0], 0, 0);
                int k = 0;
#pragma unroll
                for (int ip = 0; ip < TN / 2; ++ip) {
#pragma unroll
                    for (int j = 0; j < TM; ++j) {
#pragma unroll
                        for (int ii = 0; ii < 2; ++ii) {
                            const int i = 2 * ip + ii;
#pragma unroll
                            for (int g = 0; g < 4; g += 2) {
                                uint32_t pk[2][2];
#pragma unroll
                                for (int h = 0; h < 2; ++h, ++k) {
                                    {   // the group after this one, in this loop nest's order
                                        int gn = g + h + 1, iin = ii, jn = j, ipn = ip;
                                        if (gn == 4) { gn = 0; if (++iin == 2) { iin = 0; if (++jn == TM) { jn = 0; ++ipn; } } }
                                        if (ipn < TN / 2) fetch(cv[(k + 1) & 1], 2 * ipn + iin, gn);
                                    }
                                    const ChannelVec &c = cv[k & 1];
                                    const int r = (g + h) * 4;
                                    float o[4];
#pragma unroll
                                    for (int e = 0; e < 4; ++e) {
                                        if constexpr (ZP) {
                                            const int z = (int)(int8_t)(c.zq >> (8 * e));
                                            if constexpr (FP6) o[e] = (float)unzero(acc_int(acc[i][j][r + e]), z, rsum[j]) * xs_l[j];
                                            else o[e] = (float)unzero((int)acc[i][j][r + e], z * (1 << SHIFT), rsum[j]) * xs_l[j];
                                        } else {
                                            o[e] = (float)acc[i][j][r + e] * xs_l[j];
                                        }
                                    }
                                    o[0] *= c.ws.x;
                                    o[1] *= c.ws.y;
                                    o[2] *= c.ws.z;
                                    o[3] *= c.ws.w;
                                    if (bias) {
                                        o[0] += __uint_as_float(c.bb.x << 16);
                                        o[1] += __uint_as_float(c.bb.x & 0xFFFF0000u);
                                        o[2] += __uint_as_float(c.bb.y << 16);
                                        o[3] += __uint_as_float(c.bb.y & 0xFFFF0000u);
                                    }
                                    pk[h][0] = pack_bf16x2(o[0], o[1]);
                                    pk[h][1] = pack_bf16x2(o[2], o[3]);
                                }
#pragma unroll
                                for (int d = 0; d < 2; ++d) {
                                    auto sw = __builtin_amdgcn_permlane32_swap(pk[0][d], pk[1][d], false, false);
                                    pk[0][d] = sw[0];
                                    pk[1][d] = sw[1];
                                }
                                const int piece = ii * 4 + g + fhalf;   // 16-byte piece of the 64-channel row
                                *reinterpret_cast<uint4 *>(stg + frow * 128 + ((piece ^ (frow & 7)) << 4)) =
                                    make_uint4(pk[0][0], pk[0][1], pk[1][0], pk[1][1]);
                            }
                        }
                        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                        __builtin_amdgcn_wave_barrier();
                        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                        uint16_t *yb = y + (int64_t)(m0 + wm + j * 32 + rd_row) * N + (n0 + wn + ip * 64 + rd_piece * 8);
                        uint4 v[4];
#pragma unroll
                        for (int pass = 0; pass < 4; ++pass) {
                            const int row = pass * 8 + rd_row;
                            v[pass] = *reinterpret_cast<const uint4 *>(stg + row * 128 + ((rd_piece ^ (row & 7)) << 4));
                        }
#pragma unroll
                        for (int pass = 0; pass < 4; ++pass) store_streaming16(yb + (int64_t)pass * 8 * N, v[pass]);
                        __builtin_amdgcn_wave_barrier();   // the next chunk's LDS writes stay behind these reads
                    }
                }
            };
            if (w_zero) interior(std::true_type{});
            else interior(std::false_type{});
        } else {
            // ---- edge tiles, N not a multiple of 8, or the accumulator hook: predicated per element, through the
            // integer accumulator (same values and rounding order as the interior path)
            int lane_s = lane;
            asm volatile("" : "+v"(lane_s));
            const int frow = lane_s & 31, fhalf = lane_s >> 5;
#pragma unroll
            for (int j = 0; j < TM; ++j) {
                const int m = m0 + wm + j * 32 + frow;
                const bool m_ok = m < M;
                const float xs = s_xs[wm + j * 32 + frow];
                const int rs = w_zero ? s_rsum[wm + j * 32 + frow] : 0;
#pragma unroll
                for (int i = 0; i < TN; ++i) {
                    const int nb = n0 + wn + i * 32;   // this MFMA tile's first output channel
                    int a[16];
#pragma unroll
                    for (int g = 0; g < 4; ++g)
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const int n = nb + g * 8 + fhalf * 4 + e;
                            a[g * 4 + e] = acc_int(acc[i][j][g * 4 + e]);
                            if (w_zero && n < N) a[g * 4 + e] = unzero(a[g * 4 + e], (int)w_zero[n], rs);
                        }
                    if (acc_out && m_ok) {
#pragma unroll
                        for (int g = 0; g < 4; ++g) {
                            const int n = nb + g * 8 + fhalf * 4;
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                if (n + e < N) acc_out[(int64_t)m * N + n + e] = a[g * 4 + e];
                        }
                    }
                    if (vec8) {
                        uint32_t pk[4][2];
#pragma unroll
                        for (int g = 0; g < 4; ++g) {
                            const int n = nb + g * 8 + fhalf * 4;
                            float o[4];
                            if (n < N) {  // N % 8 == 0 and n % 4 == 0: n + 3 < N as well
                                const float4 ws = *reinterpret_cast<const float4 *>(s_ws + (n - n0));
                                o[0] = (float)a[g * 4 + 0] * xs * ws.x;
                                o[1] = (float)a[g * 4 + 1] * xs * ws.y;
                                o[2] = (float)a[g * 4 + 2] * xs * ws.z;
                                o[3] = (float)a[g * 4 + 3] * xs * ws.w;
                                if (bias) {
                                    const uint2 bb = *reinterpret_cast<const uint2 *>(bias + n);
                                    o[0] += __uint_as_float(bb.x << 16);
                                    o[1] += __uint_as_float(bb.x & 0xFFFF0000u);
                                    o[2] += __uint_as_float(bb.y << 16);
                                    o[3] += __uint_as_float(bb.y & 0xFFFF0000u);
                                }
                            } else {
                                o[0] = o[1] = o[2] = o[3] = 0.f;
                            }
                            pk[g][0] = pack_bf16x2(o[0], o[1]);
                            pk[g][1] = pack_bf16x2(o[2], o[3]);
                        }
#pragma unroll
                        for (int g = 0; g < 4; g += 2) {
#pragma unroll
                            for (int d = 0; d < 2; ++d) {
                                auto r = __builtin_amdgcn_permlane32_swap(pk[g][d], pk[g + 1][d], false, false);
                                pk[g][d] = r[0];
                                pk[g + 1][d] = r[1];
                            }
                            const int n = nb + g * 8 + fhalf * 8;
                            if (m_ok && n < N)
                                *reinterpret_cast<uint4 *>(y + (int64_t)m * N + n) =
                                    make_uint4(pk[g][0], pk[g][1], pk[g + 1][0], pk[g + 1][1]);
                        }
                    } else if (m_ok) {
#pragma unroll
                        for (int g = 0; g < 4; ++g) {
                            const int n = nb + g * 8 + fhalf * 4;
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                if (n + e >= N) break;
                                float o = (float)a[g * 4 + e] * xs * s_ws[n + e - n0];
                                if (bias) o += __uint_as_float((uint32_t)bias[n + e] << 16);
                                y[(int64_t)m * N + n + e] = (uint16_t)(pack_bf16x2(o, 0.f) & 0xFFFFu);
                            }
                        }
                    }
                }
            }
        }
        if (comp_tile < 0) break;
        clear_acc();
        // the staging buffer is the one the next slice's loads go to: nobody may issue them before everyone
        // has stored its part of the tile
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
    }
    wait_vmcnt<0>();   // no LDS-direct load may still be in flight when the workgroup's LDS is released
    leave();
}

namespace {

template <bool FP6>
int launch_wide(const uint8_t *codes, const float *x_scale, const uint8_t *w, const float *w_scale, const int8_t *w_zero,
                const int32_t *code_rowsum, const uint16_t *bias, int M, int N, int K, uint16_t *y, int32_t *acc_out,
                hipStream_t stream) {
    constexpr int BM = 256, BN = 256, STAGES = 3;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    const int n_groups = (tiles_n + 15) / 16;   // column tiles per L2 sharing group: balanced groups of at most 16
    const int group_n = (tiles_n + n_groups - 1) / n_groups;
    const int total = tiles_m * tiles_n;
    int grid = 256;
    if (total < grid) grid = (total + 7) / 8 * 8;
    const size_t smem = (size_t)STAGES * 48 * 1024 + 3 * ((BM + BN) * 4 + BN * 2 + BM * 4 + BN) + 8 * sizeof(int);
    auto k = w4ax_gemm_wide_kernel<FP6>;
    static std::atomic<uint64_t> configured{0};
    allow_dynamic_lds(reinterpret_cast<const void *>(k), smem, configured);
    hipLaunchKernelGGL(k, dim3((unsigned)grid), dim3(256), smem, stream, codes, x_scale, w, w_scale, w_zero, code_rowsum,
                       bias, M, N, K, y, acc_out, tiles_m, tiles_n, group_n,
                       K / kBK >= 2 ? sched_slot(stream) : nullptr);   // a tile draw takes two slices to come back
    return check_launch();
}

}  // namespace

int launch_w4ax_gemm_wide(const uint8_t *codes, const float *x_scale, const uint8_t *w, const float *w_scale,
                          const int8_t *w_zero, const int32_t *code_rowsum, const uint16_t *bias, int64_t M, int64_t N,
                          int64_t K, bool fp6, uint16_t *y, int32_t *acc_out, hipStream_t stream) {
    if (fp6)
        return launch_wide<true>(codes, x_scale, w, w_scale, w_zero, code_rowsum, bias, (int)M, (int)N, (int)K, y, acc_out,
                                 stream);
    return launch_wide<false>(codes, x_scale, w, w_scale, w_zero, code_rowsum, bias, (int)M, (int)N, (int)K, y, acc_out,
                              stream);
}

}  // namespace dvdq

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
// slice q, slice q+1 is landing and loads of slice q+2 are dealt out between the MFMAs (INT8 path: all twelve
// per wave; FP6 path: its second half, the first half having gone out behind the last step of slice q-1, and
// behind the last step of slice q the first half of slice q+3); the barrier of iteration q publishes slice
// q+1 and frees buffer q % 3 for slice q+3.  Everything else -- LDS-direct loads
// with hand-kept vmcnt, persistent workgroups drawing tiles per XCD, tile scales staged in LDS, whole-line
// epilogue through the ring buffer that was consumed last -- follows w4ax_gemm.hip.  The epilogue stages 4 KB
// per wave in the weight half of that buffer; on the FP6 path (tiles of three slices or more) its code half is
// filled meanwhile with the first half of the next tile's slice 2, so that the loads cross a tile boundary in the
// same order as inside a tile and a tile's first step issues six loads, not twelve, behind the stores of the
// tile before (measured per tile on K = 1536: 970 of 27300 clocks less on 32 workgroups, 1280 of 28600 on the
// whole chip, where the output of all compute units leaves at once and the loads queue behind it).
//
// What the single wave per SIMD is sensitive to (measured with shader-clock timestamps around the steps and
// with register-only loops): an FP6 MFMA occupies the pipe for 32 clocks and the wave issues about six other
// instructions in that time; whatever else stands between two MFMAs delays the second.  Hence: a run of
// LDS-direct loads shares one M0 and one base address and moves by the instruction offset (which applies to
// the global and to the LDS address alike) instead of three scalar instructions per load; the per-slice
// bookkeeping has a branch-free common path and is dealt out over several MFMA slots; and, on the FP6 path,
// the twelve loads of a slice are spread over both steps of an iteration (the path from L2 into LDS moves 64
// bytes per clock and compute unit, a slice is 48 KB, a step is 512 clocks: twelve loads within one step back
// up and hold the MFMAs behind them).  Together: 1980 -> 1360 clocks per slice on K = 13824 (1024 would be
// the matrix pipe alone).
#include <type_traits>

#include "gemm_common.h"

namespace dvdq {

namespace {

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v6i __attribute__((ext_vector_type(6)));

constexpr int kFp6Block = kGroup * kBK * 6 / 8;   // 3072: 32 rows of one K slice as E2M3 patterns

// compile-time loop: f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>), in order
template <int V> using I = std::integral_constant<int, V>;
template <int N, int K0 = 0, class F>
__device__ __forceinline__ void static_for(F &&f) {
    if constexpr (K0 < N) {
        f(I<K0>{});
        static_for<N, K0 + 1>(f);
    }
}

#include "wide_acc.inc"


}  // namespace

// ACROSS (FP6 path, tiles of three K slices or more): the load pipeline runs across tile boundaries exactly as
// inside a tile.  A kernel of its own rather than a run-time flag: with both orders in one loop the compiler copies
// registers at the loop's edges, among them the pending reply of the tile draw, and waits for every outstanding
// load in front of such a copy.
template <bool FP6, bool ACROSS>
__global__ __launch_bounds__(256, 1) void w4ax_gemm_wide_kernel(
    const uint8_t *__restrict__ codes, const float *__restrict__ x_scale, const uint8_t *__restrict__ w,
    const float *__restrict__ w_scale, const int8_t *__restrict__ w_zero, const int32_t *__restrict__ code_rowsum,
    const uint16_t *__restrict__ bias, int M, int N, int K, uint16_t *__restrict__ y, int32_t *__restrict__ acc_out,
    int tiles_m, int tiles_n, int group_n, unsigned *__restrict__ sched) {
    constexpr int BM = 256, BN = 256, NW = 4, WM = 128, WN = 128, TM = 4, TN = 4, STAGES = 3;
    // (pipeline steps per slice: FP6 path 2 of 64 channels, INT8 path 4 of 32)
    constexpr int A_ROW = kBK;                               // INT8 path: bytes of one code row per slice
    constexpr int A_STAGE = FP6 ? BM / 32 * kFp6Block : BM * A_ROW;
    constexpr int W_STAGE = FP6 ? BN / 32 * kFp6Block : BN * kBK / 2;
    constexpr int STAGE = A_STAGE + W_STAGE;                 // 48 KB on both paths
    constexpr int A_DMA = A_STAGE / 1024 / NW, W_DMA = W_STAGE / 1024 / NW, DMA = A_DMA + W_DMA;   // 12 per wave and slice
    constexpr int OFF_BIAS = (BM + BN) * 4, OFF_RSUM = OFF_BIAS + BN * 2, OFF_ZERO = OFF_RSUM + BM * 4;
    constexpr int SCALES = OFF_ZERO + BN;
    constexpr int SHIFT = 4;                                 // INT8 path: the widened weights carry a factor 16
    constexpr float kFp6Unit = 64.f;                         // FP6 path: accumulator * 64 = integer sum
    constexpr int STORES = TM * TN * 2;                      // 16-byte store instructions per wave per full tile
    static_assert(STAGE == 48 * 1024 && DMA == 12, "ring geometry");
    static_assert(DMA + STORES < 64 && (STAGES - 1) * DMA + 8 < 64, "vmcnt is 6 bits");
    static_assert(FP6 || !ACROSS, "the INT8 path issues a slice's loads in one piece");
    static_assert(NW * 4096 <= W_STAGE, "the epilogue stages 4 KB per wave in the weight half of one ring buffer");

    extern __shared__ __align__(16) uint8_t smem[];
    const uint32_t smem_base = lds_address(smem);
    claim_all_agprs();

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = (wave & 1) * WM, wn = (wave >> 1) * WN;
    const int KT = K / kBK;
    const int G = ((N + kNPad - 1) / kNPad) * (kNPad / kGroup);   // 32-row groups in the padded weight buffer
    const int64_t w_slice_stride = (int64_t)G * (FP6 ? kFp6Block : kGroupBytes);
    const int last_block = (M - 1) / 32;                          // FP6 codes: row blocks past it do not exist

    // ---- tiles: persistent workgroups, per-XCD runs of tile numbers drawn through counters (sched) or dealt
    // in fixed shares (sched == nullptr); numbers travel through an 8-entry ring in LDS.  See w4ax_gemm.hip.
    const TileSource tiles(tiles_m, tiles_n, sched);
    typedef volatile __attribute__((address_space(3))) int lds_int;
    lds_int *s_tiles = (lds_int *)DVDQ_LDS(smem + STAGES * STAGE + 3 * SCALES);
    // Fixed shares (no counters): the ordinal-th tile of this workgroup follows from its number alone, which
    // every wave computes for itself.  Drawn tiles (K / 128 >= 2), two protocols:
    // FP6 path: the number drawn while slice `draw_kt` of tile n is issued belongs to tile n + 2; wave 0 writes it
    //   into the ring before the barrier after next (by then the loads issued around the atomic have been
    //   awaited, so its reply is there), two barriers before it is read.  Draws are at least two slices apart,
    //   so at most one is pending.
    // INT8 path: the number of tile n + 2 is drawn by wave 0 at the start of the epilogue of tile n and written
    //   into the ring in front of that tile's first stores; the workgroup barrier that closes the epilogue makes
    //   it visible; it is first read when slice 0 of tile n + 2 is issued, during tile n + 1.
    // Why two: a reply that stays pending across loop iterations lives in a register the compiler may copy, and
    // it waits for every outstanding vector memory operation of the wave in front of such a copy.  In the INT8
    // kernel it put one into the K loop (5 % of the kernel's time); in the FP6 kernel it does not (a test on the
    // assembly watches that), and there the epilogue protocol costs more than it saves: wave 0 waits for the
    // reply about a thousand clocks into every epilogue, 10 % on tiles of twelve slices.
    constexpr bool DRAW_IN_EPILOGUE = !FP6;
    int published = 2;       // tile numbers written into the ring
    unsigned drawn = 0;      // wave 0, lane 0: reply of the pending draw
    int draw_wait = 0;       // barriers until the pending draw is written into the ring (0: none pending)
    auto draw = [&] __device__() {
        if (DRAW_IN_EPILOGUE || !tiles.ctr) return;
        if (wave == 0 && lane == 0) drawn = tiles.draw();
        draw_wait = 2;
    };
    auto before_barrier = [&] __device__() {   // every wave, before each workgroup barrier of the pipeline
        if constexpr (DRAW_IN_EPILOGUE) return;
        draw_wait = __builtin_amdgcn_readfirstlane(draw_wait);   // (wave-uniform: keep it in a scalar register)
        if (__builtin_expect(draw_wait > 0, 0) && --draw_wait == 0) {
            if (wave == 0) {
                if (lane == 0) s_tiles[published & 7] = tiles.tile(drawn, 0);
                asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
            }
            ++published;
        }
    };
    if (tiles.ctr && wave == 0) {
        if (lane == 0) {
            int t0, t1;
            tiles.first_two(t0, t1);
            s_tiles[0] = t0;
            s_tiles[1] = t1;
        } else if (lane >= 2 && lane < 8) {
            s_tiles[lane] = -1;   // a ring entry read before it was written would end the workgroup's work, not misdirect it
        }
    }
    __syncthreads();
    auto tile_number = [&] __device__(int ordinal) {   // the ordinal-th tile of this workgroup (-1: none left)
        return tiles.ctr ? __builtin_amdgcn_readfirstlane(s_tiles[ordinal & 7]) : tiles.tile(0u, ordinal);
    };
    int comp_tile = tile_number(0);
    if (comp_tile < 0) return;   // (whole workgroup: nothing below is reached, no barrier is missed)

    // ---- LDS-direct loads of one slice: 12 pieces of 1 KB per wave.
    // INT8 path, codes: piece i of wave v fills 8 consecutive LDS rows (128 B each) of the stage; LDS position p
    // of a row holds the row's 16-byte chunk p ^ swz(row) (see swz_bk); rows past M re-read the last valid row.
    // Weights: the tile's slice is one linear run of the native buffer (16 KB).
    // FP6 path: a 32-row block of codes of one slice is 3 KB contiguous in memory and in LDS (blocks past the last
    // one repeat it; their rows are never stored); the tile's weight slice is one 24 KB run.
    const uint32_t lane16 = lane * 16, lane16_hi = lane16 + 4096;
    int a_row[FP6 ? 1 : A_DMA];
    uint32_t a_voff[FP6 ? 1 : A_DMA];
    if constexpr (!FP6) {
#pragma unroll
        for (int i = 0; i < A_DMA; ++i) a_row[i] = (wave * A_DMA + i) * 8 + lane / 8;
    }
    const uint8_t *a_base = codes, *a_base2 = codes;   // FP6: the wave's two code blocks of the slice being issued
    const uint8_t *w_base = w;
    int issue_tile = 0, issue_kt = 0;
    int issue_live = 1;   // (wave-uniform, kept in a scalar register)
    const int draw_kt = KT > 1 ? 1 : 0;
    uint32_t issue_sa_a = 0, issue_sa_w = 0;   // LDS addresses of this wave's first code piece and first weight piece
    auto issue_prepare = [&] __device__(uint32_t buf_off) {
        int issue_no = -1;
        if (__builtin_expect((issue_kt <= draw_kt ? issue_live : 0) != 0, 0)) {   // (a tile's first slice or two: off the common path)
            if (issue_kt == 0) {
                issue_no = tile_number(issue_tile);
                issue_live = __builtin_amdgcn_readfirstlane(issue_no >= 0 ? 1 : 0);
            }
            if (issue_live && issue_kt == draw_kt) draw();
        }
        if (__builtin_expect(issue_no >= 0, 0)) {
            int m0, n0;
            tile_origin(issue_no, tiles_m, tiles_n, group_n, BM, BN, m0, n0);
            if constexpr (FP6) {
                a_base = uniform_ptr(codes + (int64_t)min(m0 / 32 + 2 * wave, last_block) * KT * kFp6Block);
                a_base2 = uniform_ptr(codes + (int64_t)min(m0 / 32 + 2 * wave + 1, last_block) * KT * kFp6Block);
                w_base = uniform_ptr(w + (int64_t)(n0 / kGroup) * kFp6Block + wave * W_DMA * 1024);
            } else {
                a_base = uniform_ptr(codes + (int64_t)m0 * K);
                w_base = uniform_ptr(w + (int64_t)(n0 / kGroup) * kGroupBytes + wave * W_DMA * 1024);
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
        issue_sa_a = smem_base + buf_off + wave * A_DMA * 1024;
        issue_sa_w = smem_base + buf_off + A_STAGE + wave * W_DMA * 1024;
    };
    // Piece idx of the wave's 12.  Pieces whose source and destination both advance by 1 KB share M0 and the base
    // address and differ in the instruction offset: the FP6 path sets M0 four times per slice (first and second
    // code block, weight pieces 0-3 and 4-5), the INT8 path once per code piece and once for its four weight pieces.
    auto issue_one = [&] __device__(auto idx_c) __attribute__((always_inline)) {
        constexpr int idx = decltype(idx_c)::value;
        // (the LDS addresses are wave-uniform, but short of scalar registers the compiler may keep them in a vector
        // register across a step and would then hand that register to the load's scalar operand: the explicit
        // first-lane read makes it a scalar again, and is nothing where the value already is one)
        auto sa = [] __device__(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); };
        if constexpr (FP6) {
            if constexpr (idx == 0) lds_direct_load16(a_base, lane16, sa(issue_sa_a));
            else if constexpr (idx < 3) lds_direct_load16_more<idx * 1024>(a_base, lane16);
            else if constexpr (idx == 3) lds_direct_load16(a_base2, lane16, sa(issue_sa_a + 3072));
            else if constexpr (idx < A_DMA) lds_direct_load16_more<(idx - 3) * 1024>(a_base2, lane16);
            else if constexpr (idx == A_DMA) lds_direct_load16(w_base, lane16, sa(issue_sa_w));
            else if constexpr (idx < A_DMA + 4) lds_direct_load16_more<(idx - A_DMA) * 1024>(w_base, lane16);
            else if constexpr (idx == A_DMA + 4) lds_direct_load16(w_base, lane16_hi, sa(issue_sa_w + 4096));
            else lds_direct_load16_more<(idx - A_DMA - 4) * 1024>(w_base, lane16_hi);
        } else {
            if constexpr (idx < A_DMA) lds_direct_load16(a_base, a_voff[idx], issue_sa_a + idx * 1024);
            else if constexpr (idx == A_DMA) lds_direct_load16(w_base, lane16, issue_sa_w);
            else lds_direct_load16_more<(idx - A_DMA) * 1024>(w_base, lane16);
        }
    };
    // To the next slice of the tile, or to slice 0 of the next tile, whose addresses issue_prepare sets (or none:
    // stay on this slice).  Without branches: it runs once per slice between two MFMAs.
    // In three parts, so that each fits in the shadow of one MFMA (a wave issues about six other instructions
    // while an FP6 MFMA occupies the pipe; what does not fit delays the next MFMA).  The empty asm statements pin
    // each part where it is called: the compiler would otherwise sink it to the barrier behind the step.
    int adv_more = 0;
    auto issue_advance_part = [&] __device__(auto part_c) __attribute__((always_inline)) {
        constexpr int PART = decltype(part_c)::value;
        if constexpr (PART == 0) {
            // (wave-uniform values the compiler would otherwise keep in vector registers and test lane by lane)
            adv_more = __builtin_amdgcn_readfirstlane(issue_kt + 1 < KT ? issue_live : 0);
            const int a_step = adv_more ? (FP6 ? kFp6Block : A_ROW) : 0;
            a_base += a_step;
            if constexpr (FP6) a_base2 += a_step;
            asm volatile("" : "+s"(adv_more), "+s"(a_base), "+s"(a_base2));
        } else if constexpr (PART == 1) {
            w_base += adv_more ? w_slice_stride : (int64_t)0;
            asm volatile("" : "+s"(w_base));
        } else {
            issue_tile = __builtin_amdgcn_readfirstlane(issue_tile + issue_live - adv_more);
            issue_kt = __builtin_amdgcn_readfirstlane(adv_more ? issue_kt + 1 : 0);
            asm volatile("" : "+s"(issue_kt), "+s"(issue_tile));
        }
    };
    auto issue_advance = [&] __device__() {
        issue_advance_part(I<0>{});
        issue_advance_part(I<1>{});
        issue_advance_part(I<2>{});
    };

    // ---- fragments.  MFMA operand row = lane % 32, K half = lane / 32.
    const int frow = lane & 31, fhalf = lane >> 5;
    // INT8 path: a step is 32 channels.  Code fragment: 16-byte chunk 2 s + fhalf of the row (xor swizzle);
    // weight fragment: 8 bytes at [32-row group][k32 step s][k16 half fhalf][row], widened to int8 lanes of 16 * code.
    // FP6 path: a step is 64 channels.  The 24-byte fragment 2 fhalf + s of a row is bytes 24 f .. 24 f + 23 of its
    // 96: step 0 takes chunk 3 fhalf whole ("head") and the lower half of chunk 3 fhalf + 1 ("tail"), step 1 the
    // upper half of that chunk (tail, the operand's first two registers) and chunk 3 fhalf + 2 whole (head).
    // A fragment set is 8 fragments in 16 parts (FP6: head and tail; INT8: the 4 code fragments count as one part
    // each, the 4 weight fragments as one part each, 8 parts); part p of the NEXT step is requested right behind
    // MFMA p of the current step.  With one wave per SIMD nothing but this interleaving keeps the matrix cores
    // fed: a wave issues about one instruction per 4 - 5 clocks, an MFMA occupies its pipe for 32, so every
    // MFMA can carry about six other instructions in its shadow, but only if they stand between MFMAs.
    // (FP6 operands are kept as whole 6-register vectors that the two reads of a fragment fill in halves: pieces
    // put together from separate 4- and 2-register members make the compiler widen loads across the members,
    // after which the set no longer lives in registers)
    struct FragsI8 { v4i a[TM]; v2i w[TN]; };
    struct FragsF6 { v6i a[TM]; v6i w[TN]; };
    using Frags = std::conditional_t<FP6, FragsF6, FragsI8>;
    const int a_frag_off = FP6 ? (wm / 32) * kFp6Block + fhalf * 1536 + frow * 16 : (wm + frow) * A_ROW;
    const int w_frag_off = FP6 ? A_STAGE + (wn / 32) * kFp6Block + fhalf * 1536 + frow * 16
                               : A_STAGE + (wn / kGroup) * kGroupBytes + frow * 8 + fhalf * 256;
    const int a_xor = swz_bk<A_ROW>(frow);
    constexpr int PARTS = FP6 ? 16 : 8;
    // request part P of the fragments of step S of the slice at LDS byte offset `off` (P, S compile-time: every
    // register of a fragment set keeps a fixed place)
    auto load_part = [&] __device__(Frags &f, uint32_t off, auto s_c, auto p_c) __attribute__((always_inline)) {
        constexpr int S = decltype(s_c)::value, P = decltype(p_c)::value;
        const uint8_t *st = smem + off;
        if constexpr (FP6) {
            // order: w0.h w0.t a0.h a0.t a1.h a1.t a2.h a2.t a3.h a3.t w1.h w1.t w2.h w2.t w3.h w3.t
            constexpr bool is_w = P < 2 || P >= 10;
            constexpr int idx = P < 2 ? 0 : (P < 10 ? (P - 2) / 2 : (P - 8) / 2);
            constexpr bool tail = P & 1;
            const uint8_t *q = st + (is_w ? w_frag_off : a_frag_off) + idx * kFp6Block;
            v6i v = is_w ? f.w[idx] : f.a[idx];
            if constexpr (!tail) {   // the whole chunk: registers 0-3 (step 0) or 2-5 (step 1) of the operand
                const v4i h = *reinterpret_cast<const v4i *>(q + (S == 0 ? 0 : 1024));
                constexpr int o = S == 0 ? 0 : 2;
                v[o] = h[0]; v[o + 1] = h[1]; v[o + 2] = h[2]; v[o + 3] = h[3];
            } else {                 // half of the middle chunk: registers 4-5 (step 0) or 0-1 (step 1)
                const v2i t = *reinterpret_cast<const v2i *>(q + (S == 0 ? 512 : 512 + 8));
                constexpr int o = S == 0 ? 4 : 0;
                v[o] = t[0]; v[o + 1] = t[1];
            }
            if constexpr (is_w) f.w[idx] = v;
            else f.a[idx] = v;
        } else {
            // order: w0 a0 a1 a2 a3 w1 w2 w3
            if constexpr (P >= 1 && P <= 4) {
                f.a[P - 1] = *reinterpret_cast<const v4i *>(st + a_frag_off + (P - 1) * 32 * A_ROW + (((S * 2 + fhalf) ^ a_xor) << 4));
            } else {
                constexpr int i = P == 0 ? 0 : P - 4;
                f.w[i] = *reinterpret_cast<const v2i *>(st + w_frag_off + i * kGroupBytes + S * 512);
            }
        }
    };
    auto widen = [] __device__(auto p) {   // INT8 path: two packed dwords (16 codes) -> int8 lanes of 16 * code, channel order
        if constexpr (sizeof(p) == sizeof(v2i)) {
            const uint32_t lo = (uint32_t)p[0], hi = (uint32_t)p[1];
            return v4i{(int)((lo << 4) & 0xF0F0F0F0u), (int)(lo & 0xF0F0F0F0u), (int)((hi << 4) & 0xF0F0F0F0u), (int)(hi & 0xF0F0F0F0u)};
        } else {
            return v4i{0, 0, 0, 0};
        }
    };

    // One step: 16 MFMAs on the fragment set `cur`.  Behind MFMA p: the caller's hook for slot p, then part p of step S_NXT of the slice at `nxt_off` into `nxt`,
    // and LDS-direct loads DMA0 .. DMA0 + DMA_N - 1 of the slice being issued, one every DMA_EVERY MFMAs from
    // MFMA DMA_FROM on.  INT8 path: the widened weights of the next group are formed behind a group's second MFMA.
    v4i fw_cur = {0, 0, 0, 0};   // INT8 path: widened weight fragment of the group being multiplied
    auto mfma_step = [&] __device__(auto first_c, const Frags &cur, Frags &nxt, uint32_t nxt_off, auto s_nxt_c, auto dma0_c,
                                    auto dma_n_c, auto dma_from_c, auto dma_every_c, auto &&hook) __attribute__((always_inline)) {
        constexpr bool FIRST = decltype(first_c)::value != 0;   // the tile's first step: the accumulators start from zero
        constexpr int DMA0 = decltype(dma0_c)::value, DMA_N = decltype(dma_n_c)::value;
        constexpr int DMA_FROM = decltype(dma_from_c)::value, DMA_EVERY = decltype(dma_every_c)::value;
        static_for<TN * TM>([&](auto p_c) __attribute__((always_inline)) {
            constexpr int P = decltype(p_c)::value, i = P / TM, j = P % TM;
            // (INT8 path: the s_nop variant covers the wait states between a VALU write of an operand -- the
            // widening -- and the MFMA, which the compiler cannot insert for an instruction it does not see)
            if constexpr (FP6) mfma_fp6_acc<P, FIRST, false>(cur.w[i], cur.a[j]);
            else mfma_i8_acc<P, FIRST, j == 0>(fw_cur, cur.a[j]);
            hook(p_c);   // the caller's bookkeeping for this slot (scalar work in the MFMA's shadow)
            // (FP6: a fragment's head and tail behind one MFMA, so the set is complete -- and the wait before the
            // slice barrier over -- half a step before the step ends)
            if constexpr (FP6 && 2 * P < PARTS) {
                load_part(nxt, nxt_off, s_nxt_c, I<2 * P>{});
                load_part(nxt, nxt_off, s_nxt_c, I<2 * P + 1>{});
            }
            if constexpr (!FP6 && P < PARTS) load_part(nxt, nxt_off, s_nxt_c, p_c);
            if constexpr (DMA_N > 0 && P >= DMA_FROM && (P - DMA_FROM) % DMA_EVERY == 0 && (P - DMA_FROM) / DMA_EVERY < DMA_N)
                issue_one(I<DMA0 + (P - DMA_FROM) / DMA_EVERY>{});
            if constexpr (!FP6 && j == TM - 1) {   // the next group's widened weights (the next step's first group after the last)
                if constexpr (i + 1 < TN) fw_cur = widen(cur.w[i + 1]);
                else fw_cur = widen(nxt.w[0]);
            }
            __builtin_amdgcn_sched_barrier(0);
        });
    };
    // ---- prologue: slices 0 and 1 on their way, slice 0 published, its first fragments requested
#pragma unroll
    for (int st = 0; st < STAGES - 1; ++st) {
        issue_prepare(st * STAGE);
        static_for<DMA>([&](auto d_c) __attribute__((always_inline)) { issue_one(d_c); });
        issue_advance();
    }
    wait_vmcnt<DMA>();
    before_barrier();
    __builtin_amdgcn_s_barrier();
    Frags f0, f1;
    static_for<PARTS>([&](auto p_c) __attribute__((always_inline)) { load_part(f0, 0u, I<0>{}, p_c); });
    if constexpr (!FP6) fw_cur = widen(f0.w[0]);

    // LDS byte offsets of the ring buffers holding slice q (being multiplied), q + 1 and q + 2 (being issued)
    uint32_t cur_off = 0, nxt_off = STAGE, fill_off = 2 * STAGE;
    // ACROSS: the first half of slice 2 is under way before the loop, like the halves issued behind a slice's last step
    if constexpr (ACROSS) {
        issue_prepare(fill_off);
        static_for<DMA / 2>([&](auto d_c) __attribute__((always_inline)) { issue_one(d_c); });
    }
    int store_credit = 0, tile_j = 0;
    for (;;) {
        for (int kt = 0; kt < KT; ++kt) {
            // Steps 0 .. last - 1 of slice q, loads of slice q + 2 dealt out between their MFMAs.  The scalar
            // bookkeeping of the load pipeline stands behind MFMAs as well: the addresses of a slice (it goes where
            // slice q - 1 was) behind the MFMA before its first load, the advance to the next behind MFMAs after its last.
            // (A tile's very first step starts its accumulators from zero: that step exists twice in the code.)
            auto none = [] __device__(auto) __attribute__((always_inline)) {};
            if constexpr (FP6) {
                // The path from L2 into LDS takes 64 bytes per clock and compute unit: the 48 KB of a slice cannot be
                // requested within one step (16 MFMAs, 512 clocks) without the load instructions backing up and
                // holding the MFMAs behind them.  So pieces 0-5 of slice q + 2 went out behind the last step of slice
                // q - 1 (its buffer was free from that slice's barrier on) and pieces 6-11 go out here, one every
                // other MFMA.  Across a tile boundary too (ACROSS): the epilogue stages the tile in the weight half of
                // the buffer that pieces 0-5, code blocks, are landing in meanwhile.  Tiles of one or two slices keep the
                // older order (nothing behind the tile's last slice, all twelve pieces here in its first): there a
                // slice-2 position is where the tile draws and tile numbers are read, timed by the barriers in between.
                if (kt == 0 && ACROSS) {
                    auto hook = [&] __device__(auto p_c) __attribute__((always_inline)) {
                        if constexpr (decltype(p_c)::value >= 12 && decltype(p_c)::value <= 14)
                            issue_advance_part(I<decltype(p_c)::value - 12>{});
                    };
                    mfma_step(I<1>{}, f0, f1, cur_off, I<1>{}, I<DMA / 2>{}, I<DMA / 2>{}, I<1>{}, I<2>{}, hook);
                } else if (kt == 0) {
                    auto hook = [&] __device__(auto p_c) __attribute__((always_inline)) {
                        if constexpr (decltype(p_c)::value == 0) issue_prepare(fill_off);
                        if constexpr (decltype(p_c)::value == 14) issue_advance();
                    };
                    mfma_step(I<1>{}, f0, f1, cur_off, I<1>{}, I<0>{}, I<DMA>{}, I<2>{}, I<1>{}, hook);
                } else {
                    auto hook = [&] __device__(auto p_c) __attribute__((always_inline)) {
                        if constexpr (decltype(p_c)::value >= 12 && decltype(p_c)::value <= 14)
                            issue_advance_part(I<decltype(p_c)::value - 12>{});
                    };
                    mfma_step(I<0>{}, f0, f1, cur_off, I<1>{}, I<DMA / 2>{}, I<DMA / 2>{}, I<1>{}, I<2>{}, hook);
                }
            } else {
                auto hook0 = [&] __device__(auto p_c) __attribute__((always_inline)) {
                    if constexpr (decltype(p_c)::value == 0) issue_prepare(fill_off);
                };
                auto hook2 = [&] __device__(auto p_c) __attribute__((always_inline)) {
                    if constexpr (decltype(p_c)::value == 15) issue_advance();
                };
                if (kt == 0) mfma_step(I<1>{}, f0, f1, cur_off, I<1>{}, I<0>{}, I<4>{}, I<8>{}, I<2>{}, hook0);
                else mfma_step(I<0>{}, f0, f1, cur_off, I<1>{}, I<0>{}, I<4>{}, I<8>{}, I<2>{}, hook0);
                mfma_step(I<0>{}, f1, f0, cur_off, I<2>{}, I<4>{}, I<4>{}, I<8>{}, I<2>{}, none);
                mfma_step(I<0>{}, f0, f1, cur_off, I<3>{}, I<8>{}, I<4>{}, I<8>{}, I<2>{}, hook2);
            }
            // Publish slice q + 1: it has landed once at most the loads of slice q + 2 (just issued) are
            // outstanding, plus, right after a full tile's epilogue, that tile's stores.  Every fragment read of
            // slice q has been issued; once they are back (lgkmcnt) and everyone is here, buffer q % 3 is free.
            if (__builtin_expect(store_credit > 0, 0)) {
                wait_vmcnt<DMA + STORES>();
                store_credit = 0;
            } else {
                wait_vmcnt<DMA>();
            }
            before_barrier();
            // (the barrier itself stands inside both branches below: the branch is then taken in the shadow of the
            // step's last MFMA, not between the barrier's release and the next step's first MFMA; the comments in
            // the asm statements keep the compiler from merging the two copies again)
            // the last step of slice q multiplies while step 0 of slice q + 1 is fetched (past the workgroup's
            // last slice: a stale but in-bounds buffer, never used)
            auto rotate = [&] __device__(auto p_c) __attribute__((always_inline)) {
                if constexpr (decltype(p_c)::value == 15) {   // (the step's reads of nxt_off have all been issued)
                    const uint32_t t = cur_off;
                    cur_off = nxt_off;
                    nxt_off = fill_off;
                    fill_off = t;
                }
            };
            if (FP6 && (ACROSS || kt + 1 < KT)) {
                asm volatile("; slice barrier, loads follow\n\ts_waitcnt lgkmcnt(0)" ::: "memory");
                __builtin_amdgcn_s_barrier();
                // FP6 path (tiles of one or two slices: not behind the tile's last slice): the barrier has freed the buffer of slice q, which takes slice
                // q + 3; its addresses (and, at a tile's start, the tile's vectors and the next draw) behind the first
                // MFMA, its pieces 0-5 behind every other MFMA from the third on
                auto early = [&] __device__(auto p_c) __attribute__((always_inline)) {
                    if constexpr (decltype(p_c)::value == 0) issue_prepare(cur_off);
                    rotate(p_c);
                };
                mfma_step(I<0>{}, f1, f0, nxt_off, I<0>{}, I<0>{}, I<DMA / 2>{}, I<2>{}, I<2>{}, early);
            } else {
                asm volatile("; slice barrier\n\ts_waitcnt lgkmcnt(0)" ::: "memory");
                __builtin_amdgcn_s_barrier();
                mfma_step(I<0>{}, f1, f0, nxt_off, I<0>{}, I<0>{}, I<0>{}, I<0>{}, I<1>{}, rotate);
            }
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
        comp_tile = tile_number(tile_j);   // the next one (its loads are under way)
        // INT8 path: the number of the tile after next, requested now and written into the ring in front of this
        // tile's first stores (behind them the compiler's wait for the reply would be the stores' round trip)
        const bool drawer = DRAW_IN_EPILOGUE && tiles.ctr && comp_tile >= 0 && wave == 0 && lane == 0;
        unsigned draw_reply = 0;
        if (drawer) draw_reply = tiles.draw();
        auto publish_draw = [&] __device__() {
            if (drawer) s_tiles[(tile_j + 1) & 7] = tiles.tile(draw_reply, 0);
        };
        const bool vec8 = (N & 7) == 0;
        const uint8_t *s_tile = smem + STAGES * STAGE + ((tile_j - 1) % 3) * SCALES;
        const float *s_xs = reinterpret_cast<const float *>(s_tile);
        const float *s_ws = s_xs + BM;
        const int32_t *s_rsum = reinterpret_cast<const int32_t *>(s_tile + OFF_RSUM);
        // sum q (c - z) = acc - z * rs with a 24-bit multiply (ranges: C ABI)
        auto unzero = [] __device__(int a, int z, int rs) { return a - __mul24(z, rs); };
        // staging: 4 KB per wave in the weight half of the buffer of the slice consumed last (next to be filled; on
        // the FP6 path its code half is already being filled with the next tile's slice 2 while the epilogue runs)
        uint8_t *stg = smem + fill_off + A_STAGE + wave * 4096;
        if (vec8 && !acc_out && m0 + BM <= M && n0 + BN <= N) {
            // ---- interior tile: no predicates; channel vectors fetched one register group ahead; the bf16 tile
            // is transposed through LDS, 32 tokens x 64 channels at a time, into whole-line streaming stores
            if (KT >= 2) store_credit = 1;
            // Four specializations (zero-points, bias), chosen once per tile: inside the unrolled units a run-time
            // test costs a branch each, and a lone wave per SIMD pays every taken branch with an idle front end.
            auto interior = [&] __device__(auto has_zero, auto has_bias) __attribute__((always_inline)) {
                // (scale, then add the bias, each rounded: a fused multiply-add would differ from the per-element path in the last bit)
#pragma clang fp contract(off)
                constexpr bool ZP = decltype(has_zero)::value, BIAS = decltype(has_bias)::value;
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
                    if constexpr (BIAS) cv.bb = *reinterpret_cast<const uint2 *>(bias_l + c / 2);
                    if constexpr (ZP) cv.zq = zero_l[c / 4];
                };
                // The 8 channel vectors of a pair of MFMA tile columns serve all TM token blocks: fetched once per pair
                // into registers (the operand fragments' registers are free here), not once per unit.
                ChannelVec cv[8];
                uint32_t pk[2][2];
                uint4 pend[4];            // a staged chunk on its way back from LDS, and where it goes
                uint16_t *pend_y = y;
                // 64 units of 4 values: unit u = ((ip * TM + j) * 2 + ii) * 4 + (g + h), MFMA tile column i = 2 ip + ii,
                // token block j, accumulator registers 4 (g + h) .. + 3; 8 units make a 32-token x 64-channel chunk
                static_for<(TN / 2) * TM * 8>([&](auto u_c) __attribute__((always_inline)) {
                    constexpr int U = decltype(u_c)::value, q = U & 3, h = U & 1, g = q - h, ii = (U >> 2) & 1;
                    constexpr int j = (U >> 3) % TM, ip = U / (8 * TM), i = 2 * ip + ii;
                    if constexpr (U % (8 * TM) == 0) {
#pragma unroll
                        for (int v = 0; v < 8; ++v) fetch(cv[v], 2 * ip + (v >> 2), v & 3);
                    }
                    const ChannelVec &c = cv[ii * 4 + q];
                    const v4i raw = read_acc4<i * TM + j, q>();
                    float o[4];
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if constexpr (ZP) {
                            const int z = (int)(int8_t)(c.zq >> (8 * e));
                            if constexpr (FP6) o[e] = (float)unzero((int)(__int_as_float(raw[e]) * kFp6Unit), z, rsum[j]) * xs_l[j];
                            else o[e] = (float)unzero(raw[e], z * (1 << SHIFT), rsum[j]) * xs_l[j];
                        } else {
                            if constexpr (FP6) o[e] = __int_as_float(raw[e]) * xs_l[j];
                            else o[e] = (float)raw[e] * xs_l[j];
                        }
                    }
                    o[0] *= c.ws.x;
                    o[1] *= c.ws.y;
                    o[2] *= c.ws.z;
                    o[3] *= c.ws.w;
                    if constexpr (BIAS) {
                        o[0] += __uint_as_float(c.bb.x << 16);
                        o[1] += __uint_as_float(c.bb.x & 0xFFFF0000u);
                        o[2] += __uint_as_float(c.bb.y << 16);
                        o[3] += __uint_as_float(c.bb.y & 0xFFFF0000u);
                    }
                    pk[h][0] = pack_bf16x2(o[0], o[1]);
                    pk[h][1] = pack_bf16x2(o[2], o[3]);
                    if constexpr (h == 1) {
                        // lanes l and l + 32 hold channels (8 g' .. + 3) and (8 g' + 4 .. + 7): after the swap each lane
                        // owns 8 consecutive channels
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
                    // A staged chunk is read back right away (its LDS round trip then runs under the next chunk's
                    // arithmetic; a wave's LDS instructions execute in order, so the next chunk's writes into the
                    // same area stay behind these reads) and stored to memory half a chunk later.
                    if constexpr (U == 11) publish_draw();
                    if constexpr ((U & 7) == 3 && U > 8) {
#pragma unroll
                        for (int pass = 0; pass < 4; ++pass) store_streaming16(pend_y + (int64_t)pass * 8 * N, pend[pass]);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    if constexpr ((U & 7) == 7) {   // the chunk is staged: whole rows back, 8 lanes per 128-byte row
                        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                        __builtin_amdgcn_wave_barrier();
                        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                        pend_y = y + (int64_t)(m0 + wm + j * 32 + rd_row) * N + (n0 + wn + ip * 64 + rd_piece * 8);
                        const uint8_t *sg = stg;
#pragma unroll
                        for (int pass = 0; pass < 4; ++pass) {
                            const int row = pass * 8 + rd_row;
                            pend[pass] = *reinterpret_cast<const uint4 *>(sg + row * 128 + ((rd_piece ^ (row & 7)) << 4));
                        }
                        __builtin_amdgcn_wave_barrier();   // later LDS writes into this area stay behind these reads
                        __builtin_amdgcn_sched_barrier(0);
                    }
                });
#pragma unroll
                for (int pass = 0; pass < 4; ++pass) store_streaming16(pend_y + (int64_t)pass * 8 * N, pend[pass]);   // the last chunk
            };
            if (w_zero) {
                if (bias) interior(std::true_type{}, std::true_type{});
                else interior(std::true_type{}, std::false_type{});
            } else {
                if (bias) interior(std::false_type{}, std::true_type{});
                else interior(std::false_type{}, std::false_type{});
            }
        } else {
            // ---- edge tiles, N not a multiple of 8, or the accumulator hook: predicated per element, through the
            // integer accumulator (same values and rounding order as the interior path)
            int lane_s = lane;
            asm volatile("" : "+v"(lane_s));
            const int frow = lane_s & 31, fhalf = lane_s >> 5;
            static_for<TM * TN>([&](auto t_c) __attribute__((always_inline)) {
                constexpr int j = decltype(t_c)::value / TN, i = decltype(t_c)::value % TN;
                const int m = m0 + wm + j * 32 + frow;
                const bool m_ok = m < M;
                const float xs = s_xs[wm + j * 32 + frow];
                const int rs = w_zero ? s_rsum[wm + j * 32 + frow] : 0;
                const int nb = n0 + wn + i * 32;   // this MFMA tile's first output channel
                int a[16];
                static_for<4>([&](auto g_c) __attribute__((always_inline)) {
                    constexpr int g = decltype(g_c)::value;
                    const v4i raw = read_acc4<i * TM + j, g>();
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int n = nb + g * 8 + fhalf * 4 + e;
                        if constexpr (FP6) a[g * 4 + e] = (int)(__int_as_float(raw[e]) * kFp6Unit);
                        else a[g * 4 + e] = raw[e] >> SHIFT;
                        if (w_zero && n < N) a[g * 4 + e] = unzero(a[g * 4 + e], (int)w_zero[n], rs);
                    }
                });
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
            });
            publish_draw();
        }
        if (comp_tile < 0) break;
        // the staging buffer is the one the next slice's loads go to: nobody may issue them before everyone
        // has stored its part of the tile (the same barrier makes a ring entry written in the epilogue visible)
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        __builtin_amdgcn_s_barrier();
    }
    wait_vmcnt<0>();   // no LDS-direct load may still be in flight when the workgroup's LDS is released
}

namespace {

template <bool FP6, bool ACROSS>
int launch_wide(const uint8_t *codes, const float *x_scale, const uint8_t *w, const float *w_scale, const int8_t *w_zero,
                const int32_t *code_rowsum, const uint16_t *bias, int M, int N, int K, uint16_t *y, int32_t *acc_out,
                hipStream_t stream) {
    constexpr int BM = 256, BN = 256, STAGES = 3;
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    // Column tiles per L2 sharing group (the 32 workgroups of an XCD then work on about 32 / group_n token panels
    // x group_n channel panels at a time, so a width near 6 pulls the fewest panels through the XCD's L2).
    // Measured on the DiT shapes (whole layer steps): groups of 12, 18 or 20 columns cost 4-9 % against groups of
    // 5-10; equal groups that split the columns among the 8 XCDs' tile ranges evenly (1, 2, 4 or 8 groups) are as
    // fast as any width in that range, groups of unequal width (7, 7, 6 of 20 columns; 5, 5, 2 of 12) lose 2-5 %
    // again; between 5 and 10 columns of 20 the time is the same and the L2 fetches differ by a fifth.  So: that
    // many equal groups of at most 10 columns, the width nearest 6, where the column count allows it; else balanced
    // groups of at most 16.
    int n_groups = (tiles_n + 15) / 16;
    for (int g = 1, best = 1 << 30; g <= 8; g *= 2) {
        const int width = tiles_n / g, off = width > 6 ? width - 6 : 6 - width;
        if (tiles_n % g == 0 && width <= 10 && off < best) {
            best = off;
            n_groups = g;
        }
    }
    const int group_n = (tiles_n + n_groups - 1) / n_groups;
    const int total = tiles_m * tiles_n;
    int grid = 256;
    if (total < grid) grid = (total + 7) / 8 * 8;
    grid = limited_grid(grid);
    const size_t smem = (size_t)STAGES * 48 * 1024 + 3 * ((BM + BN) * 4 + BN * 2 + BM * 4 + BN) + 8 * sizeof(int);
    auto k = w4ax_gemm_wide_kernel<FP6, ACROSS>;
    static std::atomic<uint64_t> configured{0};
    allow_dynamic_lds(reinterpret_cast<const void *>(k), smem, configured);
    bool is_clear = false;
    unsigned *sched = sched_slot(stream, &is_clear);
    if (K / kBK < 2) sched = nullptr;   // a tile draw takes two slices to come back
    if (sched && !is_clear && clear_sched_slot(sched, stream) != DVDQ_OK) return DVDQ_ERR_HIP;
    hipLaunchKernelGGL(k, dim3((unsigned)grid), dim3(256), smem, stream, codes, x_scale, w, w_scale, w_zero, code_rowsum,
                       bias, M, N, K, y, acc_out, tiles_m, tiles_n, group_n, sched);
    return check_launch();
}

}  // namespace

int launch_w4ax_gemm_wide(const uint8_t *codes, const float *x_scale, const uint8_t *w, const float *w_scale,
                          const int8_t *w_zero, const int32_t *code_rowsum, const uint16_t *bias, int64_t M, int64_t N,
                          int64_t K, bool fp6, uint16_t *y, int32_t *acc_out, hipStream_t stream) {
    if (fp6 && K / kBK >= 3)
        return launch_wide<true, true>(codes, x_scale, w, w_scale, w_zero, code_rowsum, bias, (int)M, (int)N, (int)K, y,
                                       acc_out, stream);
    if (fp6)
        return launch_wide<true, false>(codes, x_scale, w, w_scale, w_zero, code_rowsum, bias, (int)M, (int)N, (int)K, y,
                                        acc_out, stream);
    return launch_wide<false, false>(codes, x_scale, w, w_scale, w_zero, code_rowsum, bias, (int)M, (int)N, (int)K, y, acc_out,
                                     stream);
}

}  // namespace dvdq

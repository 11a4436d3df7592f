// W4A4 GEMM on the FP6 matrix path of gfx950 (Sec. 3.2: Y = X^ Lambda W^^T with 4-bit codes on both
// sides; Sec. 3.1 DeQuant, optional zero-points).
//
// Why FP6.  CDNA4 has no INT4 matrix instruction.  Its f8f6f4 MFMAs run 6-bit operands at twice the
// INT8 rate, and the E2M3 format represents the integers a 4-bit code can take exactly: the value of
// the bit pattern (sign << 5 | m), 0 <= m <= 15, is +-m / 8 (m < 8 are the format's subnormals, m >= 8
// has exponent field 1 and mantissa m - 8).  Products of two such values are multiples of 1/64 and
// their fp32 sum is exact while |sum of code products| < 2^24 (checked by the C ABI), so the fp32
// accumulator times 64 IS the integer accumulator of the INT8 path, bit for bit.  There is no operand
// widening in registers at all; the price is 6 instead of 4 bits per code in LDS and in HBM.
//
// Operand layout ("FP6 native", for the weights written by the prepack kernel below and for the
// activation codes by the quantizer): K in slices of 128 channels, rows in blocks of 32.  One
// block-slice is 3072 bytes: [16-byte chunk c = 0..5][row 0..31][16 B], where the 96 bytes
// (c = 0..5) of a row hold its 128 codes of the slice as 6-bit fields, field e of 24-byte fragment
// f = 2 h + s at bit 6 e, for channel 64 h + 32 s + e of the slice.  h is the MFMA's K half (lane / 32),
// s the 64-channel step: a lane's two fragments of a slice are 48 contiguous bytes = three 16-byte
// chunks, read from LDS as three conflict-free ds_read_b128 (8 lanes = 8 rows = 128 contiguous bytes)
// straight into the 12 registers the two MFMAs take their operands from.  Weights: slices outermost,
// then the 32-row groups of N (padded to 256).  Codes: row blocks outermost, then slices (rows padded
// to 32).  Either way a tile's slice is a few linear runs, copied HBM/L2 -> LDS by LDS-direct loads.
//
// Everything else (ring of LDS buffers, hand-kept vmcnt, persistent workgroups drawing tiles, staged
// whole-line epilogue) is the design of the INT8 kernel in w4ax_gemm.hip.
#include <type_traits>

#include "gemm_common.h"

namespace dvdq {

namespace {

typedef int v8i __attribute__((ext_vector_type(8)));

constexpr int kFp6RowBytes = kBK * 6 / 8;              // 96: one row's codes of one K slice
constexpr int kFp6Block = kGroup * kFp6RowBytes;       // 3072: 32 rows of one K slice
constexpr float kFp6Unit = 64.f;                       // accumulator * 64 = integer sum of code products

}  // namespace

template <int BM, int BN, int WAVES_M, int WAVES_N, int STAGES, int OCC>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N, OCC) void w4a4_fp6_gemm_kernel(
    const uint8_t *__restrict__ codes, const float *__restrict__ x_scale, const uint8_t *__restrict__ w,
    const float *__restrict__ w_scale, const int8_t *__restrict__ w_zero, const int32_t *__restrict__ code_rowsum,
    const uint16_t *__restrict__ bias, int M, int N, int K, uint16_t *__restrict__ y, int32_t *__restrict__ acc_out,
    int tiles_m, int tiles_n, int group_n, unsigned *__restrict__ sched) {
    constexpr int NW = WAVES_M * WAVES_N;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;  // wave sub-tile
    constexpr int TM = WM / 32, TN = WN / 32;            // MFMA tiles per wave
    constexpr int A_STAGE = BM / 32 * kFp6Block, W_STAGE = BN / 32 * kFp6Block, STAGE = A_STAGE + W_STAGE;
    constexpr int A_DMA = 3;                             // one 32-row block of codes (3 KB) per wave and item
    constexpr int W_DMA = W_STAGE / 1024 / NW;
    constexpr int DMA = A_DMA + W_DMA;
    constexpr int GROUPS = 2 * TN;                       // MFMA groups (TM MFMAs each) per item
    constexpr int DMA_PER_GROUP = 2;                     // the next slice's loads go out with the first MFMA groups
    static_assert(GROUPS * DMA_PER_GROUP >= DMA, "not every load of an item would be issued");
    // one tile's epilogue vectors in LDS: token scales, channel scales (fp32), bias (bf16), and for
    // weights with zero-points the tokens' code sums (int32) and the channels' zero-points (int8)
    typedef TileVectors<BM, BN> TV;
    constexpr int OFF_BIAS = TV::OFF_BIAS, OFF_RSUM = TV::OFF_RSUM, OFF_ZERO = TV::OFF_ZERO, SCALES = TV::BYTES;
    constexpr int STORES = TM * TN * 2;                  // 16-byte store instructions per wave per full tile
    static_assert(BM / 32 == NW, "one block of code rows per wave");
    static_assert(W_DMA >= 1 && W_DMA * 1024 * NW == W_STAGE, "weight tile does not split over the waves");
    static_assert(STAGES >= 2 && (STAGES - 1) * DMA < 64, "too many loads in flight for vmcnt");
    static_assert((STAGES - 2) * DMA + STORES < 64, "store-aware wait exceeds vmcnt");
    static_assert(NW * 4096 <= STAGE && TN % 2 == 0, "the epilogue stages 4 KB per wave in one ring buffer");

    extern __shared__ __align__(16) uint8_t smem[];
    const uint32_t smem_base = lds_address(smem);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = (wave % WAVES_M) * WM, wn = (wave / WAVES_M) * WN;
    const int KT = K / kBK;
    const int G = ((N + kNPad - 1) / kNPad) * (kNPad / kGroup);  // 32-row groups in the padded weight buffer
    const int64_t w_slice_stride = (int64_t)G * kFp6Block;
    const int last_block = (M - 1) / 32;                         // code row blocks past it do not exist

    // Persistent workgroups draw their tiles exactly as in the INT8 kernel (see there, and TileSource): per-XCD
    // counters, fixed shares when sched is null; tile numbers travel through an 8-entry ring in LDS.
    const TileSource tiles(tiles_m, tiles_n, sched);
    typedef volatile __attribute__((address_space(3))) int lds_int;
    lds_int *s_tiles = (lds_int *)DVDQ_LDS(smem + STAGES * STAGE + 2 * SCALES);
    int draws = 0;
    unsigned drawn = 0;
    bool draw_pending = false;
    int draw_wait = 0;   // loop tops until the pending draw's reply is older than loads already awaited
    auto draw = [&] __device__() {
        if (wave == 0 && tiles.ctr && lane == 0) drawn = tiles.draw();
        ++draws;
        draw_pending = true;
        draw_wait = STAGES - 1;
    };
    auto publish_draw = [&] __device__() {   // before a workgroup barrier
        if (wave == 0) {
            if (lane == 0) s_tiles[(draws - 1) & 7] = tiles.tile(drawn, draws - 1);
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }
        draw_pending = false;
    };
    if (wave == 0 && lane == 0) {
        int t0, t1;
        tiles.first_two(t0, t1);
        s_tiles[0] = t0;
        s_tiles[1] = t1;
    }
    draws = 2;
    __syncthreads();
    int comp_tile = __builtin_amdgcn_readfirstlane(s_tiles[0]);
    if (comp_tile < 0) return;   // (whole workgroup: nothing below is reached, no barrier is missed)

    // ---- LDS-direct loads: every piece is 1 KB that is contiguous in memory and in LDS, so a lane's
    // offset is 16 * lane on both sides and the rest is wave-uniform.  Codes: this wave's row block of
    // the tile (blocks past the last one repeat it; their rows are never stored).  Weights: the tile's
    // 8 groups of a slice are one 24 KB run.
    const uint32_t lane16 = lane * 16;
    const uint8_t *a_base = codes;   // this wave's code block, slice issue_kt
    const uint8_t *w_base = w;       // the tile's weight run, slice issue_kt
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
            a_base = uniform_ptr(codes + (int64_t)min(m0 / 32 + wave, last_block) * KT * kFp6Block);
            w_base = uniform_ptr(w + (int64_t)(n0 / kGroup) * kFp6Block + wave * W_DMA * 1024);   // (this wave's pieces)
            const uint32_t sc = smem_base + STAGES * STAGE + (issue_tile & 1) * SCALES;
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
    // Piece idx of the wave's DMA (a constant wherever it is called: the switch folds away).  The code pieces and
    // the weight pieces are runs whose source and destination both advance by 1 KB: the first of a run sets M0,
    // the others reuse it and move by the instruction offset (weight pieces 4 .. through a second lane offset).
    static_assert(A_DMA == 3 && W_DMA <= 8, "piece runs");
    const uint32_t lane16_hi = lane16 + 4096;
    auto issue_one = [&] __device__(int idx) __attribute__((always_inline)) {
        const uint32_t sa_a = issue_sa + wave * A_DMA * 1024, sa_w = issue_sa + A_STAGE + wave * W_DMA * 1024;
        switch (idx) {
            case 0: lds_direct_load16(a_base, lane16, sa_a); break;
            case 1: lds_direct_load16_more<1024>(a_base, lane16); break;
            case 2: lds_direct_load16_more<2048>(a_base, lane16); break;
            case 3: lds_direct_load16(w_base, lane16, sa_w); break;
            case 4: lds_direct_load16_more<1024>(w_base, lane16); break;
            case 5: lds_direct_load16_more<2048>(w_base, lane16); break;
            case 6: lds_direct_load16_more<3072>(w_base, lane16); break;
            case 7: lds_direct_load16(w_base, lane16_hi, sa_w + 4096); break;
            case 8: lds_direct_load16_more<1024>(w_base, lane16_hi); break;
            case 9: lds_direct_load16_more<2048>(w_base, lane16_hi); break;
            default: lds_direct_load16_more<3072>(w_base, lane16_hi); break;
        }
    };
    auto issue_advance = [&] __device__() {
        if (!issue_live) return;
        if (issue_kt + 1 < KT) {
            a_base += kFp6Block;
            w_base += w_slice_stride;
            ++issue_kt;
        } else {   // next: slice 0 of the next tile, whose addresses issue_prepare sets (or none: stay on this slice)
            issue_kt = 0;
            ++issue_tile;
        }
    };

    v16f acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    // ---- fragment addressing: MFMA operand row = lane % 32, K half = lane / 32
    const int frow = lane & 31, fhalf = lane >> 5;
    const int frag_off = fhalf * 1536 + frow * 16;   // chunks 3 h .. 3 h + 2 of the row, 512 bytes apart

    // ---- prologue: fill STAGES - 1 buffers
#pragma unroll
    for (int st = 0; st < STAGES - 1; ++st) {
        issue_prepare(st);
#pragma unroll
        for (int d = 0; d < DMA; ++d) issue_one(d);
        issue_advance();
    }

    int kt = 0, tile_j = 0, store_credit = 0;
    for (int q = 0;; ++q) {
        // Publish slice q (it has landed once at most the loads of the STAGES - 2 younger slices are
        // outstanding: a wave's vector memory operations complete in issue order); the barrier also means
        // that everyone is done reading slice q-1, whose buffer the next loads overwrite.  Right after the
        // epilogue of a full tile exactly STORES stores are this wave's youngest operations (for the next
        // STAGES - 1 slices the awaited loads are older than them): their acknowledgement is not awaited.
        if (store_credit > 0) {
            wait_vmcnt<(STAGES - 2) * DMA + STORES>();
            --store_credit;
        } else {
            wait_vmcnt<(STAGES - 2) * DMA>();
        }
        if (draw_pending && --draw_wait == 0) publish_draw();
        __builtin_amdgcn_s_barrier();
        issue_prepare((q + STAGES - 1) % STAGES);
        if (kt == 0) __builtin_amdgcn_s_setprio(2);

        // The slice's fragments: per operand row three 16-byte chunks = the 12 registers of the two
        // steps' operands.  All are requested up front (chunks 0 and 1, which step 0 needs, first); the
        // LDS-direct loads of the next slice are dealt out between the MFMA groups.
        const uint8_t *sa = smem + (q % STAGES) * STAGE + (wm / 32) * kFp6Block + frag_off;
        const uint8_t *sw = smem + (q % STAGES) * STAGE + A_STAGE + (wn / 32) * kFp6Block + frag_off;
        v4i ra[TM][3], rw[TN][3];
#pragma unroll
        for (int c = 0; c < 3; ++c) {
#pragma unroll
            for (int j = 0; j < TM; ++j) ra[j][c] = *reinterpret_cast<const v4i *>(sa + j * kFp6Block + c * 512);
#pragma unroll
            for (int i = 0; i < TN; ++i) rw[i][c] = *reinterpret_cast<const v4i *>(sw + i * kFp6Block + c * 512);
            if (c == 0) continue;   // (chunks 0 and 1 go out together)
            __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int s = 0; s < 2; ++s) {
            v8i fa[TM];
#pragma unroll
            for (int j = 0; j < TM; ++j)
                fa[j] = s == 0 ? v8i{ra[j][0][0], ra[j][0][1], ra[j][0][2], ra[j][0][3], ra[j][1][0], ra[j][1][1], 0, 0}
                               : v8i{ra[j][1][2], ra[j][1][3], ra[j][2][0], ra[j][2][1], ra[j][2][2], ra[j][2][3], 0, 0};
#pragma unroll
            for (int i = 0; i < TN; ++i) {
                const v8i fw = s == 0 ? v8i{rw[i][0][0], rw[i][0][1], rw[i][0][2], rw[i][0][3], rw[i][1][0], rw[i][1][1], 0, 0}
                                      : v8i{rw[i][1][2], rw[i][1][3], rw[i][2][0], rw[i][2][1], rw[i][2][2], rw[i][2][3], 0, 0};
#pragma unroll
                for (int j = 0; j < TM; ++j)   // both operands FP6 E2M3 (format code 2), no block scales
                    acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fw, fa[j], acc[i][j], 2, 2, 0, 0, 0, 0);
#pragma unroll
                for (int d = (s * TN + i) * DMA_PER_GROUP; d < DMA && d < (s * TN + i + 1) * DMA_PER_GROUP; ++d) issue_one(d);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        issue_advance();
        if (++kt < KT) continue;
        __builtin_amdgcn_s_setprio(0);

        // ---- epilogue of tile comp_tile (shared with the INT8 kernel: see epilogue_interior / epilogue_edge; here
        // the fp32 accumulators hold the integer sum / 64, exactly: see the top of this file)
        int m0, n0;
        tile_origin(comp_tile, tiles_m, tiles_n, group_n, BM, BN, m0, n0);
        kt = 0;
        ++tile_j;
        comp_tile = __builtin_amdgcn_readfirstlane(s_tiles[tile_j & 7]);   // the next one (its loads are under way)
        const uint8_t *s_tile = smem + STAGES * STAGE + ((tile_j - 1) & 1) * SCALES;
        // Lane-dependent addresses of the epilogue are derived from a lane number the compiler cannot trace
        // back: computed here once per tile instead of being kept (and spilled) across the K loop.
        int lane_e = lane;
        asm volatile("" : "+v"(lane_e));
        if ((N & 7) == 0 && !acc_out && m0 + BM <= M && n0 + BN <= N) {
            if (KT >= STAGES) store_credit = STAGES - 1;
            uint8_t *stg = smem + (q % STAGES) * STAGE + wave * 4096;
            __builtin_amdgcn_s_barrier();   // every wave is done reading the last slice: its buffer stages the tile
            if (w_zero) {
                if (bias) epilogue_interior<AccF32x64, BM, BN, TM, TN, true, 1>(acc, s_tile, true, lane_e, wm, wn, stg, y, m0, n0, N);
                else epilogue_interior<AccF32x64, BM, BN, TM, TN, true, 0>(acc, s_tile, true, lane_e, wm, wn, stg, y, m0, n0, N);
            } else {
                if (bias) epilogue_interior<AccF32x64, BM, BN, TM, TN, false, 1>(acc, s_tile, true, lane_e, wm, wn, stg, y, m0, n0, N);
                else epilogue_interior<AccF32x64, BM, BN, TM, TN, false, 0>(acc, s_tile, true, lane_e, wm, wn, stg, y, m0, n0, N);
            }
        } else {
            epilogue_edge<AccF32x64, BM, BN, TM, TN>(acc, s_tile, bias, w_zero, lane_e, wm, wn, y, acc_out, m0, n0, M, N);
        }
        if (comp_tile < 0) break;
    }
    wait_vmcnt<0>();   // no LDS-direct load may still be in flight when the workgroup's LDS is released
}

namespace {

// canonical [N, K/2] (two signed 4-bit codes per byte, low nibble first) -> FP6 native layout (see the top
// of this file).  One thread per 24-byte fragment (32 codes of one row).  Rows >= N are written as zero.
__global__ __launch_bounds__(256) void w4_prepack_fp6_kernel(const uint8_t *__restrict__ src, uint32_t *__restrict__ dst,
                                                             int N, int K, int G, int KT) {
    const int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t frags = (int64_t)KT * G * kGroup * 4;
    if (o >= frags) return;
    int64_t v = o;
    const int f = (int)(v & 3); v >>= 2;       // fragment 2 h + s of the row's slice
    const int r = (int)(v & 31); v >>= 5;
    const int g = (int)(v % G);
    const int kt = (int)(v / G);
    const int n = g * kGroup + r;
    const int k = kt * kBK + (f >> 1) * 64 + (f & 1) * 32;   // first channel of the fragment
    uint32_t out[6] = {0, 0, 0, 0, 0, 0};
    if (n < N) {
        const uint4 p = *reinterpret_cast<const uint4 *>(src + (int64_t)n * (K / 2) + k / 2);
        const uint32_t q[4] = {p.x, p.y, p.z, p.w};
        uint64_t lo = 0, mid = 0, hi = 0;      // 192 bits, 64 each
#pragma unroll
        for (int e = 0; e < 32; ++e) {
            const int c = (int)(q[e >> 3] << (28 - 4 * (e & 7))) >> 28;          // signed nibble e
            const uint64_t field = (uint64_t)((c < 0 ? 32 : 0) | (c < 0 ? -c : c));
            const int bit = 6 * e;
            if (bit < 64) { lo |= field << bit; if (bit > 58) mid |= field >> (64 - bit); }
            else if (bit < 128) { mid |= field << (bit - 64); if (bit > 122) hi |= field >> (128 - bit); }
            else hi |= field << (bit - 128);
        }
        out[0] = (uint32_t)lo; out[1] = (uint32_t)(lo >> 32); out[2] = (uint32_t)mid;
        out[3] = (uint32_t)(mid >> 32); out[4] = (uint32_t)hi; out[5] = (uint32_t)(hi >> 32);
    }
    // byte b of the row's 96 bytes lives in chunk b / 16 at [chunk][row][b % 16]
    uint32_t *blk = dst + ((int64_t)kt * G + g) * (kFp6Block / 4);
#pragma unroll
    for (int d = 0; d < 6; ++d) {
        const int b = f * 24 + d * 4;
        blk[(b / 16) * (kGroup * 4) + r * 4 + (b % 16) / 4] = out[d];
    }
}

template <int BM, int BN, int WAVES_M, int WAVES_N, int STAGES, int OCC>
int launch_fp6(const uint8_t *codes, const float *x_scale, const uint8_t *w, const float *w_scale, const int8_t *w_zero,
               const int32_t *code_rowsum, const uint16_t *bias, int M, int N, int K, uint16_t *y, int32_t *acc_out,
               hipStream_t stream) {
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    // column tiles are walked in groups of at most 16, so that workgroups at work at the same time share
    // weight panels in the L2s (2 to 16 measured within 3 % of each other)
    constexpr int kMaxGroupN = 16;
    const int n_groups = (tiles_n + kMaxGroupN - 1) / kMaxGroupN;
    const int group_n = (tiles_n + n_groups - 1) / n_groups;
    const int total = tiles_m * tiles_n;
    int grid = 256 * OCC;
    if (total < grid) grid = (total + 7) / 8 * 8;
    grid = limited_grid(grid);
    const size_t smem = (size_t)STAGES * (BM / 32 + BN / 32) * kFp6Block + 2 * ((BM + BN) * 4 + BN * 2 + BM * 4 + BN) +
                        8 * sizeof(int);
    auto k = w4a4_fp6_gemm_kernel<BM, BN, WAVES_M, WAVES_N, STAGES, OCC>;
    static std::atomic<uint64_t> configured{0};
    allow_dynamic_lds(reinterpret_cast<const void *>(k), smem, configured);
    bool is_clear = false;
    unsigned *sched = sched_slot(stream, &is_clear);
    if (sched && !is_clear && clear_sched_slot(sched, stream) != DVDQ_OK) return DVDQ_ERR_HIP;
    hipLaunchKernelGGL(k, dim3((unsigned)grid), dim3(64 * WAVES_M * WAVES_N), smem, stream, codes, x_scale, w, w_scale,
                       w_zero, code_rowsum, bias, M, N, K, y, acc_out, tiles_m, tiles_n, group_n, sched);
    return check_launch();
}

}  // namespace

int launch_w4a4_fp6_gemm(const uint8_t *codes, const float *x_scale, const uint8_t *w, const float *w_scale,
                         const int8_t *w_zero, const int32_t *code_rowsum, const uint16_t *bias, int64_t M, int64_t N,
                         int64_t K, uint16_t *y, int32_t *acc_out, hipStream_t stream) {
#define DVDQ_FP6_ARGS codes, x_scale, w, w_scale, w_zero, code_rowsum, bias, (int)M, (int)N, (int)K, y, acc_out, stream
    // Tile variants {tile M, tile N, waves M x N, ring depth, workgroups per compute unit}:
    //   1: two independent 4-wave workgroups per compute unit, 128 x 256 tiles, two buffers: while one
    //      converts and stores a tile the other multiplies;
    //   2: one 8-wave workgroup, 256 x 256 tiles, three buffers: a third fewer LDS-direct bytes per MFMA and
    //      one more slice of prefetch distance, which is what this kernel is short of (it is bound by the
    //      path from L2 / HBM into LDS, not by the matrix cores); 3-11 % faster on the DiT shapes although
    //      no second workgroup hides its epilogue.  Taken when there are at least two rounds of such tiles
    //      and K is deep enough for the ring; the benchmark hook can force either.
    //   3: the wide kernel of w4ax_gemm_wide.hip: one 4-wave workgroup, 256 x 256 tiles, 128 x 128 wave tiles with
    //      the accumulators in AGPRs: a third fewer LDS fragment bytes per MFMA and a K slice in 60 % of
    //      variant 2's time, but a larger fixed cost per tile (nothing hides its epilogue), so it pays from
    //      ten K slices on (whole layer steps on a 32760 x 4608 output, variant 3 against variant 2: 14 %
    //      slower at K = 512, 5 % at 768, equal at 1024, 3 % faster at 1280, 7 % at 1536, 8 % at 2048).
    int v = gemm_variant();
    const int64_t big_tiles = ((M + 255) / 256) * ((N + 255) / 256);
    if (v != 1 && v != 2 && v != 3) v = big_tiles >= 512 ? (K / kBK >= 10 ? 3 : 2) : 1;
    if (K / kBK < 2 && v == 2) v = 1;
    if (v == 3) return launch_w4ax_gemm_wide(codes, x_scale, w, w_scale, w_zero, code_rowsum, bias, M, N, K, true, y, acc_out, stream);
    if (v == 2) return launch_fp6<256, 256, 4, 2, 3, 1>(DVDQ_FP6_ARGS);
    return launch_fp6<128, 256, 2, 2, 2, 2>(DVDQ_FP6_ARGS);
#undef DVDQ_FP6_ARGS
}

size_t w4_native_fp6_bytes(int64_t N, int64_t K) {
    const int64_t npad = (N + kNPad - 1) / kNPad * kNPad, kpad = (K + kBK - 1) / kBK * kBK;
    return (size_t)(npad * kpad * 6 / 8);
}

size_t codes_fp6_bytes(int64_t M, int64_t K) {
    const int64_t mpad = (M + 31) / 32 * 32, kpad = (K + kBK - 1) / kBK * kBK;
    return (size_t)(mpad * kpad * 6 / 8);
}

int launch_w4_prepack_fp6(const uint8_t *w_canonical, int64_t N, int64_t K, uint8_t *w_native, hipStream_t stream) {
    const int G = (int)((N + kNPad - 1) / kNPad * (kNPad / kGroup));
    const int KT = (int)(K / kBK);
    const int64_t frags = (int64_t)KT * G * kGroup * 4;
    const int64_t blocks = (frags + 255) / 256;
    hipLaunchKernelGGL(w4_prepack_fp6_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, w_canonical,
                       reinterpret_cast<uint32_t *>(w_native), (int)N, (int)K, G, KT);
    return check_launch();
}

}  // namespace dvdq

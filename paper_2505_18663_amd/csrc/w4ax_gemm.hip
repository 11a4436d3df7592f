// W4Ax GEMM for gfx950, fast path for pre-packed ("native") weights: int8
// activation codes x packed INT4 weights on the INT8 matrix cores, exact int32
// accumulation, dequantizing epilogue to bf16 (Sec. 3.2: Y = X^ Lambda W^^T;
// Sec. 3.1 DeQuant with zero-point 0).
//
// Data movement.  Both operands travel HBM/L2 -> LDS with LDS-direct loads
// (16 bytes per lane, no VGPR staging) through a ring of STAGES buffers; K is
// consumed in slices of 128.  Completion is tracked by hand with s_waitcnt vmcnt
// because the compiler does not order LDS reads after LDS-direct loads.
//   codes  : [row][128 B], the 16-byte chunk index xor-ed with (row & 7), so the 8 lanes
//            that read the same chunk of 8 consecutive rows cover a whole 128-byte LDS
//            bank line; a wave's load instruction covers 8 full 128-byte rows.
//   weights: stay packed (two codes per byte) in LDS; the native layout is the LDS
//            image itself, so a slice is one linear, fully coalesced copy:
//            [k128 slice][32-row group][k32 step][k16 half][row][8 B].
//            The 8 bytes hold 16 consecutive channels; byte b of dword d carries
//            channel 8d+b in its low and channel 8d+b+4 in its high nibble, so that
//            (p << 4) & 0xF0F0F0F0 and p & 0xF0F0F0F0 are int8 lanes of 16*code in
//            channel order.  The MFMA then accumulates 16*acc exactly; the factor
//            is folded into the token scale (a power of two) or shifted out.
//
// Compute.  A workgroup of WAVES_M x WAVES_N waves owns a BM x BN tile; a wave a
// (BM/WAVES_M) x (BN/WAVES_N) sub-tile of 32x32x32 MFMAs.  The weight fragment is
// the MFMA's row operand and the code fragment its column operand, so a lane holds
// 4 consecutive output channels of one token; lane halves are exchanged
// (v_permlane32_swap) so that every lane stores 16 contiguous bytes of bf16.
#include <mutex>
#include <type_traits>
#include <unordered_map>
#include <vector>

#include "gemm_common.h"

namespace dvdq {

template <int BM, int BN, int BK, int WAVES_M, int WAVES_N, int STAGES, int OCC, bool A4>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N, OCC) void w4ax_gemm_native_kernel(
    const int8_t *__restrict__ codes, const float *__restrict__ x_scale, const uint8_t *__restrict__ w,
    const float *__restrict__ w_scale, const int8_t *__restrict__ w_zero, const int32_t *__restrict__ code_rowsum,
    const uint16_t *__restrict__ bias, int M, int N, int K, uint16_t *__restrict__ y, int32_t *__restrict__ acc_out,
    int tiles_m, int tiles_n, int group_n, unsigned *__restrict__ sched) {
    constexpr int NW = WAVES_M * WAVES_N;
    constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;  // wave sub-tile
    constexpr int TM = WM / 32, TN = WN / 32;            // MFMA tiles per wave
    // A4: the codes arrive packed two per byte (same nibble order as the weights) and are
    // widened to int8 lanes of 16 * code in registers like the weights.  A lane's 16-byte code
    // fragment then spans 32 channels, so one pipeline step covers 64 channels = 2 MFMAs per tile.
    constexpr int A_ROW = A4 ? BK / 2 : BK;              // bytes of one code row per item
    constexpr int NT = A4 ? 2 : 1;                       // MFMAs along K per step and output tile
    constexpr int KS = BK / (32 * NT);                   // pipeline steps per item
    constexpr int A_STAGE = BM * A_ROW, W_STAGE = BN * BK / 2, STAGE = A_STAGE + W_STAGE;
    constexpr int A_DMA = A_STAGE / 1024 / NW;           // LDS-direct loads per wave per item (1 KB each)
    constexpr int W_DMA = W_STAGE / 1024 / NW;
    constexpr int DMA = A_DMA + W_DMA;
    constexpr int CHUNKS = A_ROW / 16;                   // 16-byte chunks per code row in LDS
    constexpr int ROWS_PER_DMA = 1024 / A_ROW;           // code rows one wave-wide load covers
    constexpr int W_GROUP = kGroup * BK / 2;             // bytes of one 32-row weight group per item
    // With 3 or more buffers the item after the current one is already published, so the
    // first fragments of item q+1 are fetched while the last MFMAs of item q run.
    constexpr int AHEAD = STAGES >= 3 ? 1 : 0;
    // one tile's epilogue vectors in LDS: token scales, channel scales (fp32), bias (bf16), and for
    // weights with zero-points the tokens' code sums (int32) and the channels' zero-points (int8)
    typedef TileVectors<BM, BN> TV;
    constexpr int OFF_BIAS = TV::OFF_BIAS, OFF_RSUM = TV::OFF_RSUM, OFF_ZERO = TV::OFF_ZERO, SCALES = TV::BYTES;
    constexpr int SHIFT = A4 ? 8 : 4;                    // log2 of the factor the widened operands carry
    constexpr int STORES = TM * TN * 2;                  // 16-byte store instructions per wave per full tile
    static_assert((STAGES - 2 - AHEAD) * DMA + STORES < 64, "store-aware wait exceeds vmcnt");
    static_assert(BK == 64 || BK == 128, "K slice per item");
    static_assert(A_ROW == 64 || A_ROW == 128, "code row bytes per item");
    static_assert(A_DMA >= 1 && W_DMA >= 1 && A_DMA * 1024 * NW == A_STAGE && W_DMA * 1024 * NW == W_STAGE,
                  "tile does not split over the waves");
    static_assert(STAGES >= 2 && (STAGES - 1) * DMA < 64, "too many loads in flight for vmcnt");
    static_assert(NW * 4096 <= STAGE && TN % 2 == 0, "the epilogue stages 4 KB per wave in one ring buffer");

    extern __shared__ __align__(16) uint8_t smem[];
    const uint32_t smem_base = lds_address(smem);

    auto swz = [] __device__(int row) { return swz_bk<A_ROW>(row); };
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = (wave % WAVES_M) * WM, wn = (wave / WAVES_M) * WN;
    const int KT = K / BK;
    const int G = ((N + kNPad - 1) / kNPad) * (kNPad / kGroup);  // 32-row groups in the padded weight buffer
    const int64_t w_slice_stride = (int64_t)G * kGroupBytes;
    const int code_row_bytes = A4 ? K / 2 : K;

    // Persistent workgroups take tiles until none is left: drawn per XCD through counters (sched), or in
    // fixed shares (see TileSource).  The two workgroups of a compute unit do not run at the same speed (the
    // older one wins the issue arbitration), so equal shares would leave the faster ones idle for the last
    // tenth of the kernel.
    // The tile numbers a workgroup has drawn go through an 8-entry ring in LDS (s_tiles; -1 = no
    // tile left).  Wave 0 draws tile n + 2 while the loads of tile n are being enqueued and writes the
    // number into the ring one item later, before that item's barrier: the atomic's reply is then
    // older than loads the wave has already awaited, so the draw never stalls anything.
    const TileSource tiles(tiles_m, tiles_n, sched);
    typedef volatile __attribute__((address_space(3))) int lds_int;   // (explicitly LDS: a generic volatile access would be a flat one)
    lds_int *s_tiles = (lds_int *)DVDQ_LDS(smem + STAGES * STAGE + 2 * SCALES);
    int draws = 0;           // tiles drawn so far (the same in every wave)
    unsigned drawn = 0;      // wave 0, lane 0: reply of the draw not yet written into the ring
    bool draw_pending = false;
    auto draw = [&] __device__() {
        if (wave == 0 && tiles.ctr && lane == 0) drawn = tiles.draw();
        ++draws;
        draw_pending = true;
    };
    auto publish_draw = [&] __device__() {   // before a workgroup barrier
        if (wave == 0) {
            if (lane == 0) s_tiles[(draws - 1) & 7] = tiles.tile(drawn, draws - 1);
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
        }
        draw_pending = false;
    };
    // the first two tiles are drawn together
    if (wave == 0 && lane == 0) {
        int t0, t1;
        tiles.first_two(t0, t1);
        s_tiles[0] = t0;
        s_tiles[1] = t1;
    }
    draws = 2;
    __syncthreads();
    int comp_tile = __builtin_amdgcn_readfirstlane(s_tiles[0]);   // tile being multiplied
    if (comp_tile < 0) return;   // (whole workgroup: nothing below is reached, no barrier is missed)

    // ---- LDS-direct load addressing: wave-uniform base pointer + per-lane 32-bit offset.
    // codes: load slot i of this wave fills ROWS_PER_DMA consecutive LDS rows of the stage;
    // LDS position p of a row holds the row's 16-byte chunk p ^ swz(row), where swz spreads
    // the 16 rows that one quarter-wave reads over the 64 banks (see swz_bk).
    int a_row[A_DMA];
    uint32_t a_voff[A_DMA];
#pragma unroll
    for (int i = 0; i < A_DMA; ++i) a_row[i] = (wave * A_DMA + i) * ROWS_PER_DMA + lane / CHUNKS;
    // weights: per item and 32-row group a contiguous run of W_GROUP bytes in the native buffer, so the
    // 1 KB piece p of the stage's weight image starts at byte p * W_PIECE of the item's slice: a
    // wave-uniform term (added to the scalar base) plus 16 bytes per lane
    constexpr int W_PIECE = 1024 / W_GROUP * kGroupBytes + 1024 % W_GROUP;
    static_assert(W_GROUP == kGroupBytes || W_GROUP == 1024, "piece offsets are linear for whole slices or one group per piece");
    const uint32_t lane16 = lane * 16;
    const int8_t *a_base = codes;   // start of the tile's first code row, advanced by BK per item
    const uint8_t *w_base = w;      // start of the tile's weight image for the item
    int issue_tile = 0, issue_kt = 0;   // next item to enqueue: K slice issue_kt of this workgroup's tile issue_tile
    bool issue_live = true;             // false once the ring says there is no further tile
    const int draw_kt = KT > 1 ? 1 : 0; // slice at whose enqueueing the tile after next is drawn
    uint32_t issue_sa = 0;                          // LDS address of the buffer being filled
    // The loads of one item are enqueued one at a time (issue_one) so they can be spread
    // between the MFMAs of the slice being multiplied.  Past the last item the same slice
    // is enqueued again (harmless, keeps the load count per item uniform for vmcnt).
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
            a_base = uniform_ptr(codes + (int64_t)m0 * code_row_bytes);
            w_base = uniform_ptr(w + (int64_t)(n0 / kGroup) * kGroupBytes);
#pragma unroll
            for (int i = 0; i < A_DMA; ++i) {
                const int row = min(a_row[i], M - 1 - m0);   // rows past M re-read the last valid row
                a_voff[i] = (uint32_t)row * code_row_bytes + (((lane % CHUNKS) ^ swz(a_row[i])) << 4);
            }
            // The tile's scales go to LDS as well ([BM token scales][BN channel scales], two tiles
            // deep), so that the epilogue needs no vector-memory load: such a load would queue
            // behind the LDS-direct loads in flight.  Indices past M / N repeat the last valid one.
            // They are issued ahead of the tile's first data loads and are therefore complete
            // whenever that item is published.
            const uint32_t sc = smem_base + STAGES * STAGE + (issue_tile & 1) * SCALES;
#pragma unroll
            for (int j = 0; j < (BM + BN) / 64; ++j) {
                if (j % NW != wave) continue;
                if (j < BM / 64)
                    lds_direct_load4(x_scale, (uint32_t)min(m0 + j * 64 + lane, M - 1) * 4, sc + j * 256);
                else
                    lds_direct_load4(w_scale, (uint32_t)min(n0 + (j - BM / 64) * 64 + lane, N - 1) * 4, sc + j * 256);
            }
            // bias of a tile that lies fully inside N (the only case in which the epilogue reads it from LDS)
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
    // (idx is a constant wherever this is called.  With 128-channel slices the weight pieces of a wave are one
    // run in memory and in LDS: the first sets M0, the others reuse it and move by the instruction offset; the
    // loops below issue a wave's pieces in ascending order, weight pieces last, so nothing comes between them.)
    auto issue_one = [&] __device__(int idx) __attribute__((always_inline)) {
        if (idx < A_DMA) {
            lds_direct_load16(a_base, a_voff[idx], issue_sa + (wave * A_DMA + idx) * 1024);
        } else if (W_PIECE != 1024 || W_DMA > 4 || idx == A_DMA) {
            lds_direct_load16(w_base + (wave * W_DMA + idx - A_DMA) * W_PIECE, lane16,
                              issue_sa + A_STAGE + (wave * W_DMA + idx - A_DMA) * 1024);
        } else {
            const uint8_t *run = w_base + wave * W_DMA * 1024;
            switch (idx - A_DMA) {
                case 1: lds_direct_load16_more<1024>(run, lane16); break;
                case 2: lds_direct_load16_more<2048>(run, lane16); break;
                default: lds_direct_load16_more<3072>(run, lane16); break;
            }
        }
    };
    auto issue_advance = [&] __device__() {
        if (!issue_live) return;
        if (issue_kt + 1 < KT) {
            a_base += A_ROW;
            // items alternate between the halves of a 128-channel slice of the native layout when BK = 64
            w_base += (BK == 128 || (issue_kt & 1)) ? w_slice_stride - (kBK - BK) * (kGroup / 2) : (int64_t)W_GROUP;
            ++issue_kt;
        } else {   // next: slice 0 of the next tile, whose addresses issue_prepare sets (or none: stay on this slice)
            issue_kt = 0;
            ++issue_tile;
        }
    };

    v16i acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    // ---- fragment addressing: MFMA operand row = lane % 32, K half = lane / 32
    const int frow = lane & 31, fhalf = lane >> 5;
    int a_row_off[TM];
#pragma unroll
    for (int j = 0; j < TM; ++j) a_row_off[j] = (wm + j * 32 + frow) * A_ROW;
    const int a_xor = swz(frow);  // == swz(row): wm and 32 j are multiples of 32
    // Weight fragment of MFMA t of step ks: the 16 channels at 32 (NT ks + t) + 16 fhalf of the slice
    // with int8 codes; with packed codes lane half fhalf owns channels 64 ks + 32 fhalf + 16 t
    // (what its 16-byte code fragment holds), i.e. k32 step 2 ks + fhalf, k16 half t of the layout.
    const int w_off = (wn / kGroup) * W_GROUP + frow * 8 + fhalf * (A4 ? 512 : 256);

    // fragments of one step: TM code fragments (16 B) and NT x TN packed weight fragments (8 B)
    struct Frags { v4i a[TM]; uint2 w[NT][TN]; };
    auto load_frags = [&] __device__(Frags &f, int buf, int ks) {
        const uint8_t *sa = smem + buf * STAGE, *sw = sa + A_STAGE;
#pragma unroll
        for (int j = 0; j < TM; ++j) {
            f.a[j] = *reinterpret_cast<const v4i *>(sa + a_row_off[j] + (((ks * 2 + fhalf) ^ a_xor) << 4));
        }
#pragma unroll
        for (int t = 0; t < NT; ++t)
#pragma unroll
            for (int i = 0; i < TN; ++i) {
                f.w[t][i] = *reinterpret_cast<const uint2 *>(sw + w_off + i * W_GROUP +
                                                             (A4 ? ks * 1024 + t * 256 : ks * 512));
            }
    };
    // two packed dwords (16 codes) -> int8 lanes of 16 * code, channel order
    auto widen = [] __device__(uint32_t lo, uint32_t hi) {
        v4i f;
        f[0] = (int)((lo << 4) & 0xF0F0F0F0u);
        f[1] = (int)(lo & 0xF0F0F0F0u);
        f[2] = (int)((hi << 4) & 0xF0F0F0F0u);
        f[3] = (int)(hi & 0xF0F0F0F0u);
        return f;
    };

    // ---- prologue: fill STAGES-1 buffers; with look-ahead also publish slice 0 and fetch its first fragments
#pragma unroll
    for (int s = 0; s < STAGES - 1; ++s) {
        issue_prepare(s);
#pragma unroll
        for (int d = 0; d < DMA; ++d) issue_one(d);
        issue_advance();
    }
    Frags f0, f1;
    if (AHEAD) {
        wait_vmcnt<(STAGES - 2) * DMA>();
        __builtin_amdgcn_s_barrier();
        load_frags(f0, 0, 0);
    }

    int kt = 0, tile_j = 0, store_credit = 0;
    for (int q = 0;; ++q) {
        // Publish slice q + AHEAD: it has landed once at most the loads of the
        // (STAGES - 2 - AHEAD) younger slices are outstanding (a wave's vector memory
        // operations complete in issue order).  The barrier also means that everyone is
        // done reading slice q-1, whose buffer the next loads overwrite.
        {
            // Right after the epilogue of a full tile exactly STORES stores are this wave's youngest
            // operations (for the next STAGES-1-AHEAD items the awaited loads are older than them):
            // do not wait for their acknowledgement.
            if (store_credit > 0) {
                wait_vmcnt<(STAGES - 2 - AHEAD) * DMA + STORES>();
                --store_credit;
            } else {
                wait_vmcnt<(STAGES - 2 - AHEAD) * DMA>();
            }
            if (draw_pending) publish_draw();
            __builtin_amdgcn_s_barrier();
        }
        issue_prepare((q + STAGES - 1) % STAGES);
        // A wave feeding the matrix cores outranks one that converts and stores a finished tile (the
        // two workgroups of a compute unit are in different phases most of the time).
        if (kt == 0) __builtin_amdgcn_s_setprio(2);

        // Software pipeline over the K=32 steps of the item: the fragments of step s+1 (or of
        // step 0 of the next item) are requested before the MFMAs of step s are issued, and the
        // LDS-direct loads of item q+STAGES-1 are dealt out between the MFMA groups.  The
        // scheduling barriers keep the compiler from regrouping any of it.
        const int buf = q % STAGES;
        if (!AHEAD) load_frags(f0, buf, 0);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            Frags &cur = (ks & 1) ? f1 : f0;
            Frags &nxt = (ks & 1) ? f0 : f1;
            if (ks + 1 < KS) load_frags(nxt, buf, ks + 1);
            else if (AHEAD) load_frags(nxt, (q + 1) % STAGES, 0);   // after the last item: stale but in-bounds, unused
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                v4i fa[TM];
#pragma unroll
                for (int j = 0; j < TM; ++j)
                    fa[j] = A4 ? widen((uint32_t)cur.a[j][2 * t], (uint32_t)cur.a[j][2 * t + 1]) : cur.a[j];
#pragma unroll
                for (int i = 0; i < TN; ++i) {
                    const v4i fw = widen(cur.w[t][i].x, cur.w[t][i].y);
#pragma unroll
                    for (int j = 0; j < TM; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fw, fa[j], acc[i][j], 0, 0, 0);
#pragma unroll
                    for (int d = (ks * NT + t) * TN + i; d < DMA; d += KS * NT * TN) issue_one(d);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
        issue_advance();
        if (++kt < KT) continue;
        __builtin_amdgcn_s_setprio(0);   // the epilogue yields issue slots to the other workgroup's K loop

        // ---- epilogue of tile tile_j (shared with the FP6 kernel: see epilogue_interior / epilogue_edge; here the
        // accumulators hold 2^SHIFT times the sum of code products)
        int m0, n0;
        tile_origin(comp_tile, tiles_m, tiles_n, group_n, BM, BN, m0, n0);
        kt = 0;
        ++tile_j;
        comp_tile = __builtin_amdgcn_readfirstlane(s_tiles[tile_j & 7]);   // the next one (its loads are under way)
        const uint8_t *s_tile = smem + STAGES * STAGE + ((tile_j - 1) & 1) * SCALES;
        typedef AccI32<SHIFT> Acc;
        if ((N & 7) == 0 && !acc_out && m0 + BM <= M && n0 + BN <= N) {
            // Interior tile: every lane of every wave stores all its values, so the number of stores is exact
            // (see the store-aware wait above).
            if (KT >= STAGES) store_credit = STAGES - 1 - AHEAD;
            uint8_t *stg = smem + (q % STAGES) * STAGE + wave * 4096;
            __builtin_amdgcn_s_barrier();   // every wave is done reading the last slice: its buffer stages the tile
            // Two specializations, with and without weight zero-points, chosen once per tile (with four, bias as
            // well, this kernel spills).
            if (w_zero) epilogue_interior<Acc, BM, BN, TM, TN, true, -1>(acc, s_tile, bias != nullptr, lane, wm, wn, stg, y, m0, n0, N);
            else epilogue_interior<Acc, BM, BN, TM, TN, false, -1>(acc, s_tile, bias != nullptr, lane, wm, wn, stg, y, m0, n0, N);
        } else {
            epilogue_edge<Acc, BM, BN, TM, TN>(acc, s_tile, bias, w_zero, lane, wm, wn, y, acc_out, m0, n0, M, N);
        }
        if (comp_tile < 0) break;
    }
    wait_vmcnt<0>();   // no LDS-direct load may still be in flight when the workgroup's LDS is released
}

namespace {

// canonical [N, K/2] -> native layout (see the top of this file).  One thread per
// output dword (8 channels).  Rows >= N and channels >= K are written as zero.
__global__ __launch_bounds__(256) void w4_prepack_kernel(const uint8_t *__restrict__ src, uint32_t *__restrict__ dst,
                                                         int N, int K, int G, int KT) {
    const int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t words = (int64_t)KT * G * (kGroupBytes / 4);
    if (o >= words) return;
    int64_t v = o;
    const int d = (int)(v & 1); v >>= 1;
    const int r = (int)(v & 31); v >>= 5;
    const int half = (int)(v & 1); v >>= 1;
    const int ks = (int)(v & 3); v >>= 2;
    const int g = (int)(v % G);
    const int kt = (int)(v / G);
    const int n = g * kGroup + r;
    const int k = kt * kBK + ks * 32 + half * 16 + d * 8;
    uint32_t p = 0;
    if (n < N && k < K) p = *reinterpret_cast<const uint32_t *>(src + (int64_t)n * (K / 2) + k / 2);
    // nibble i of p is channel k+i; wanted: byte b = channel b (low nibble) | channel b+4 (high nibble)
    uint32_t q = 0;
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        q |= ((p >> (4 * b)) & 0xFu) << (8 * b);
        q |= ((p >> (4 * (b + 4))) & 0xFu) << (8 * b + 4);
    }
    dst[o] = q;
}

std::atomic<int> g_variant{-1};   // -1: pick by shape; set by the benchmark's sweep hook
std::atomic<int> g_schedule{-1};  // -1: tiles drawn from counters where possible; 0: fixed shares (benchmark hook)
std::atomic<int> g_grid_limit{0}; // 0: persistent grids fill the chip; else at most this many workgroups (benchmark hook)

// Tile counters of the persistent kernels: one slot of 16 words (the first 8 one per XCD; 64 bytes) per stream;
// kernels of one stream run one after the other.  What a slot holds between launches does not matter (see
// TileSource): it is cleared on the stream right before every kernel that counts in it.
constexpr int kSchedSlots = 512;
__device__ __align__(64) unsigned g_sched[kSchedSlots][16];

struct SchedTable {
    unsigned *base = nullptr;
    std::unordered_map<uint64_t, int> slot_of;   // stream handle -> slot
    std::vector<int> free_slots;                 // released slots, reused before fresh ones
    int fresh = 0;                               // slots never handed out yet
    bool clear[kSchedSlots] = {};                // the last library kernel enqueued on the slot's stream zeroes the slot
};
std::mutex g_sched_mu;
SchedTable g_sched_table[64];

__global__ void fill_sched_kernel(unsigned *p, unsigned value, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = value;
}

}  // namespace

// The counter slot of `stream`, or nullptr (fixed shares): when the stream is being captured into a graph
// -- the same node may later run in several graph instances at once, which must not share counters -- or
// when all slots are taken.  *index: the slot's number.
static unsigned *slot_of_stream(hipStream_t stream, int *dev_out, int *index) {
    if (g_schedule.load(std::memory_order_relaxed) == 0) return nullptr;
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &cap) != hipSuccess) {
        (void)hipGetLastError();
        return nullptr;
    }
    if (cap != hipStreamCaptureStatusNone) return nullptr;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return nullptr;
    SchedTable &t = g_sched_table[dev];
    if (!t.base) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_sched)) != hipSuccess) {
            (void)hipGetLastError();
            return nullptr;
        }
        t.base = static_cast<unsigned *>(p);
    }
    auto it = t.slot_of.find(reinterpret_cast<uint64_t>(stream));
    if (it == t.slot_of.end()) {
        int slot;
        if (!t.free_slots.empty()) {
            slot = t.free_slots.back();
            t.free_slots.pop_back();
        } else if (t.fresh < kSchedSlots) {
            slot = t.fresh++;
        } else {
            return nullptr;
        }
        t.clear[slot] = false;
        it = t.slot_of.emplace(reinterpret_cast<uint64_t>(stream), slot).first;
    }
    *dev_out = dev;
    *index = it->second;
    return t.base + it->second * 16;
}

// For a GEMM about to be enqueued on `stream`: its counter slot (or nullptr: fixed shares), and whether the
// library kernel enqueued last on the stream zeroes it (a quantizer; then the GEMM needs no clearing kernel
// of its own).  The GEMM leaves the slot dirty.  (Calls on one stream are in the caller's order, as the
// stream's own semantics require.)
unsigned *sched_slot(hipStream_t stream, bool *is_clear) {
    std::lock_guard<std::mutex> lock(g_sched_mu);
    int dev = 0, index = 0;
    *is_clear = false;
    unsigned *slot = slot_of_stream(stream, &dev, &index);
    if (slot) {
        *is_clear = g_sched_table[dev].clear[index];
        g_sched_table[dev].clear[index] = false;
    }
    return slot;
}

// For a quantizer about to be enqueued on `stream`: the 16 words it should zero (or nullptr), and, once it
// is enqueued, the note that it does.
unsigned *sched_slot_to_clear(hipStream_t stream) {
    std::lock_guard<std::mutex> lock(g_sched_mu);
    int dev = 0, index = 0;
    return slot_of_stream(stream, &dev, &index);
}
void sched_slot_cleared(hipStream_t stream) {
    std::lock_guard<std::mutex> lock(g_sched_mu);
    int dev = 0, index = 0;
    if (slot_of_stream(stream, &dev, &index)) g_sched_table[dev].clear[index] = true;
}

int clear_sched_slot(unsigned *slot, hipStream_t stream) {
    hipLaunchKernelGGL(fill_sched_kernel, dim3(1), dim3(64), 0, stream, slot, 0u, 16);
    return check_launch();
}

int fill_sched_slots(uint32_t value, hipStream_t stream) {
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_sched)) != hipSuccess) return DVDQ_ERR_HIP;
    const int n = kSchedSlots * 16;
    hipLaunchKernelGGL(fill_sched_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, static_cast<unsigned *>(p), value, n);
    {
        std::lock_guard<std::mutex> lock(g_sched_mu);
        for (auto &t : g_sched_table)
            for (bool &c : t.clear) c = false;
    }
    return check_launch();
}

// Forget `stream` on the current device (its slot goes to the next stream that needs one).
void release_sched_slot(hipStream_t stream) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return;
    std::lock_guard<std::mutex> lock(g_sched_mu);
    SchedTable &t = g_sched_table[dev];
    auto it = t.slot_of.find(reinterpret_cast<uint64_t>(stream));
    if (it == t.slot_of.end()) return;
    t.free_slots.push_back(it->second);
    t.slot_of.erase(it);
}

namespace {

template <int BM, int BN, int BK, int WAVES_M, int WAVES_N, int STAGES, int OCC, bool A4 = false>
int launch_native(const int8_t *codes, const float *x_scale, const uint8_t *w, const float *w_scale,
                  const int8_t *w_zero, const int32_t *code_rowsum, const uint16_t *bias, int M, int N, int K,
                  uint16_t *y, int32_t *acc_out, hipStream_t stream) {
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    // column tiles per L2 sharing group: balanced groups of at most 16
    const int n_groups = (tiles_n + 15) / 16;
    const int group_n = (tiles_n + n_groups - 1) / n_groups;
    const int total = tiles_m * tiles_n;
    // persistent: OCC workgroups per compute unit (256 CUs), grid a multiple of the 8 XCDs
    int grid = 256 * OCC;
    if (total < grid) grid = (total + 7) / 8 * 8;
    grid = limited_grid(grid);
    // the ring, then two tiles' epilogue vectors (scales, bias, code sums, zero-points; see the kernel)
    const size_t smem = (size_t)STAGES * (BM * (A4 ? BK / 2 : BK) + BN * BK / 2) +
                        2 * ((BM + BN) * 4 + BN * 2 + BM * 4 + BN) + 8 * sizeof(int);   // + the ring of tile numbers
    auto k = w4ax_gemm_native_kernel<BM, BN, BK, WAVES_M, WAVES_N, STAGES, OCC, A4>;
    static std::atomic<uint64_t> configured{0};   // one per template instantiation
    allow_dynamic_lds(reinterpret_cast<const void *>(k), smem, configured);
    bool is_clear = false;
    unsigned *sched = sched_slot(stream, &is_clear);
    if (sched && !is_clear && clear_sched_slot(sched, stream) != DVDQ_OK) return DVDQ_ERR_HIP;
    hipLaunchKernelGGL(k, dim3((unsigned)grid), dim3(64 * WAVES_M * WAVES_N), smem, stream, codes, x_scale, w,
                       w_scale, w_zero, code_rowsum, bias, M, N, K, y, acc_out, tiles_m, tiles_n, group_n, sched);
    return check_launch();
}

}  // namespace

void set_gemm_variant(int v) { g_variant.store(v, std::memory_order_relaxed); }
int gemm_variant() { return g_variant.load(std::memory_order_relaxed); }
void set_gemm_schedule(int v) { g_schedule.store(v, std::memory_order_relaxed); }
void set_gemm_grid_limit(int v) { g_grid_limit.store(v, std::memory_order_relaxed); }
int limited_grid(int grid) {
    const int limit = g_grid_limit.load(std::memory_order_relaxed);
    if (limit <= 0 || grid <= limit) return grid;
    return limit < 8 ? 8 : limit / 8 * 8;
}

int launch_w4ax_gemm(const int8_t *codes, const float *x_scale, const uint8_t *w, const float *w_scale,
                     const int8_t *w_zero, const int32_t *code_rowsum, const uint16_t *bias, int64_t M, int64_t N,
                     int64_t K, int codes_format, int w_layout, uint16_t *y, int32_t *acc_out, hipStream_t stream) {
    if (w_layout == DVDQ_W_CANONICAL) {
        if (codes_format != DVDQ_CODES_INT8 || w_zero) return DVDQ_ERR_UNSUPPORTED;
        return launch_w4ax_gemm_canonical(codes, x_scale, w, w_scale, bias, M, N, K, y, acc_out, stream);
    }
    const int m = (int)M, n = (int)N, k = (int)K;
#define DVDQ_GEMM_ARGS codes, x_scale, w, w_scale, w_zero, code_rowsum, bias, m, n, k, y, acc_out, stream
    // Tile variants: {tile M, tile N, K slice, waves M x N, ring depth, workgroups per compute unit}.
    // Variant 2 is the default of the two-wave kernels for every shape: two independent 4-wave workgroups per compute unit,
    // each owning a 128 x 256 tile (64 x 128 per wave) with K slices of 128 through two buffers.  In
    // interleaved sweeps over the DiT shapes (K = 1536 ... 13824) it was fastest or within 1 % of the
    // fastest: while one workgroup converts and stores its tile the other keeps the matrix cores busy,
    // which the one-workgroup 256 x 256 variants cannot do.  The others remain for sweeps; a shape with
    // fewer K slices than a variant's ring needs falls back to variant 2, which always qualifies.
    const int forced = gemm_variant();
    int v = forced < 0 ? 2 : forced;
    if (codes_format == DVDQ_CODES_PACKED4) {
        if ((v == 1 && k / 128 < 2) || (v > 2 && k / 128 < 3)) v = 2;
        switch (v) {
            case 1: return launch_native<256, 256, 128, 2, 4, 3, 1, true>(DVDQ_GEMM_ARGS);
            case 2: return launch_native<128, 256, 128, 2, 2, 2, 2, true>(DVDQ_GEMM_ARGS);
            case 3: return launch_native<256, 256, 128, 2, 4, 4, 1, true>(DVDQ_GEMM_ARGS);
            case 4: return launch_native<256, 256, 128, 4, 2, 4, 1, true>(DVDQ_GEMM_ARGS);
            default: return DVDQ_ERR_UNSUPPORTED;
        }
    }
    // Variant 5 is the wide kernel of w4ax_gemm_wide.hip (int8 codes only).  Measured on the DiT shapes it is 2 %
    // (K = 1536) to 6 % (K = 3072) faster than variant 2 and level with it at K = 13824; it is taken by itself when
    // a tile has at least 12 K slices and there are at least two rounds of 256 x 256 tiles (fewer tiles are dealt
    // out more evenly in variant 2's 128 x 256 pieces).
    if (forced < 0 && codes_format == DVDQ_CODES_INT8 && k / 128 >= 12 && ((M + 255) / 256) * ((N + 255) / 256) >= 512) v = 5;
    if (v == 5)
        return launch_w4ax_gemm_wide(reinterpret_cast<const uint8_t *>(codes), x_scale, w, w_scale, w_zero, code_rowsum, bias,
                                     M, N, K, false, y, acc_out, stream);
    {
        const int bk = v == 4 ? 64 : 128, stages = v == 2 ? 2 : (v == 4 ? 4 : 3);
        if (k / bk < stages - 1) v = 2;
    }
    switch (v) {
        case 1: return launch_native<256, 256, 128, 4, 2, 3, 1>(DVDQ_GEMM_ARGS);
        case 2: return launch_native<128, 256, 128, 2, 2, 2, 2>(DVDQ_GEMM_ARGS);
        case 3: return launch_native<256, 256, 128, 2, 4, 3, 1>(DVDQ_GEMM_ARGS);
        case 4: return launch_native<128, 256, 64, 2, 2, 4, 2>(DVDQ_GEMM_ARGS);
        default: return DVDQ_ERR_UNSUPPORTED;
    }
#undef DVDQ_GEMM_ARGS
}

size_t w4_native_bytes(int64_t N, int64_t K) {
    const int64_t npad = (N + kNPad - 1) / kNPad * kNPad, kpad = (K + kBK - 1) / kBK * kBK;
    return (size_t)(npad * kpad / 2);
}

int launch_w4_prepack(const uint8_t *w_canonical, int64_t N, int64_t K, uint8_t *w_native, hipStream_t stream) {
    const int G = (int)((N + kNPad - 1) / kNPad * (kNPad / kGroup));
    const int KT = (int)((K + kBK - 1) / kBK);
    const int64_t words = (int64_t)KT * G * (kGroupBytes / 4);
    const int64_t blocks = (words + 255) / 256;
    hipLaunchKernelGGL(w4_prepack_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, w_canonical,
                       reinterpret_cast<uint32_t *>(w_native), (int)N, (int)K, G, KT);
    return check_launch();
}

}  // namespace dvdq

// Device helpers shared by the persistent GEMM kernels (INT8 matrix path in w4ax_gemm.hip, FP6 matrix
// path in w4a4_fp6_gemm.hip, both operand types with one wave per SIMD in w4ax_gemm_wide.hip): LDS-direct
// loads, hand-kept vmcnt waits, streaming stores, tile order, tile draws.
#pragma once
#include "dvdq_internal.h"

namespace dvdq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v16f __attribute__((ext_vector_type(16)));

constexpr int kBK = 128;      // K slice (bytes of int8 codes per row)
constexpr int kGroup = 32;    // weight rows per native-layout group
constexpr int kGroupBytes = kGroup * kBK / 2;  // 2048: one group, one K slice, packed
constexpr int kNPad = 256;    // native layout pads N to a multiple of this

#define DVDQ_LDS(p) ((__attribute__((address_space(3))) void *)(p))

static __device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
    typedef __bf16 v2bf __attribute__((ext_vector_type(2)));
    v2bf p = {(__bf16)a, (__bf16)b};  // round-to-nearest-even conversions
    return __builtin_bit_cast(uint32_t, p);
}

// 16-byte store of output the kernel never reads again.  Non-temporal: with whole 128-byte lines
// per instruction (the staged epilogue) the output stream then bypasses the L2 instead of evicting
// code and weight panels and leaving dirty lines to flush at the kernel's end.  (For partial-line
// stores the same hint is much slower than write-back caching.)
static __device__ __forceinline__ void store_streaming16(uint16_t *p, uint4 v) {
    typedef uint32_t v4u __attribute__((ext_vector_type(4)));
    const v4u vv = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(vv, reinterpret_cast<v4u *>(p));
}

// vmcnt-only wait (leave expcnt / lgkmcnt alone): gfx9 encoding, vmcnt = {imm[15:14], imm[3:0]}
template <int N>
static __device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt is 6 bits");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

// One LDS-direct load: 16 bytes per lane from global address `sbase` + `voff` (sbase
// wave-uniform, voff per lane) to LDS address `lds_base` + 16 * lane (lds_base
// wave-uniform).  Written as inline assembly so that the compiler's waitcnt insertion
// does not know about it: with the builtin it makes every later LDS read wait for ALL
// outstanding LDS-direct loads (it cannot tell the ring buffers apart), which
// serializes the pipeline.  Completion is awaited by hand (wait_vmcnt) before the
// workgroup barrier that publishes a buffer.
// (The wait states cover two hazards the compiler cannot see inside the statement: M0 written by the s_mov
// needs one before an LDS-direct load, and a scalar register written by a vector instruction -- a base address
// the compiler has just reloaded with v_readlane or made uniform with v_readfirstlane -- needs five before a
// vector memory instruction reads it: the load would otherwise go to whatever address the register pair held
// before.)
static __device__ __forceinline__ void lds_direct_load16(const void *sbase, uint32_t voff, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 3\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(voff), "s"(sbase), "s"(lds_base)
                 : "memory");
}

// Follow-up of lds_direct_load16 with the same M0: the instruction offset OFF is added to the global address
// and to the LDS address alike (checked on the hardware), so a run of loads whose source and destination
// advance by the same number of bytes needs one M0 and one base address.  No other M0 write may stand
// between it and the load that set M0, and the base address must not have been written by a vector instruction
// within the last five wait states (it is the register pair the run's first load used; tests/test_kernel_asm.py
// checks both on the kernels' assembly).
template <int OFF>
static __device__ __forceinline__ void lds_direct_load16_more(const void *sbase, uint32_t voff) {
    static_assert(OFF > 0 && OFF < 4096, "13-bit signed instruction offset");
    asm volatile("global_load_lds_dwordx4 %0, %1 offset:%2" : : "v"(voff), "s"(sbase), "n"(OFF) : "memory");
}

// chunk swizzle of a code row in LDS (see the kernel).  A 16-byte read is served 16 lanes = 16 rows at a
// time by the 64 banks (256 bytes), and rows 128 bytes apart alternate between the two halves of the
// banks: the 8 rows of a half take 8 different chunk slots with (row >> 1) & 7.  With 64-byte rows four
// rows share a quarter of the banks and take its 4 slots with (row >> 2) & 3.
template <int BK>
static __device__ __forceinline__ int swz_bk(int row) { return BK == 128 ? ((row >> 1) & 7) : ((row >> 2) & 3); }

// Same, 4 bytes per lane (LDS address lds_base + 4 * lane): used for the per-tile scale vectors.
static __device__ __forceinline__ void lds_direct_load4(const void *sbase, uint32_t voff, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 3\n\tglobal_load_lds_dword %0, %1"
                 :
                 : "v"(voff), "s"(sbase), "s"(lds_base)
                 : "memory");
}

static __device__ __forceinline__ uint32_t lds_address(const void *p) {
    return (uint32_t)(uintptr_t)DVDQ_LDS(p);
}

// make a 64-bit pointer provably wave-uniform (lives in SGPRs)
template <typename T>
static __device__ __forceinline__ const T *uniform_ptr(const T *p) {
    const uint64_t v = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
    return reinterpret_cast<const T *>(((uint64_t)hi << 32) | lo);
}

// Tile order.  Tiles are numbered so that `group_n` output-column tiles run fastest,
// then token tiles, then column groups: tiles with neighbouring numbers share code
// panels and a bounded set of weight panels, which is what stays in an XCD's L2.
static __device__ __forceinline__ void tile_origin(int t, int tiles_m, int tiles_n, int group_n, int BM, int BN, int &m0,
                                            int &n0) {
    const int per_group = tiles_m * group_n;
    const int grp = t / per_group;
    const int in_grp = t - grp * per_group;
    const int gw = min(group_n, tiles_n - grp * group_n);  // columns in this (possibly last, narrower) group
    const int tile_m = in_grp / gw;
    m0 = tile_m * BM;
    n0 = (grp * group_n + (in_grp - tile_m * gw)) * BN;
}


// ---- tile numbers of a persistent launch
// Workgroup ids are dealt round-robin to the 8 XCDs, and the workgroups of one XCD work on one contiguous
// run of tile numbers at a time.
//   ctr != nullptr: XCD x owns tile numbers [x total / 8, (x + 1) total / 8) and its workgroups draw from them
//     in order through one counter word (an atomic add).  The word is zero when the kernel starts: whatever
//     runs on the stream right before the GEMM clears the slot (the quantizer kernel, if that is what the
//     library enqueued last on the stream, else a one-wave kernel the GEMM's launcher puts in front), so no
//     launch depends on what an earlier one -- finished or not -- left behind, and nothing has to be put back
//     at the end.
//   ctr == nullptr: fixed shares, the j-th tile of workgroup b is number j * grid + (b % 8) * (grid / 8) + b / 8.
struct TileSource {
    int total, grid, xcd, first_tile, run_lo;
    unsigned run_len;
    unsigned *ctr;   // this XCD's counter

    __device__ __forceinline__ TileSource(int tiles_m, int tiles_n, unsigned *sched) {
        total = tiles_m * tiles_n;
        grid = gridDim.x;   // a multiple of 8
        xcd = blockIdx.x % 8;
        first_tile = xcd * (grid / 8) + blockIdx.x / 8;
        run_lo = (int)((int64_t)xcd * total / 8);
        run_len = (unsigned)((int64_t)(xcd + 1) * total / 8) - (unsigned)run_lo;
        ctr = sched ? sched + xcd : nullptr;
    }
    // the tile a draw's reply stands for (drawn mode), or the workgroup's ordinal-th tile (fixed shares); -1: none left
    __device__ __forceinline__ int tile(unsigned reply, int ordinal) const {
        if (ctr) return reply < run_len ? run_lo + (int)reply : -1;
        const int t = first_tile + ordinal * grid;
        return t < total ? t : -1;
    }
    // one further tile (one lane; drawn mode only).  The reply may be awaited as late as the caller likes.
    __device__ __forceinline__ unsigned draw() const { return atomicAdd(ctr, 1u); }
    // the workgroup's first two tiles (one lane; either mode)
    __device__ __forceinline__ void first_two(int &t0, int &t1) const {
        const unsigned v = ctr ? atomicAdd(ctr, 2u) : 0u;
        t0 = tile(v, 0);
        t1 = tile(v + 1u, 1);
    }
};

// ---- epilogues of the two-waves-per-SIMD kernels (INT8 matrix path and FP6 matrix path)
// Both kernels end a tile the same way; what differs is how an accumulator register turns into the integer sum
// of code products, which an accumulator policy states:
//   AccI32<SHIFT>: int32 registers holding 2^SHIFT times the sum (the widened operands' factor);
//   AccF32x64:     fp32 registers holding the sum / 64 exactly (FP6 values are codes / 8).
// Accumulator register r = 4 g + e of MFMA tile (i, j) in lane l is
//   n = n0 + wn + 32 i + 8 g + 4 (l / 32) + e,   m = m0 + wm + 32 j + (l % 32).
// With weight zero-points, sum q (c - z) = acc - z * rs (rs the token's code sum) is taken with a 24-bit
// multiply: operands and product are in range (checked by the C ABI), so it is exact.
template <int SHIFT>
struct AccI32 {
    typedef v16i vec;
    // factor folded into the token scale (a power of two: exact)
    static __device__ __forceinline__ constexpr float fold(bool) { return 1.f / (float)(1 << SHIFT); }
    template <bool ZP>
    static __device__ __forceinline__ float scaled(int a, int z, int rs, float xs_folded) {
        if constexpr (ZP) a -= __mul24(z * (1 << SHIFT), rs);
        return (float)a * xs_folded;
    }
    // per-element path: the register's integer (still times 2^SHIFT), its zero-point term, the plain sum
    static __device__ __forceinline__ int integer(int a) { return a; }
    static __device__ __forceinline__ int unzero(int v, int z, int rs) { return v - __mul24(z * (1 << SHIFT), rs); }
    static __device__ __forceinline__ int sum(int v) { return v >> SHIFT; }
    static __device__ __forceinline__ constexpr float edge_fold() { return 1.f / (float)(1 << SHIFT); }
};

struct AccF32x64 {
    typedef v16f vec;
    // without zero-points the token scale times 64 multiplies the fp32 accumulator directly
    static __device__ __forceinline__ constexpr float fold(bool zp) { return zp ? 1.f : 64.f; }
    template <bool ZP>
    static __device__ __forceinline__ float scaled(float a, int z, int rs, float xs_folded) {
        if constexpr (ZP) return (float)((int)(a * 64.f) - __mul24(z, rs)) * xs_folded;
        else return a * xs_folded;
    }
    static __device__ __forceinline__ int integer(float a) { return (int)(a * 64.f); }
    static __device__ __forceinline__ int unzero(int v, int z, int rs) { return v - __mul24(z, rs); }
    static __device__ __forceinline__ int sum(int v) { return v; }
    static __device__ __forceinline__ constexpr float edge_fold() { return 1.f; }
};

// LDS image of a tile's epilogue vectors (staged by LDS-direct loads with the tile's first slice): token scales
// fp32 [BM], channel scales fp32 [BN], bias bf16 [BN], code sums int32 [BM], zero-points int8 [BN]
template <int BM, int BN>
struct TileVectors {
    static constexpr int OFF_BIAS = (BM + BN) * 4, OFF_RSUM = OFF_BIAS + BN * 2, OFF_ZERO = OFF_RSUM + BM * 4;
    static constexpr int BYTES = OFF_ZERO + BN;
};

// Interior tile (whole tile inside M x N, N a multiple of 8; specialized on zero-points and, where the caller
// can afford the code, on bias: a run-time test inside the unrolled loops costs a branch per register group): no predicates, every vector the epilogue needs
// comes from LDS, one row pointer per lane.  The bf16 tile goes through LDS so that every store instruction
// writes whole 128-byte lines: in the accumulator layout a lane owns one token and 8 consecutive channels per
// register group, so a direct store touches 32 token rows with 32 bytes each.  32 tokens x 64 channels at a
// time are staged in `stg` (this wave's 4 KB of the ring buffer whose slice was consumed last: after the
// barrier no wave reads it any more, and the next loads into it are only issued after the next K loop's first
// barrier; 16-byte pieces, piece index xor-ed with the row against bank conflicts) and read back with 8 lanes
// per token row.  A lane's channel vectors (4 channel scales, bias, zero-points) for register group g of MFMA
// tile column i are fetched one group ahead of their use: a read issued where its value is needed would
// expose the LDS latency once per group, 32 times per tile.  The accumulators are left at zero.
// BIAS: 1 / 0 = with / without bias, fixed at compile time; -1 = `has_bias` decides at run time (for kernels
// whose register budget does not survive four inlined copies of this function).
template <class P, int BM, int BN, int TM, int TN, bool ZP, int BIAS>
static __device__ __forceinline__ void epilogue_interior(typename P::vec (&acc)[TN][TM], const uint8_t *s_tile, bool has_bias,
                                                         int lane, int wm, int wn, uint8_t *stg, uint16_t *y, int m0,
                                                         int n0, int N) {
    // (scale, then add the bias, each rounded: a fused multiply-add would differ from the per-element path in the last bit)
#pragma clang fp contract(off)
    if constexpr (BIAS >= 0) has_bias = BIAS != 0;
    typedef TileVectors<BM, BN> TV;
    const int frow = lane & 31, fhalf = lane >> 5;
    const float *s_xs = reinterpret_cast<const float *>(s_tile);
    const float *ws_l = s_xs + BM + wn + fhalf * 4;
    const int32_t *s_rsum = reinterpret_cast<const int32_t *>(s_tile + TV::OFF_RSUM);
    const uint32_t *bias_l = reinterpret_cast<const uint32_t *>(s_tile + TV::OFF_BIAS) + (wn + fhalf * 4) / 2;
    const uint32_t *zero_l = reinterpret_cast<const uint32_t *>(s_tile + TV::OFF_ZERO) + (wn + fhalf * 4) / 4;
    float xs_l[TM];
    int rsum[TM];
#pragma unroll
    for (int j = 0; j < TM; ++j) {
        xs_l[j] = s_xs[wm + j * 32 + frow] * P::fold(ZP);
        rsum[j] = ZP ? s_rsum[wm + j * 32 + frow] : 0;
    }
    const int rd_row = lane >> 3, rd_piece = lane & 7;
    struct ChannelVec { float4 ws; uint2 bb; uint32_t zq; };
    auto fetch = [&] __device__(ChannelVec &cv, int i, int g) {
        const int c = i * 32 + g * 8;
        cv.ws = *reinterpret_cast<const float4 *>(ws_l + c);
        if (has_bias) cv.bb = *reinterpret_cast<const uint2 *>(bias_l + c / 2);
        if constexpr (ZP) cv.zq = zero_l[c / 4];
    };
    ChannelVec cv[2];   // group k of the tile's groups lives in cv[k & 1]
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
                            o[e] = P::template scaled<ZP>(acc[i][j][r + e], (int)(int8_t)(c.zq >> (8 * e)), rsum[j], xs_l[j]);
                            acc[i][j][r + e] = 0;
                        }
                        o[0] *= c.ws.x;
                        o[1] *= c.ws.y;
                        o[2] *= c.ws.z;
                        o[3] *= c.ws.w;
                        if (has_bias) {
                            o[0] += __uint_as_float(c.bb.x << 16);
                            o[1] += __uint_as_float(c.bb.x & 0xFFFF0000u);
                            o[2] += __uint_as_float(c.bb.y << 16);
                            o[3] += __uint_as_float(c.bb.y & 0xFFFF0000u);
                        }
                        pk[h][0] = pack_bf16x2(o[0], o[1]);
                        pk[h][1] = pack_bf16x2(o[2], o[3]);
                    }
                    // lanes l and l+32 hold channels (8g .. 8g+3) and (8g+4 .. 8g+7): swap the upper half
                    // of group g with the lower half of group g+1 so each lane owns 8 consecutive channels
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
}

// Edge tiles, N not a multiple of 8, or the accumulator hook: predicated per element, through the integer
// accumulator (same values and rounding order as the interior path).  The accumulators are left at zero.
template <class P, int BM, int BN, int TM, int TN>
static __device__ __forceinline__ void epilogue_edge(typename P::vec (&acc)[TN][TM], const uint8_t *s_tile, const uint16_t *bias,
                                                     const int8_t *w_zero, int lane, int wm, int wn, uint16_t *y,
                                                     int32_t *acc_out, int m0, int n0, int M, int N) {
    typedef TileVectors<BM, BN> TV;
    const int frow = lane & 31, fhalf = lane >> 5;
    const float *s_xs = reinterpret_cast<const float *>(s_tile);
    const float *s_ws = s_xs + BM;
    const int32_t *s_rsum = reinterpret_cast<const int32_t *>(s_tile + TV::OFF_RSUM);
    const bool vec8 = (N & 7) == 0;
#pragma unroll
    for (int j = 0; j < TM; ++j) {
        const int m = m0 + wm + j * 32 + frow;
        const bool m_ok = m < M;
        const float xs = s_xs[wm + j * 32 + frow] * P::edge_fold();
        const int rs = w_zero ? s_rsum[wm + j * 32 + frow] : 0;
#pragma unroll
        for (int i = 0; i < TN; ++i) {
            const int nb = n0 + wn + i * 32;   // this MFMA tile's first output channel
            int a[16];
#pragma unroll
            for (int g = 0; g < 4; ++g)
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    // (channels past N: some valid zero-point, for values that are never stored)
                    const int z = w_zero ? (int)w_zero[min(nb + g * 8 + fhalf * 4 + e, N - 1)] : 0;
                    a[g * 4 + e] = P::unzero(P::integer(acc[i][j][g * 4 + e]), z, rs);
                    acc[i][j][g * 4 + e] = 0;
                }
            if (acc_out && m_ok) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const int n = nb + g * 8 + fhalf * 4;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (n + e < N) acc_out[(int64_t)m * N + n + e] = P::sum(a[g * 4 + e]);
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
                // lanes l and l+32 hold channels (8g .. 8g+3) and (8g+4 .. 8g+7): swap the upper half of
                // group g with the lower half of group g+1 so each lane owns 8 consecutive channels
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

// Enqueues the one-wave kernel that zeroes a counter slot (sched_slot; defined in w4ax_gemm.hip).
int clear_sched_slot(unsigned *slot, hipStream_t stream);
int gemm_variant();   // the benchmark hook's tile variant (-1: the kernels' own choice)

}  // namespace dvdq

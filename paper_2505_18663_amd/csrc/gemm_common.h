// Device helpers shared by the persistent GEMM kernels (INT8 matrix path in w4ax_gemm.hip, FP6 matrix
// path in w4a4_fp6_gemm.hip, both operand types with one wave per SIMD in w4ax_gemm_wide.hip): LDS-direct
// loads, hand-kept vmcnt waits, streaming stores, tile order, tile draws.
#pragma once
#include "dvdq_internal.h"

namespace dvdq {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

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
static __device__ __forceinline__ void lds_direct_load16(const void *sbase, uint32_t voff, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(voff), "s"(sbase), "s"(lds_base)
                 : "memory");
}

// chunk swizzle of a code row in LDS (see the kernel).  A 16-byte read is served 16 lanes = 16 rows at a
// time by the 64 banks (256 bytes), and rows 128 bytes apart alternate between the two halves of the
// banks: the 8 rows of a half take 8 different chunk slots with (row >> 1) & 7.  With 64-byte rows four
// rows share a quarter of the banks and take its 4 slots with (row >> 2) & 3.
template <int BK>
static __device__ __forceinline__ int swz_bk(int row) { return BK == 128 ? ((row >> 1) & 7) : ((row >> 2) & 3); }

// Same, 4 bytes per lane (LDS address lds_base + 4 * lane): used for the per-tile scale vectors.
static __device__ __forceinline__ void lds_direct_load4(const void *sbase, uint32_t voff, uint32_t lds_base) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1"
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

// Enqueues the one-wave kernel that zeroes a counter slot (sched_slot; defined in w4ax_gemm.hip).
int clear_sched_slot(unsigned *slot, hipStream_t stream);
int gemm_variant();   // the benchmark hook's tile variant (-1: the kernels' own choice)

}  // namespace dvdq

// Internal declarations shared by the translation units of libdvdq (not installed).
#pragma once
#include <hip/hip_runtime.h>
#include <atomic>
#include <stddef.h>
#include <stdint.h>

#include "../../include/dvdq.h"

namespace dvdq {

// Launchers: arguments are already validated by the C-ABI layer in api.hip.
// Each returns DVDQ_OK or DVDQ_ERR_HIP.
int launch_rotate_quant(const uint16_t *x, int64_t M, int64_t K, int log2_block, int act_bits, int codes_format,
                        int group_log2, int8_t *codes, float *x_scale, int32_t *code_rowsum, hipStream_t stream);


int launch_w4ax_gemm(const int8_t *codes, const float *x_scale, const uint8_t *w, const float *w_scale,
                     const int8_t *w_zero, const int32_t *code_rowsum, const uint16_t *bias, int64_t M, int64_t N,
                     int64_t K, int codes_format, int w_layout, uint16_t *y, int32_t *acc_out, hipStream_t stream);

int launch_w4ax_gemm_canonical(const int8_t *codes, const float *x_scale, const uint8_t *w, const float *w_scale,
                               const uint16_t *bias, int64_t M, int64_t N, int64_t K, uint16_t *y, int32_t *acc_out,
                               hipStream_t stream);

// W4A4 on the FP6 matrix path (w4a4_fp6_gemm.hip): codes and weights in the FP6 block-slice layouts
int launch_w4a4_fp6_gemm(const uint8_t *codes, const float *x_scale, const uint8_t *w, const float *w_scale,
                         const int8_t *w_zero, const int32_t *code_rowsum, const uint16_t *bias, int64_t M, int64_t N,
                         int64_t K, uint16_t *y, int32_t *acc_out, hipStream_t stream);
// One 4-wave workgroup per compute unit, 128 x 128 wave tiles, accumulators in AGPRs (w4ax_gemm_wide.hip):
// int8 codes x native weights (fp6 = false) or FP6 codes x FP6 native weights (fp6 = true)
int launch_w4ax_gemm_wide(const uint8_t *codes, const float *x_scale, const uint8_t *w, const float *w_scale,
                          const int8_t *w_zero, const int32_t *code_rowsum, const uint16_t *bias, int64_t M, int64_t N,
                          int64_t K, bool fp6, uint16_t *y, int32_t *acc_out, hipStream_t stream);
size_t w4_native_fp6_bytes(int64_t N, int64_t K);
size_t codes_fp6_bytes(int64_t M, int64_t K);
int launch_w4_prepack_fp6(const uint8_t *w_canonical, int64_t N, int64_t K, uint8_t *w_native, hipStream_t stream);

size_t w4_native_bytes(int64_t N, int64_t K);
void set_gemm_variant(int v);  // benchmark sweeps only; -1 = choose by shape
void set_gemm_schedule(int v); // benchmark only; 0 = fixed tile shares, -1 = drawn from counters where possible
void set_gemm_grid_limit(int v); // benchmark only; 0 = persistent grids fill the chip, else at most v workgroups
int limited_grid(int grid);
// the stream's tile-counter slot (16 words; nullptr: fixed tile shares): for a GEMM, with whether the kernel enqueued last
// on the stream zeroes it; for a quantizer, the words to zero and the note that it does (w4ax_gemm.hip)
unsigned *sched_slot(hipStream_t stream, bool *is_clear);
unsigned *sched_slot_to_clear(hipStream_t stream);
void sched_slot_cleared(hipStream_t stream);
void release_sched_slot(hipStream_t stream);               // forget a stream's tile-counter slot (host bookkeeping only)
int fill_sched_slots(uint32_t value, hipStream_t stream);  // robustness tests only: overwrite every tile counter

int launch_w4_prepack(const uint8_t *w_canonical, int64_t N, int64_t K, uint8_t *w_native, hipStream_t stream);

size_t gbs_workspace_bytes();
int launch_gbs_reset(void *state, int bits, hipStream_t stream);
int launch_gbs_step(const uint16_t *ft, const uint16_t *fp, int64_t n, double delta, int b_low, int b_high,
                    void *state, void *workspace, hipStream_t stream);

int launch_bgr(const float *w, int64_t N, int64_t K, int n_steps, int max_refine, double eps, int search,
               uint8_t *w_packed, float *w_scale, int8_t *w_zero, double *row_error, hipStream_t stream);

// Raise a kernel's dynamic-LDS limit to `bytes` once per kernel and device (`done` is the call
// site's own bit mask of devices already configured).  Not a stream operation: after the first
// launch on a device nothing but the launch itself is issued, also under stream capture.
inline void allow_dynamic_lds(const void *kernel, size_t bytes, std::atomic<uint64_t> &done) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return;
    const uint64_t bit = dev >= 0 && dev < 64 ? (uint64_t)1 << dev : 0;
    if (bit && (done.load(std::memory_order_acquire) & bit)) return;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes) == hipSuccess && bit)
        done.fetch_or(bit, std::memory_order_release);
}

inline int check_launch() { return hipGetLastError() == hipSuccess ? DVDQ_OK : DVDQ_ERR_HIP; }

}  // namespace dvdq

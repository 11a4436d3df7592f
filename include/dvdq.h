/*
 * dvdq -- the quantized linear layer of a video DiT on MI355X (gfx950).
 *
 * C ABI of the hot path of DVD-Quant's quantized inference: one linear layer
 *
 *     X~ = X H            online block Walsh-Hadamard rotation      (Sec. 3.2, ARQ)
 *     s  = max|X~| / qmax  online auto-scale, one per token row      (Sec. 3.2, ARQ equation)
 *     X^ = Q(X~ / s)      symmetric low-bit codes                   (Sec. 3.2, ARQ equation)
 *     Y  = s * (X^ W^^T) * Delta    low-bit GEMM and rescale        (Sec. 3.2 ARQ equation, Sec. 3.1 DeQuant)
 *
 * with W^ the offline-quantized INT4 weights (codes + one step size Delta per
 * output channel), already expressed in the rotated basis (W H, Sec. 3.2).
 * The activation bit-width is an argument: delta-Guided Bit Switching (Sec. 3.3)
 * picks it per denoising step outside this library.
 *
 * Conventions shared by every entry point
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library
 *     never allocates or frees device memory.  Its only state: the measurement hooks
 *     of dvdq_bench.h, the scratch array of dvdq_qlinear_static, and a fixed 32 KB array
 *     of device memory per GPU (part of the loaded code object) that the GEMM kernels
 *     use as tile counters, 64 bytes per stream.  No launch depends on what an earlier
 *     one left in its counters: they are zeroed on the stream right before every GEMM
 *     that counts in them (by the quantizer kernel when that is what the library enqueued
 *     last on the stream, as in dvdq_qlinear; else by a one-wave kernel in front of the
 *     GEMM), so a launch that never finished or a stray write cannot make a later GEMM
 *     skip tiles.  Calls on one stream from several host threads must be ordered by the
 *     caller, as for any stream.  Kernels of one stream run one after the
 *     other and therefore share a slot; up to 512 streams per GPU hold slots at a time
 *     (dvdq_release_stream gives one back), further streams and launches under stream
 *     capture use fixed tile shares instead (same results; nothing extra is captured).
 *     Two GEMMs must not run at the same time on one stream handle, which HIP rules out
 *     as long as a handle is not used after its stream was destroyed.
 *   - `hip_stream` is the caller's hipStream_t (NULL = the default stream).  All
 *     work is enqueued on it; calls return without synchronizing.
 *   - Inputs are read-only; outputs must not overlap inputs or each other.
 *   - Base pointers must be 16-byte aligned (DVDQ_ERR_ALIGN otherwise).
 *   - Return value: DVDQ_OK (0) or a dvdq_status code.  Argument errors are found
 *     on the host before anything is enqueued.  Nothing is printed, nothing throws.
 *   - NaN / Inf in X: no fault, result unspecified.
 *   - Tensors are dense row-major.  bf16 is passed as `void*` to 16-bit patterns.
 *
 * Activation codes, values in [-qmax, qmax], qmax = 2^(act_bits-1) - 1 (7, 31 or 127
 * for 4, 6, 8 bits), in one of three containers (`codes_format`):
 *   DVDQ_CODES_INT8     int8 [M, K], one code per byte.  Every bit-width.
 *   DVDQ_CODES_PACKED4  uint8 [M, K/2], two 4-bit two's-complement codes per byte, act_bits = 4
 *                       only.  Channels are interleaved within groups of 8: byte b (0..3) of
 *                       group g of a row holds channel 8g+b in bits 0-3 and channel 8g+b+4 in
 *                       bits 4-7.  This is the order in which one shift and two masks turn a
 *                       32-bit word into int8 lanes in channel order; it halves the bytes the
 *                       quantizer writes and the GEMM reads.
 *   DVDQ_CODES_FP6      6 bits per code, act_bits = 4 only, for the FP6 matrix path (twice the INT8
 *                       rate on gfx950): a code c is the E2M3 bit pattern (c < 0) << 5 | |c|, whose
 *                       value is c / 8 exactly.  dvdq_codes_bytes(M, K, DVDQ_CODES_FP6) bytes, K a
 *                       multiple of 128, rows padded to a multiple of 32: blocks of 32 rows outermost,
 *                       then slices of 128 channels; one block-slice is 3072 bytes,
 *                       [16-byte chunk c = 0..5][row 0..31][16 B], where the 96 bytes c = 0..5 of a row
 *                       are four 24-byte fragments f = 0..3 and field e (bits 6e .. 6e+5, little
 *                       endian) of fragment f is channel 64 (f / 2) + 32 (f % 2) + e of the slice.
 *                       Goes with DVDQ_W_NATIVE_FP6 weights only.
 *                       All are passed as `int8_t *`.
 *
 * Weight codes, canonical layout (DVDQ_W_CANONICAL): uint8 [N, K/2]; byte j of
 * row n holds channel 2j in bits 0-3 and channel 2j+1 in bits 4-7, each a 4-bit
 * two's-complement number (offline quantizers produce [-7, 7]; -8 is accepted).
 * Native layout (DVDQ_W_NATIVE): the opaque buffer written by dvdq_w4_prepack,
 * dvdq_w4_native_bytes(N, K) bytes; same information, ordered for the GEMM kernel.
 * FP6 native layout (DVDQ_W_NATIVE_FP6): the buffer written by dvdq_w4_prepack_fp6,
 * dvdq_w4_native_fp6_bytes(N, K) bytes: the same codes as E2M3 patterns in the block-slice
 * order described above (slices outermost, N padded to 256 rows); W4A4 only.
 */
#ifndef DVDQ_H
#define DVDQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    DVDQ_OK = 0,
    DVDQ_ERR_NULL = 1,        /* a required pointer is NULL */
    DVDQ_ERR_SHAPE = 2,       /* M, N, K, had_block inconsistent (non-positive, K % had_block, K odd, ...) */
    DVDQ_ERR_UNSUPPORTED = 3, /* valid request outside what the kernels implement */
    DVDQ_ERR_WORKSPACE = 4,   /* workspace too small */
    DVDQ_ERR_ALIGN = 5,       /* a base pointer is not 16-byte aligned */
    DVDQ_ERR_HIP = 6          /* a kernel launch failed (hipGetLastError) */
} dvdq_status;

enum { DVDQ_W_CANONICAL = 0, DVDQ_W_NATIVE = 1, DVDQ_W_NATIVE_FP6 = 2 };
enum { DVDQ_CODES_INT8 = 0, DVDQ_CODES_PACKED4 = 1, DVDQ_CODES_FP6 = 2 };

/* Bytes of the activation-code buffer for M x K codes in the given container (0 for arguments
 * the container does not admit). */
size_t dvdq_codes_bytes(int64_t M, int64_t K, int codes_format);

/*
 * Rotate + auto-scale + quantize (Sec. 3.2: X~ = XH by fast Hadamard transform,
 * per-row s = ||x~||_inf / qmax, codes = round-half-even(x~ / s) clamped to +-qmax).
 *
 *   x_bf16   in   bf16 [M, K]
 *   had_block     size B of the normalized Walsh-Hadamard blocks (natural/Sylvester
 *                 order, H[i,j] = (-1)^popcount(i&j)/sqrt(B)); every contiguous group
 *                 of B channels is rotated on its own.  Power of two, 1 <= B <= 512,
 *                 B divides K.  B = 1 means no rotation.
 *   act_bits      4, 6 or 8
 *   codes_format  container of the codes (see above); DVDQ_CODES_PACKED4 with act_bits != 4 is
 *                 DVDQ_ERR_UNSUPPORTED
 *   codes    out  int8 [M, K], or uint8 [M, K/2] when packed
 *   x_scale  out  fp32 [M]; 0 for an all-zero row (its codes are all 0)
 *   code_rowsum out  int32 [M] or NULL; when given, receives sum_k codes[m,k], which the GEMM needs
 *                 to apply weight zero-points (see dvdq_w4ax_gemm)
 *
 * K must be a multiple of 8 (DVDQ_ERR_SHAPE) and at most 65536 (DVDQ_ERR_UNSUPPORTED).
 */
int dvdq_rotate_quant(const void *x_bf16, int64_t M, int64_t K, int had_block, int act_bits, int codes_format,
                      int8_t *codes, float *x_scale, int32_t *code_rowsum, void *hip_stream);

/*
 * Block-wise scaled variant of dvdq_rotate_quant (Sec. 3.2 closes by saying the deployed kernels
 * scale block-wise; its definition is in a supplement that is not available, so this is a
 * reading).  Every group of `group` consecutive channels of a token is quantized with its own
 * step, a power-of-two fraction of the token's step s_m = max|x~_m| / qmax:
 *     e_mg = largest e in [0, emax] with  max_{k in g}|x~_mk| * 2^e <= max_k|x~_mk|,   emax = 8 - act_bits
 *     q_mk = clamp(rint(x~_mk / (s_m 2^-e_mg)), -qmax, qmax)
 * and stored in the int8 container as  values[m,k] = q_mk * 2^(emax - e_mg), with
 * x_scale[m] = s_m * 2^-emax, so that x_scale[m] * values[m,k] dequantizes every group and
 * dvdq_w4ax_gemm runs on `values` unchanged: call it with act_bits = 8 (|values| <= 127) and
 * DVDQ_CODES_INT8.  Quiet groups of a token are quantized up to 2^emax times finer at no cost
 * in the GEMM.
 *
 *   act_bits      4 or 6 (8 leaves no headroom: DVDQ_ERR_UNSUPPORTED)
 *   group         128, 256 or 512 channels (DVDQ_ERR_UNSUPPORTED otherwise); must divide K (DVDQ_ERR_SHAPE)
 *   values   out  int8 [M, K]
 *   x_scale  out  fp32 [M]
 *   value_rowsum out int32 [M] or NULL: sum_k values[m,k], for weights with zero-points
 * Other arguments and limits as for dvdq_rotate_quant.
 */
int dvdq_rotate_quant_blockwise(const void *x_bf16, int64_t M, int64_t K, int had_block, int act_bits, int group,
                                int8_t *values, float *x_scale, int32_t *value_rowsum, void *hip_stream);

/*
 * Low-bit GEMM with exact int32 accumulation and the dequantizing epilogue
 * (Sec. 3.2: Y = X^ Lambda W^^T; Sec. 3.1 DeQuant, w^ = Delta (w_q - z)):
 *
 *     acc[m,n] = sum_k codes[m,k] * (w[n,k] - w_zero[n])         (exact, int32; w_zero = 0 when NULL)
 *     y[m,n]   = bf16( float(acc[m,n]) * x_scale[m] * w_scale[n] + bias[n] )
 *
 * The zero-point term is applied as acc - w_zero[n] * code_rowsum[m], so weights with
 * zero-points need the per-token code sums that dvdq_rotate_quant can emit.
 *
 *   codes     in   int8 [M, K] or packed uint8 [M, K/2] per `codes_format`,
 *                  |code| <= 2^(act_bits-1) - 1 (not checked)
 *   x_scale   in   fp32 [M]
 *   w         in   packed INT4 weights, layout per `w_layout`
 *   w_scale   in   fp32 [N]
 *   w_zero    in   int8 [N] or NULL: signed zero-points (the unsigned zero-point of the Quant
 *                  equation minus 8, matching the signed weight codes); native layout only
 *   code_rowsum in int32 [M]: sum_k codes[m,k]; required when w_zero is given (DVDQ_ERR_NULL
 *                  otherwise), ignored when it is NULL
 *   bias_bf16 in   bf16 [N] or NULL
 *   act_bits       4, 6 or 8 (bounds the accumulator: qmax * 8 * K, or qmax * 16 * K with
 *                  zero-points, must stay below 2^27, or 2^23 with packed codes,
 *                  DVDQ_ERR_UNSUPPORTED otherwise: the kernels accumulate 16 * acc, resp. 256 * acc)
 *   codes_format   DVDQ_CODES_PACKED4 needs act_bits = 4 and the native weight layout;
 *                  DVDQ_CODES_FP6 and DVDQ_W_NATIVE_FP6 need each other, act_bits = 4 and
 *                  7 * 8 * K < 2^24 (the fp32 accumulators then hold the integer sums exactly;
 *                  results are bit-identical to the INT8 path) (DVDQ_ERR_UNSUPPORTED otherwise)
 *   y_bf16    out  bf16 [M, N]
 *   acc_out   out  int32 [M, N] or NULL; when given, receives the raw accumulators
 *                  (parity hook; costs extra bandwidth)
 *
 * K must be a multiple of 32 (DVDQ_ERR_SHAPE), and of 128 with the native layouts
 * (DVDQ_ERR_UNSUPPORTED otherwise).  Any M >= 1, N >= 1; ragged tiles are handled inside.
 */
int dvdq_w4ax_gemm(const int8_t *codes, const float *x_scale, const uint8_t *w, const float *w_scale,
                   const int8_t *w_zero, const int32_t *code_rowsum, const void *bias_bf16, int64_t M, int64_t N,
                   int64_t K, int act_bits, int codes_format, int w_layout, void *y_bf16, int32_t *acc_out,
                   void *hip_stream);

/*
 * The whole layer in one call: dvdq_rotate_quant followed by dvdq_w4ax_gemm on
 * the same stream.  `workspace` (device, 256-byte aligned) must hold at least
 * dvdq_qlinear_workspace_bytes(M, K, codes_format) bytes; after the call completes it
 * contains the activation codes (in the container `codes_format` names) at offset 0,
 * the token scales (fp32 [M]) at offset dvdq_qlinear_scale_offset(M, K, codes_format)
 * and, when w_zero is given, the token code sums (int32 [M]) at offset
 * dvdq_qlinear_rowsum_offset(M, K, codes_format), so callers and tests can inspect
 * them.  `codes_format` is the container used between the two kernels; arguments
 * as in the two calls above.
 */
int dvdq_qlinear(const void *x_bf16, const uint8_t *w, const float *w_scale, const int8_t *w_zero,
                 const void *bias_bf16, int64_t M, int64_t N, int64_t K, int had_block, int act_bits,
                 int codes_format, int w_layout, void *y_bf16, void *workspace, size_t workspace_bytes,
                 void *hip_stream);
size_t dvdq_qlinear_workspace_bytes(int64_t M, int64_t K, int codes_format);
size_t dvdq_qlinear_scale_offset(int64_t M, int64_t K, int codes_format);
size_t dvdq_qlinear_rowsum_offset(int64_t M, int64_t K, int codes_format);

/*
 * dvdq_qlinear for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and
 * bit-identical outputs, but the codes, token scales and code sums go to a fixed array of
 * DVDQ_STATIC_WORKSPACE_BYTES of device memory that is part of the library's code object (every GPU
 * the library runs on holds its own copy until the process ends) instead of a caller workspace.
 * Requests with dvdq_qlinear_workspace_bytes(M, K, codes_format) above that size return
 * DVDQ_ERR_WORKSPACE; nothing is enqueued then.  The call allocates nothing and frees nothing.  Its first call
 * on a device looks the array's address up (hipGetSymbolAddress): make that call before a stream
 * capture starts.  All calls on one GPU share the array, which keeps the previous call's contents
 * (every byte a call reads it has written itself, nothing needs clearing): calls that may run
 * concurrently on one GPU, e.g. on two streams, race on it and must be ordered by the caller.
 */
#define DVDQ_STATIC_WORKSPACE_BYTES (64u << 20)
int dvdq_qlinear_static(const void *x_bf16, const uint8_t *w, const float *w_scale, const int8_t *w_zero,
                        const void *bias_bf16, int64_t M, int64_t N, int64_t K, int had_block, int act_bits,
                        int codes_format, int w_layout, void *y_bf16, void *hip_stream);
size_t dvdq_static_workspace_bytes(void);

/*
 * Optional: forget a stream (on the current GPU) before it is destroyed, so that its
 * counter slot can serve another stream.  Host-only bookkeeping, nothing is enqueued;
 * using the stream again later simply assigns a slot again.  Unknown streams: no-op.
 */
int dvdq_release_stream(void *hip_stream);

/*
 * One-time, offline: reorder canonical packed weights into the GEMM kernel's
 * native layout (the rotated, quantized weights of Sec. 3.2 are fixed after
 * quantization, so this runs once per layer).  w_native must hold
 * dvdq_w4_native_bytes(N, K) bytes.  K must be a multiple of 128 (DVDQ_ERR_UNSUPPORTED
 * otherwise; dvdq_w4_native_bytes then returns 0).
 */
int dvdq_w4_prepack(const uint8_t *w_canonical, int64_t N, int64_t K, uint8_t *w_native, void *hip_stream);
size_t dvdq_w4_native_bytes(int64_t N, int64_t K);
/* The same for the FP6 native layout (DVDQ_W_NATIVE_FP6; 6 bits per weight). */
int dvdq_w4_prepack_fp6(const uint8_t *w_canonical, int64_t N, int64_t K, uint8_t *w_native, void *hip_stream);
size_t dvdq_w4_native_fp6_bytes(int64_t N, int64_t K);

/*
 * One-time, offline: Bounded-init Grid Refinement (Sec. 3.1, Alg. 1), the INT4 weight
 * quantizer.  For every row n of w (an output channel, already expressed in the rotated
 * basis W H of Sec. 3.2) it finds a step size Delta_n and an integer zero-point z_n for
 *     Quant    q = clamp(rint(w / Delta) + z, 0, 15)        DeQuant  w^ = Delta (q - z)
 * by searching progressively clipped MinMax ranges [min + i s, max - i s], s = (max - min) / n_steps,
 * while the range is non-empty, refining each start with at most max_refine rounds of
 * {least-squares Delta, relaxed-then-rounded z clamped to [0, 15], re-quantization}, a start's
 * refinement ending with the round that improves the row error ||w - w^||_2 by less than eps.
 * `search` selects what competes for the smallest row error:
 *   DVDQ_BGR_LISTING      Alg. 1 as printed: i = 1, 2, ...; a start's result is the grid of its last
 *                         round (the start itself when max_refine = 0).  n_steps >= 3 (DVDQ_ERR_SHAPE).
 *   DVDQ_BGR_BEST_OF_ALL  a superset search: i = 0 (plain MinMax) is a start too and every grid
 *                         evaluated, each start and every round, competes; never worse than MinMax.
 * Ties keep the earliest grid.  Arithmetic is fp64; rint rounds half to even.
 *
 *   w          in   fp32 [N, K]
 *   n_steps         >= 1 (100 is customary); max_refine >= 0; eps >= 0
 *   w_packed   out  canonical packed codes uint8 [N, K/2]: signed nibbles q - 8
 *   w_scale    out  fp32 [N]: Delta_n
 *   w_zero     out  int8 [N]: z_n - 8, the signed zero-point dvdq_w4ax_gemm takes
 *   row_error  out  fp64 [N] or NULL: ||w_n - w^_n||_2 of the returned grid
 *
 * K must be even (DVDQ_ERR_SHAPE) and at most 32768 (DVDQ_ERR_UNSUPPORTED).  A constant row
 * is represented exactly.  Results do not depend on the launch (no atomics).
 */
enum { DVDQ_BGR_LISTING = 0, DVDQ_BGR_BEST_OF_ALL = 1 };
int dvdq_bgr_quantize(const float *w, int64_t N, int64_t K, int n_steps, int max_refine, double eps, int search,
                      uint8_t *w_packed, float *w_scale, int8_t *w_zero, double *row_error, void *hip_stream);

/*
 * delta-Guided Bit Switching (Sec. 3.3): choose the activation bit-width of the next
 * denoising step from how much the model output changed.
 *
 * `state` is 16 bytes of device memory owned by the caller:
 *     offset 0   double  running sum of relative L1 changes since the last reset
 *     offset 8   float   the change L1(F, t) computed by the latest dvdq_gbs_step
 *     offset 12  int32   bit-width for the next step (read this one scalar back)
 * dvdq_gbs_reset starts a new sampling run: sum 0, bits = initial_bits (the first
 * step has no predecessor to compare with; b_high is the safe choice).
 *
 * dvdq_gbs_step, called after a denoising step produced f_t (bf16, n elements; f_prev
 * is the previous step's output): computes
 *     L1 = sum|f_t - f_prev| / sum|f_prev|          (fp32 per thread, fp64 across threads)
 * adds it to the running sum, and sets bits = b_low while the sum stays below `delta`,
 * or bits = b_high and sum = 0 once it reaches `delta` (the B_{t_i} case equation).
 * A zero denominator gives +inf (or 0 when the numerator is zero too).
 * `workspace`: device, at least dvdq_gbs_workspace_bytes() bytes, scratch.
 * delta >= 0; b_low <= b_high, each 4, 6 or 8.  Results are bit-reproducible (no atomics).
 */
size_t dvdq_gbs_workspace_bytes(void);
int dvdq_gbs_reset(void *state, int initial_bits, void *hip_stream);
int dvdq_gbs_step(const void *f_t_bf16, const void *f_prev_bf16, int64_t n, float delta, int b_low, int b_high,
                  void *state, void *workspace, size_t workspace_bytes, void *hip_stream);

const char *dvdq_status_string(int status);
int dvdq_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DVDQ_H */

/*
 * CPU oracle for the rotated, auto-scaled, low-bit quantized linear layer.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a deliberately plain,
 * slow, fp64 / int64 restatement of what the layer computes, written so that a
 * reader can check it against the method section by eye.  It shares no code,
 * header, table or helper with the GPU library and is never called by it; only
 * the tests, the smoke check and the benchmark's CPU-baseline leg use it.
 *
 * What it computes, step by step (method Sec. 3.2, the ARQ equation
 *   X^ = Q(X H Lambda^-1),  Y = X^ Lambda W^^T ;  dequantization as in Sec. 3.1):
 *
 *   1. X~ = X * blockdiag(H_B)          dense fp64 matrix product, no butterfly
 *   2. s_m = max_k |x~_mk| / qmax       one online scale per token row
 *   3. q_mk = clamp(rint(x~_mk / s_m))  symmetric codes, round-half-to-even
 *   4. acc_mn = sum_k q_mk * w_nk       exact integer sum (int64)
 *   5. y_mn = bf16(acc_mn * s_m * ws_n [+ bias_n])
 *
 * Readings taken where the text leaves a choice (per-token scale granularity,
 * symmetric range +-(2^(b-1)-1), Sylvester ordering of H, tie rule, nibble
 * order) are listed in the repository's design notes; each function below says
 * which one it relies on.
 *
 * Further down: the delta-guided bit switching controller (Sec. 3.3), the offline
 * weight quantizer (Sec. 3.1: MinMax start, grid refinement, Alg. 1) and the GEMM
 * with weight zero-points.
 *
 * Parity status: every function here is pinned by CPU tests against closed
 * forms, hand-derived examples, a library Hadamard matrix, a library least-squares
 * solver, and brute force on tiny shapes.  Nothing about video quality is pinned
 * (it needs the real model).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---------------------------------------------------------------- bf16 */

/* bf16 bit pattern -> double (exact). */
static double bf16_to_f64(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/* double -> bf16 bit pattern with a single round-to-nearest-even
 * (not via float, which would round twice). */
static uint16_t f64_to_bf16(double v)
{
    if (isnan(v)) return 0x7FC0;
    if (isinf(v)) return v > 0 ? 0x7F80 : 0xFF80;
    if (v == 0.0) return signbit(v) ? 0x8000 : 0x0000;
    int e = ilogb(v);                 /* v = m * 2^e, 1 <= |m| < 2 */
    if (e < -126) e = -126;           /* subnormal bf16 range: fixed quantum */
    double quantum = ldexp(1.0, e - 7);
    double r = nearbyint(v / quantum) * quantum;   /* both scalings are exact */
    float f = (float)r;               /* r has <= 8 significant bits: exact, or inf on overflow */
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    return (uint16_t)(u >> 16);
}

void dvdq_oracle_f64_to_bf16(const double *in, int64_t n, uint16_t *out)
{
    for (int64_t i = 0; i < n; ++i) out[i] = f64_to_bf16(in[i]);
}

/* ---------------------------------------------------------------- Hadamard */

/* Dense normalized Walsh-Hadamard matrix of order B (a power of two) by the
 * Sylvester recursion H_1 = [1], H_2n = [[H_n, H_n], [H_n, -H_n]], scaled by
 * 1/sqrt(B) so that H H^T = I (the orthogonality the rotation relies on,
 * Sec. 3.2).  Row-major, B*B doubles.  Returns 0, or -1 if B is not a power of two. */
int dvdq_oracle_hadamard(int B, double *H)
{
    if (B < 1 || (B & (B - 1)) != 0) return -1;
    H[0] = 1.0;
    for (int n = 1; n < B; n *= 2) {
        /* grow the top-left n x n block (stride B) into 2n x 2n */
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < n; ++j) {
                double h = H[(size_t)i * B + j];
                H[(size_t)i * B + (j + n)] = h;
                H[(size_t)(i + n) * B + j] = h;
                H[(size_t)(i + n) * B + (j + n)] = -h;
            }
    }
    double norm = 1.0 / sqrt((double)B);
    for (size_t i = 0; i < (size_t)B * B; ++i) H[i] *= norm;
    return 0;
}

/* X~ = X * blockdiag(H_B, ..., H_B): every contiguous group of B channels of a
 * token row is multiplied by H_B (Sec. 3.2, X~ = XH; block-diagonal reading for
 * channel counts that are not a power of two).  x: bf16 bits [M,K]; xrot: fp64 [M,K].
 * Returns 0, -1 bad B, -2 B does not divide K. */
int dvdq_oracle_rotate(const uint16_t *x, int64_t M, int64_t K, int B, double *xrot)
{
    if (B < 1 || (B & (B - 1)) != 0) return -1;
    if (K % B != 0) return -2;
    double *H = (double *)malloc(sizeof(double) * (size_t)B * B);
    if (!H) return -3;
    dvdq_oracle_hadamard(B, H);
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        double *xin = (double *)malloc(sizeof(double) * (size_t)B);
        for (int64_t g = 0; g < K / B; ++g) {
            const uint16_t *xb = x + m * K + g * B;
            double *ob = xrot + m * K + g * B;
            for (int i = 0; i < B; ++i) xin[i] = bf16_to_f64(xb[i]);
            for (int j = 0; j < B; ++j) {
                double s = 0.0;
                for (int i = 0; i < B; ++i) s += xin[i] * H[(size_t)i * B + j];
                ob[j] = s;
            }
        }
        free(xin);
    }
    free(H);
    return 0;
}

/* ---------------------------------------------------------------- quantizer */

/* Steps 2-3 on already rotated rows.  qmax = 2^(bits-1) - 1.  The scale is
 * rounded once to fp32 (that fp32 number is the scale the layer hands on) and
 * the codes are taken against exactly that number.  A zero row gives scale 0
 * and all-zero codes. */
int dvdq_oracle_quantize(const double *xrot, int64_t M, int64_t K, int bits,
                         int8_t *codes, float *x_scale)
{
    if (bits < 2 || bits > 8) return -1;
    const double qmax = (double)((1 << (bits - 1)) - 1);
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        const double *r = xrot + m * K;
        double amax = 0.0;
        for (int64_t k = 0; k < K; ++k) {
            double a = fabs(r[k]);
            if (a > amax) amax = a;
        }
        float s = (float)(amax / qmax);      /* round-to-nearest-even to fp32 */
        x_scale[m] = s;
        if (!(s > 0.0f)) {
            for (int64_t k = 0; k < K; ++k) codes[m * K + k] = 0;
            continue;
        }
        double sd = (double)s;
        for (int64_t k = 0; k < K; ++k) {
            double q = nearbyint(r[k] / sd);  /* default FP environment: ties to even */
            if (q > qmax) q = qmax;
            if (q < -qmax) q = -qmax;
            codes[m * K + k] = (int8_t)q;
        }
    }
    return 0;
}

/* Block-wise variant of steps 2-3 (Sec. 3.2, last paragraph: the deployed kernels scale block-wise,
 * the definition being in a supplement that is not available; this is a reading).  Every group of
 * `group` consecutive channels of a token gets its own step size, a power-of-two fraction of the
 * token's:
 *     s_m     = max_k |x~_mk| / qmax                         (as in step 2, rounded once to fp32)
 *     e_mg    = the largest e in [0, emax] with  a_mg * 2^e <= max_k |x~_mk|,  a_mg = max_{k in g} |x~_mk|
 *     s_mg    = s_m * 2^-e_mg
 *     q_mk    = clamp(rint(x~_mk / s_mg), -qmax, qmax)
 * so a quiet group is quantized up to 2^emax times finer.  Because the ratios are powers of two the
 * group scales fold into an int8 container: the stored value is v_mk = q_mk * 2^(emax - e_mg), the
 * scale handed on is s'_m = s_m * 2^-emax, and s'_m * v_mk = s_mg * q_mk; the integer GEMM runs on v
 * unchanged.  emax = 8 - bits (|v| <= qmax * 2^emax <= 127).  exps_out ([M, K/group]) may be NULL. */
int dvdq_oracle_quantize_blockwise(const double *xrot, int64_t M, int64_t K, int bits, int group,
                                   int8_t *values, float *x_scale, uint8_t *exps_out)
{
    if (bits < 2 || bits > 8 || group < 1 || K % group) return -1;
    const double qmax = (double)((1 << (bits - 1)) - 1);
    const int emax = 8 - bits;
    const int64_t G = K / group;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        const double *r = xrot + m * K;
        double amax = 0.0;
        for (int64_t k = 0; k < K; ++k) if (fabs(r[k]) > amax) amax = fabs(r[k]);
        const float s = (float)(amax / qmax);
        x_scale[m] = (float)ldexp((double)s, -emax);
        for (int64_t g = 0; g < G; ++g) {
            double a = 0.0;
            for (int64_t k = g * group; k < (g + 1) * group; ++k) if (fabs(r[k]) > a) a = fabs(r[k]);
            int e = 0;
            for (int t = 1; t <= emax; ++t) if (ldexp(a, t) <= amax) e = t;
            if (exps_out) exps_out[m * G + g] = (uint8_t)e;
            for (int64_t k = g * group; k < (g + 1) * group; ++k) {
                double q = 0.0;
                if (s > 0.0f) {
                    q = nearbyint(r[k] / ldexp((double)s, -e));
                    if (q > qmax) q = qmax;
                    if (q < -qmax) q = -qmax;
                }
                values[m * K + k] = (int8_t)ldexp(q, emax - e);
            }
        }
    }
    return 0;
}

/* Steps 1-3 in one call.  xrot_out may be NULL. */
int dvdq_oracle_rotate_quant(const uint16_t *x, int64_t M, int64_t K, int B, int bits,
                             int8_t *codes, float *x_scale, double *xrot_out)
{
    double *xr = xrot_out ? xrot_out : (double *)malloc(sizeof(double) * (size_t)M * K);
    if (!xr) return -3;
    int rc = dvdq_oracle_rotate(x, M, K, B, xr);
    if (rc == 0) rc = dvdq_oracle_quantize(xr, M, K, bits, codes, x_scale);
    if (!xrot_out) free(xr);
    return rc;
}

/* ---------------------------------------------------------------- weights */

/* Canonical packed INT4 -> int8 codes.  Byte j of a row carries channel 2j in
 * bits 0-3 and channel 2j+1 in bits 4-7, each a 4-bit two's-complement number. */
void dvdq_oracle_unpack_w4(const uint8_t *packed, int64_t N, int64_t K, int8_t *codes)
{
    for (int64_t n = 0; n < N; ++n)
        for (int64_t j = 0; j < K / 2; ++j) {
            int lo = packed[n * (K / 2) + j] & 0xF;
            int hi = (packed[n * (K / 2) + j] >> 4) & 0xF;
            codes[n * K + 2 * j] = (int8_t)(lo >= 8 ? lo - 16 : lo);
            codes[n * K + 2 * j + 1] = (int8_t)(hi >= 8 ? hi - 16 : hi);
        }
}

/* Inverse of the above, for the pack/unpack round-trip pin. */
void dvdq_oracle_pack_w4(const int8_t *codes, int64_t N, int64_t K, uint8_t *packed)
{
    for (int64_t n = 0; n < N; ++n)
        for (int64_t j = 0; j < K / 2; ++j) {
            int lo = codes[n * K + 2 * j] & 0xF;
            int hi = codes[n * K + 2 * j + 1] & 0xF;
            packed[n * (K / 2) + j] = (uint8_t)(lo | (hi << 4));
        }
}

/* ---------------------------------------------------------------- packed activation codes */

/* The 4-bit container of activation codes between quantizer and GEMM (an encoding of
 * this library, not of the method: the codes themselves are the ARQ codes of Sec. 3.2).
 * A row of K codes becomes K/2 bytes; within each group of 8 channels, byte b (0..3)
 * carries channel 8g+b in bits 0-3 and channel 8g+b+4 in bits 4-7, two's complement. */
void dvdq_oracle_unpack_a4(const uint8_t *packed, int64_t M, int64_t K, int8_t *codes)
{
    for (int64_t m = 0; m < M; ++m)
        for (int64_t g = 0; g < K / 8; ++g)
            for (int b = 0; b < 4; ++b) {
                int byte = packed[m * (K / 2) + 4 * g + b];
                int lo = byte & 0xF, hi = (byte >> 4) & 0xF;
                codes[m * K + 8 * g + b] = (int8_t)(lo >= 8 ? lo - 16 : lo);
                codes[m * K + 8 * g + b + 4] = (int8_t)(hi >= 8 ? hi - 16 : hi);
            }
}

void dvdq_oracle_pack_a4(const int8_t *codes, int64_t M, int64_t K, uint8_t *packed)
{
    for (int64_t m = 0; m < M; ++m)
        for (int64_t g = 0; g < K / 8; ++g)
            for (int b = 0; b < 4; ++b) {
                int lo = codes[m * K + 8 * g + b] & 0xF;
                int hi = codes[m * K + 8 * g + b + 4] & 0xF;
                packed[m * (K / 2) + 4 * g + b] = (uint8_t)(lo | (hi << 4));
            }
}

/* The FP6 container of 4-bit activation codes (the GPU library's own encoding for the FP6 matrix path,
 * stated in its C header; no passage of the method defines it).  A code c, |c| <= 15, is stored as the
 * 6-bit E2M3 pattern  (c < 0) << 5 | |c|,  whose value as an E2M3 number is c / 8.  Rows are padded to a
 * multiple of 32, K is a multiple of 128.  With block = m / 32, r = m % 32, slice = k / 128, c = k % 128:
 * the row's 128 fields of a slice are 96 bytes, field c at bits 6 c .. 6 c + 5 (little endian), and byte b
 * of those 96 lives at
 *     ((block * (K / 128) + slice) * 6 + b / 16) * 512 + r * 16 + b % 16
 * i.e. [32-row block][128-channel slice][16-byte chunk 0..5][row 0..31][16 B].  One field, one bit at a time. */
void dvdq_oracle_pack_fp6(const int8_t *codes, int64_t M, int64_t K, uint8_t *buf)
{
    const int64_t slices = K / 128, blocks = (M + 31) / 32;
    memset(buf, 0, (size_t)(blocks * 32 * slices * 96));
#pragma omp parallel for schedule(static)   /* rows own disjoint bytes */
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k) {
            const int c = codes[m * K + k];
            const int field = (c < 0 ? 32 : 0) | (c < 0 ? -c : c);
            const int64_t base = ((m / 32) * slices + k / 128) * 6 * 512 + (m % 32) * 16;
            for (int bit = 0; bit < 6; ++bit) {
                if (!((field >> bit) & 1)) continue;
                const int pos = 6 * (int)(k % 128) + bit;     /* bit of the row's 96 bytes */
                const int b = pos / 8;
                buf[base + (b / 16) * 512 + b % 16] |= (uint8_t)(1u << (pos % 8));
            }
        }
}

void dvdq_oracle_unpack_fp6(const uint8_t *buf, int64_t M, int64_t K, int8_t *codes)
{
    const int64_t slices = K / 128;
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t k = 0; k < K; ++k) {
            const int64_t base = ((m / 32) * slices + k / 128) * 6 * 512 + (m % 32) * 16;
            int field = 0;
            for (int bit = 0; bit < 6; ++bit) {
                const int pos = 6 * (int)(k % 128) + bit;
                const int b = pos / 8;
                field |= ((buf[base + (b / 16) * 512 + b % 16] >> (pos % 8)) & 1) << bit;
            }
            const int mag = field & 31;
            codes[m * K + k] = (int8_t)((field & 32) ? -mag : mag);
        }
}

/* ---------------------------------------------------------------- GEMM */

/* Step 4: acc[m,n] = sum_k q[m,k] * w[n,k], the plain definition, in int64. */
void dvdq_oracle_int_gemm(const int8_t *q, const int8_t *w, int64_t M, int64_t N, int64_t K,
                          int64_t *acc)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            int64_t s = 0;
            for (int64_t k = 0; k < K; ++k)
                s += (int64_t)q[m * K + k] * (int64_t)w[n * K + k];
            acc[m * N + n] = s;
        }
}

/* Step 5: rescale by the token scale (Lambda) and the weight step size (Delta),
 * add the optional bias, round once to bf16.  bias may be NULL. */
void dvdq_oracle_epilogue(const int64_t *acc, const float *x_scale, const float *w_scale,
                          const uint16_t *bias, int64_t M, int64_t N, uint16_t *y)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            double v = (double)acc[m * N + n] * (double)x_scale[m] * (double)w_scale[n];
            if (bias) v += bf16_to_f64(bias[n]);
            y[m * N + n] = f64_to_bf16(v);
        }
}

/* Steps 4-5 from codes (the GEMM half of the layer). acc_out may be NULL. */
int dvdq_oracle_w4ax_gemm(const int8_t *codes, const float *x_scale, const uint8_t *w_packed,
                          const float *w_scale, const uint16_t *bias,
                          int64_t M, int64_t N, int64_t K, uint16_t *y, int64_t *acc_out)
{
    if (K % 2) return -2;
    int8_t *w = (int8_t *)malloc((size_t)N * K);
    int64_t *acc = acc_out ? acc_out : (int64_t *)malloc(sizeof(int64_t) * (size_t)M * N);
    if (!w || !acc) { free(w); if (!acc_out) free(acc); return -3; }
    dvdq_oracle_unpack_w4(w_packed, N, K, w);
    dvdq_oracle_int_gemm(codes, w, M, N, K, acc);
    dvdq_oracle_epilogue(acc, x_scale, w_scale, bias, M, N, y);
    free(w);
    if (!acc_out) free(acc);
    return 0;
}

/* The whole layer, steps 1-5.  codes_out / scale_out / acc_out may be NULL. */
int dvdq_oracle_qlinear(const uint16_t *x, const uint8_t *w_packed, const float *w_scale,
                        const uint16_t *bias, int64_t M, int64_t N, int64_t K, int B, int bits,
                        uint16_t *y, int8_t *codes_out, float *scale_out, int64_t *acc_out)
{
    int8_t *codes = codes_out ? codes_out : (int8_t *)malloc((size_t)M * K);
    float *scale = scale_out ? scale_out : (float *)malloc(sizeof(float) * (size_t)M);
    int rc = -3;
    if (codes && scale) {
        rc = dvdq_oracle_rotate_quant(x, M, K, B, bits, codes, scale, NULL);
        if (rc == 0) rc = dvdq_oracle_w4ax_gemm(codes, scale, w_packed, w_scale, bias, M, N, K, y, acc_out);
    }
    if (!codes_out) free(codes);
    if (!scale_out) free(scale);
    return rc;
}

/* ---------------------------------------------------------------- delta-Guided Bit Switching (Sec. 3.3) */

/* Relative L1 change between successive model outputs,
 *   L1(F, t) = ||F_t - F_{t-1}||_1 / ||F_{t-1}||_1,
 * on bf16 tensors of n elements, summed in fp64.  A zero denominator gives +inf when
 * the numerator is positive and 0 when both are zero. */
double dvdq_oracle_rel_l1(const uint16_t *f_t, const uint16_t *f_prev, int64_t n)
{
    double num = 0.0, den = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        double a = bf16_to_f64(f_t[i]), b = bf16_to_f64(f_prev[i]);
        num += fabs(a - b);
        den += fabs(b);
    }
    if (den == 0.0) return num > 0.0 ? INFINITY : 0.0;
    return num / den;
}

/* One update of the bit-width controller after a denoising step has produced its
 * output: the change of that step is added to the running sum kept since the last
 * reset; while the sum stays below delta the next step runs at b_low, and once it
 * reaches delta the next step runs at b_high and the sum restarts from zero.
 * *acc is the running sum (in/out).  Returns the bit-width for the next step. */
int dvdq_oracle_gbs_update(double l1, double delta, int b_low, int b_high, double *acc)
{
    *acc += l1;
    if (*acc >= delta) {
        *acc = 0.0;
        return b_high;
    }
    return b_low;
}

/* ---------------------------------------------------------------- offline weight quantizer (Sec. 3.1)
 *
 * Asymmetric b-bit quantization of one weight row (one output channel):
 *     Quant    q = clamp(rint(w / Delta) + z, 0, 2^b - 1)
 *     DeQuant  w^ = Delta * (q - z)
 * rint = round half to even; z an integer in [0, 2^b - 1].
 */

static double rint_clamp(double v, double lo, double hi)
{
    double r = nearbyint(v);     /* default rounding mode: ties to even */
    return r < lo ? lo : (r > hi ? hi : r);
}

/* q_k and the row error ||w - Delta (q - z)||_2 for a given grid. */
static double quant_row(const float *w, int64_t K, double delta, double z, double qmax, uint8_t *q)
{
    double e2 = 0.0;
    for (int64_t k = 0; k < K; ++k) {
        double c = nearbyint((double)w[k] / delta) + z;   /* round (ties to even), then shift by z */
        c = c < 0.0 ? 0.0 : (c > qmax ? qmax : c);
        q[k] = (uint8_t)c;
        double r = (double)w[k] - delta * (c - z);
        e2 += r * r;
    }
    return sqrt(e2);
}

/* The MinMax start (Sec. 3.1, the text under the Quant/DeQuant equations), with the range
 * [lo, hi] given: Delta = (hi - lo) / (2^b - 1), z = clamp(-rint(lo / Delta), 0, 2^b - 1). */
static void minmax_grid(double lo, double hi, double qmax, double *delta, double *z)
{
    *delta = (hi - lo) / qmax;
    *z = rint_clamp(-(lo / *delta), 0.0, qmax);
}

/* One round of grid refinement (Sec. 3.1, the three primed equations): with the codes q and
 * zero-point z fixed, Delta' is the least-squares step size <q - z, w> / <q - z, q - z>; with
 * Delta' and q fixed, z' = clamp(rint(mean(q) - mean(w) / Delta'), 0, 2^b - 1); then the codes
 * are re-quantized on the new grid.  Returns 0, or -1 when the step is undefined (all codes
 * equal the zero-point, or a non-positive step size), leaving the outputs untouched. */
int dvdq_oracle_bgr_refine_step(const float *w, int64_t K, int bits, const uint8_t *q, int z,
                                double *delta_out, int *z_out, uint8_t *q_out, double *err_out)
{
    const double qmax = (double)((1 << bits) - 1);
    double num = 0.0, den = 0.0, sq = 0.0, sw = 0.0;
    for (int64_t k = 0; k < K; ++k) {
        double d = (double)q[k] - (double)z;
        num += d * (double)w[k];
        den += d * d;
        sq += (double)q[k];
        sw += (double)w[k];
    }
    if (den == 0.0) return -1;
    double delta = num / den;
    if (!(delta > 0.0)) return -1;
    double zn = rint_clamp(sq / (double)K - (sw / (double)K) / delta, 0.0, qmax);
    *err_out = quant_row(w, K, delta, zn, qmax, q_out);
    *delta_out = delta;
    *z_out = (int)zn;
    return 0;
}

/* Plain MinMax quantization of every row (the baseline the method improves on). */
int dvdq_oracle_minmax_quant(const float *w, int64_t N, int64_t K, int bits, uint8_t *q, double *delta, int *zero,
                             double *err)
{
    const double qmax = (double)((1 << bits) - 1);
    for (int64_t n = 0; n < N; ++n) {
        const float *row = w + n * K;
        double lo = row[0], hi = row[0];
        for (int64_t k = 1; k < K; ++k) { if (row[k] < lo) lo = row[k]; if (row[k] > hi) hi = row[k]; }
        if (!(hi > lo)) return -2;
        double d, z;
        minmax_grid(lo, hi, qmax, &d, &z);
        err[n] = quant_row(row, K, d, z, qmax, q + n * K);
        delta[n] = d;
        zero[n] = (int)z;
    }
    return 0;
}

/* Bounded-init Grid Refinement (Alg. 1), row by row, in two search modes.
 *
 * search = 0, "the listing": Alg. 1 as printed wherever it can be executed.
 *   for i = 1, 2, ...:  clip range [min + i * step, max - i * step], step = (max - min) / n_steps
 *     start grid (Delta0, z0) = MinMax of the clipped row, codes and error E0 of the UNCLIPPED row on it
 *     repeat  round j = 1, 2, ...: least-squares Delta, relaxed zero-point, re-quantize, error Ej
 *     until   the round gained less than eps (or lost):  E(j-1) - E(j) < eps
 *     the start's result is its LAST round's grid (also when that round made the error worse);
 *     it replaces the best grid so far iff its error is strictly smaller.
 *   Only the readings the listing forces are taken: the stop test's operands are taken in the order that
 *   makes it a convergence test (as printed, E(j-1) - E(j-2) < eps holds after every improving round);
 *   the count of shrink steps is a parameter of its own (the listing reuses the row count's letter);
 *   a range that has collapsed (lo >= hi, which happens from i = n_steps / 2 on) ends the search; the
 *   zero-point is rounded and clamped to [0, 2^b - 1] ("relax then round", and the start's must fit the
 *   same container); a round that is undefined (all codes at the zero-point, non-positive step) ends the
 *   start with the grid before it; at most max_refine rounds per start (max_refine = 0: the start itself
 *   is the result); rows are independent (one best grid per row).  n_steps >= 3, so that i = 1 exists.
 * search = 1, "best of everything": a superset search.  i starts at 0 (plain MinMax) and EVERY grid
 *   evaluated -- each start and every round -- competes for best, so the result is never worse than MinMax
 *   or any clipped start.  Not what the listing says; kept as an option.
 * Ties keep the earliest grid in both modes.
 * A constant row c is represented exactly: Delta = |c| (1 if c = 0), z = (c < 0), q = (c > 0). */
int dvdq_oracle_bgr(const float *w, int64_t N, int64_t K, int bits, int n_steps, int max_refine, double eps,
                    int search, uint8_t *q_out, double *delta_out, int *zero_out, double *err_out)
{
    if (bits < 2 || bits > 8 || n_steps < 1 || max_refine < 0 || K < 1) return -1;
    if (search != 0 && search != 1) return -1;
    if (search == 0 && n_steps < 3) return -1;
    const double qmax = (double)((1 << bits) - 1);
    int rc = 0;
#pragma omp parallel for schedule(dynamic)
    for (int64_t n = 0; n < N; ++n) {
        const float *row = w + n * K;
        uint8_t *q = (uint8_t *)malloc((size_t)K), *qn = (uint8_t *)malloc((size_t)K);
        if (!q || !qn) { rc = -3; free(q); free(qn); continue; }
        double lo0 = row[0], hi0 = row[0];
        for (int64_t k = 1; k < K; ++k) { if (row[k] < lo0) lo0 = row[k]; if (row[k] > hi0) hi0 = row[k]; }
        if (!(hi0 > lo0)) {
            const double c = lo0;
            delta_out[n] = c == 0.0 ? 1.0 : fabs(c);
            zero_out[n] = c < 0.0;
            for (int64_t k = 0; k < K; ++k) q_out[n * K + k] = (uint8_t)(c > 0.0);
            err_out[n] = 0.0;
            free(q); free(qn);
            continue;
        }
        const double step = (hi0 - lo0) / (double)n_steps;
        double best = INFINITY;
        for (int i = search == 0 ? 1 : 0; i <= n_steps; ++i) {
            const double lo = lo0 + (double)i * step, hi = hi0 - (double)i * step;
            if (!(lo < hi)) break;
            double delta, z;
            minmax_grid(lo, hi, qmax, &delta, &z);
            double e = quant_row(row, K, delta, z, qmax, q);
            if (search == 1 && e < best) {
                best = e; delta_out[n] = delta; zero_out[n] = (int)z;
                memcpy(q_out + n * K, q, (size_t)K);
            }
            int zi = (int)z;
            for (int j = 0; j < max_refine; ++j) {
                double dn, en; int zn;
                if (dvdq_oracle_bgr_refine_step(row, K, bits, q, zi, &dn, &zn, qn, &en) != 0) break;
                if (search == 1 && en < best) {
                    best = en; delta_out[n] = dn; zero_out[n] = zn;
                    memcpy(q_out + n * K, qn, (size_t)K);
                }
                const double gain = e - en;
                e = en; delta = dn; zi = zn;              /* the start's current (last) grid */
                memcpy(q, qn, (size_t)K);
                if (gain < eps) break;
            }
            if (search == 0 && e < best) {               /* the listing: only the start's last grid competes */
                best = e; delta_out[n] = delta; zero_out[n] = zi;
                memcpy(q_out + n * K, q, (size_t)K);
            }
        }
        err_out[n] = best;
        free(q); free(qn);
    }
    return rc;
}

/* ---------------------------------------------------------------- GEMM with weight zero-points
 *
 * Steps 4-5 for asymmetric weights (DeQuant of Sec. 3.1 inside Y = X^ Lambda W^^T):
 *     acc_mn = sum_k q_mk * (c_nk - z_n),    y_mn = bf16(acc_mn * s_m * ws_n [+ bias_n])
 * with c the stored signed 4-bit codes and z the signed zero-point (both the unsigned
 * quantities of the Quant equation minus 8).  Also returns, when asked, the per-token code
 * sums sum_k q_mk that a kernel needs to apply z outside its integer GEMM. */
int dvdq_oracle_w4ax_gemm_zp(const int8_t *codes, const float *x_scale, const uint8_t *w_packed,
                             const float *w_scale, const int8_t *w_zero, const uint16_t *bias,
                             int64_t M, int64_t N, int64_t K, uint16_t *y, int64_t *acc_out, int64_t *rowsum_out)
{
    if (K % 2) return -2;
    int8_t *w = (int8_t *)malloc((size_t)N * K);
    int64_t *acc = acc_out ? acc_out : (int64_t *)malloc(sizeof(int64_t) * (size_t)M * N);
    if (!w || !acc) { free(w); if (!acc_out) free(acc); return -3; }
    dvdq_oracle_unpack_w4(w_packed, N, K, w);
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m) {
        for (int64_t n = 0; n < N; ++n) {
            int64_t s = 0;
            for (int64_t k = 0; k < K; ++k)
                s += (int64_t)codes[m * K + k] * ((int64_t)w[n * K + k] - (int64_t)w_zero[n]);
            acc[m * N + n] = s;
        }
        if (rowsum_out) {
            int64_t s = 0;
            for (int64_t k = 0; k < K; ++k) s += codes[m * K + k];
            rowsum_out[m] = s;
        }
    }
    dvdq_oracle_epilogue(acc, x_scale, w_scale, bias, M, N, y);
    free(w);
    if (!acc_out) free(acc);
    return 0;
}

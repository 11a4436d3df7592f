// C ABI of libdvdq: argument validation on the host, then kernel launches.
// Every check happens before anything is enqueued; no entry point allocates,
// frees or synchronizes.
#include "dvdq_internal.h"

// Workspace of dvdq_qlinear_static: device memory that is part of the loaded code object, one copy per GPU,
// held until the process ends.  In host code this name is only a handle for hipGetSymbolAddress; the
// address of a GPU's copy is looked up once per device (scratch_ptr below) and that pointer is what
// the kernels get.
static __device__ __align__(256) uint8_t scratch[DVDQ_STATIC_WORKSPACE_BYTES];

namespace {

// Address of the current device's copy of `scratch` (nullptr on failure).  Looked up on the first call
// per device, with that device current; later calls only read the table.
uint8_t *scratch_ptr() {
    static std::atomic<uint8_t *> table[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
        (void)hipGetLastError();
        return nullptr;
    }
    uint8_t *p = table[dev].load(std::memory_order_acquire);
    if (p) return p;
    void *addr = nullptr;
    if (hipGetSymbolAddress(&addr, HIP_SYMBOL(scratch)) != hipSuccess || !addr) {
        (void)hipGetLastError();
        return nullptr;
    }
    table[dev].store(static_cast<uint8_t *>(addr), std::memory_order_release);
    return static_cast<uint8_t *>(addr);
}

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

inline int log2_exact(int v) {
    if (v < 1 || (v & (v - 1)) != 0) return -1;
    int l = 0;
    while ((1 << l) < v) ++l;
    return l;
}

inline bool bits_ok(int b) { return b == 4 || b == 6 || b == 8; }

// container of the activation codes: packed nibbles and FP6 fields only hold 4-bit codes
inline int check_format(int codes_format, int act_bits) {
    if (codes_format == DVDQ_CODES_INT8) return DVDQ_OK;
    if ((codes_format == DVDQ_CODES_PACKED4 || codes_format == DVDQ_CODES_FP6) && act_bits == 4) return DVDQ_OK;
    return DVDQ_ERR_UNSUPPORTED;
}

inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

int check_rotate_quant(const void *x, int64_t M, int64_t K, int had_block, int act_bits, int codes_format,
                       const void *codes, const void *x_scale, const void *code_rowsum, int *log2b) {
    if (!x || !codes || !x_scale) return DVDQ_ERR_NULL;
    if (M < 1 || K < 1 || (K % 8) != 0) return DVDQ_ERR_SHAPE;
    *log2b = log2_exact(had_block);
    if (*log2b < 0 || (K % had_block) != 0) return DVDQ_ERR_SHAPE;
    if (!bits_ok(act_bits) || had_block > 512 || K > 65536 || M > 0x7FFFFFFF) return DVDQ_ERR_UNSUPPORTED;
    if (check_format(codes_format, act_bits) != DVDQ_OK) return DVDQ_ERR_UNSUPPORTED;
    if (codes_format == DVDQ_CODES_FP6 && (K % 128) != 0) return DVDQ_ERR_UNSUPPORTED;
    if (!aligned16(x) || !aligned16(codes) || !aligned16(x_scale) || (code_rowsum && !aligned16(code_rowsum)))
        return DVDQ_ERR_ALIGN;
    return DVDQ_OK;
}

int check_gemm(const void *codes, const void *x_scale, const void *w, const void *w_scale, const void *w_zero,
               const void *code_rowsum, const void *bias, int64_t M, int64_t N, int64_t K, int act_bits,
               int codes_format, int w_layout, const void *y, const void *acc_out) {
    if (!codes || !x_scale || !w || !w_scale || !y || (w_zero && !code_rowsum)) return DVDQ_ERR_NULL;
    if (M < 1 || N < 1 || K < 1 || (K % 32) != 0) return DVDQ_ERR_SHAPE;
    if (!bits_ok(act_bits) ||
        (w_layout != DVDQ_W_CANONICAL && w_layout != DVDQ_W_NATIVE && w_layout != DVDQ_W_NATIVE_FP6))
        return DVDQ_ERR_UNSUPPORTED;
    if (w_layout != DVDQ_W_CANONICAL && (K % 128) != 0) return DVDQ_ERR_UNSUPPORTED;
    if (check_format(codes_format, act_bits) != DVDQ_OK) return DVDQ_ERR_UNSUPPORTED;
    if (codes_format == DVDQ_CODES_PACKED4 && w_layout != DVDQ_W_NATIVE) return DVDQ_ERR_UNSUPPORTED;
    if ((codes_format == DVDQ_CODES_FP6) != (w_layout == DVDQ_W_NATIVE_FP6)) return DVDQ_ERR_UNSUPPORTED;
    if (w_zero && w_layout == DVDQ_W_CANONICAL) return DVDQ_ERR_UNSUPPORTED;
    if (M > 0x7FFFFFFF || N > 0x7FFFFFFF || K > 0x7FFFFFFF) return DVDQ_ERR_UNSUPPORTED;
    // FP6 matrix path: sums of code products, |code| <= 7, |w| <= 8, must be exact in fp32
    if (codes_format == DVDQ_CODES_FP6 && 7 * 8 * K >= (int64_t)1 << 24) return DVDQ_ERR_UNSUPPORTED;
    // the kernel accumulates 16 * sum(code * w), or 256 * with packed codes: |code| <= qmax, |w| <= 8,
    // and |w - zero| <= 16 once a zero-point is taken out; the code sums must fit 24 bits for its multiply
    const int64_t qmax = (1 << (act_bits - 1)) - 1;
    const int64_t widen = codes_format == DVDQ_CODES_PACKED4 ? 256 : (codes_format == DVDQ_CODES_FP6 ? 1 : 16);
    if (widen * qmax * (w_zero ? 16 : 8) * K >= (int64_t)1 << 31) return DVDQ_ERR_UNSUPPORTED;
    if (w_zero && qmax * K >= (int64_t)1 << 23) return DVDQ_ERR_UNSUPPORTED;
    if (!aligned16(codes) || !aligned16(x_scale) || !aligned16(w) || !aligned16(w_scale) || !aligned16(y) ||
        (bias && !aligned16(bias)) || (acc_out && !aligned16(acc_out)) || (w_zero && !aligned16(w_zero)) ||
        (w_zero && !aligned16(code_rowsum)))
        return DVDQ_ERR_ALIGN;
    return DVDQ_OK;
}

}  // namespace

extern "C" {

int dvdq_rotate_quant(const void *x_bf16, int64_t M, int64_t K, int had_block, int act_bits, int codes_format,
                      int8_t *codes, float *x_scale, int32_t *code_rowsum, void *hip_stream) {
    int log2b = 0;
    const int rc = check_rotate_quant(x_bf16, M, K, had_block, act_bits, codes_format, codes, x_scale, code_rowsum,
                                      &log2b);
    if (rc != DVDQ_OK) return rc;
    return dvdq::launch_rotate_quant(static_cast<const uint16_t *>(x_bf16), M, K, log2b, act_bits, codes_format, 0,
                                     codes, x_scale, code_rowsum, static_cast<hipStream_t>(hip_stream));
}

int dvdq_rotate_quant_blockwise(const void *x_bf16, int64_t M, int64_t K, int had_block, int act_bits, int group,
                                int8_t *values, float *x_scale, int32_t *value_rowsum, void *hip_stream) {
    int log2b = 0;
    const int rc = check_rotate_quant(x_bf16, M, K, had_block, act_bits, DVDQ_CODES_INT8, values, x_scale,
                                      value_rowsum, &log2b);
    if (rc != DVDQ_OK) return rc;
    if (group < 1 || (K % group) != 0) return DVDQ_ERR_SHAPE;
    if (group != 128 && group != 256 && group != 512) return DVDQ_ERR_UNSUPPORTED;
    if (act_bits == 8) return DVDQ_ERR_UNSUPPORTED;   // 8-bit codes leave no room in the int8 container
    return dvdq::launch_rotate_quant(static_cast<const uint16_t *>(x_bf16), M, K, log2b, act_bits, DVDQ_CODES_INT8,
                                     log2_exact(group), values, x_scale, value_rowsum,
                                     static_cast<hipStream_t>(hip_stream));
}

int dvdq_w4ax_gemm(const int8_t *codes, const float *x_scale, const uint8_t *w, const float *w_scale,
                   const int8_t *w_zero, const int32_t *code_rowsum, const void *bias_bf16, int64_t M, int64_t N,
                   int64_t K, int act_bits, int codes_format, int w_layout, void *y_bf16, int32_t *acc_out,
                   void *hip_stream) {
    const int rc = check_gemm(codes, x_scale, w, w_scale, w_zero, code_rowsum, bias_bf16, M, N, K, act_bits,
                              codes_format, w_layout, y_bf16, acc_out);
    if (rc != DVDQ_OK) return rc;
    if (w_layout == DVDQ_W_NATIVE_FP6)
        return dvdq::launch_w4a4_fp6_gemm(reinterpret_cast<const uint8_t *>(codes), x_scale, w, w_scale, w_zero,
                                          code_rowsum, static_cast<const uint16_t *>(bias_bf16), M, N, K,
                                          static_cast<uint16_t *>(y_bf16), acc_out, static_cast<hipStream_t>(hip_stream));
    return dvdq::launch_w4ax_gemm(codes, x_scale, w, w_scale, w_zero, code_rowsum,
                                  static_cast<const uint16_t *>(bias_bf16), M, N, K, codes_format, w_layout,
                                  static_cast<uint16_t *>(y_bf16), acc_out, static_cast<hipStream_t>(hip_stream));
}

size_t dvdq_codes_bytes(int64_t M, int64_t K, int codes_format) {
    if (M < 1 || K < 1) return 0;
    if (codes_format == DVDQ_CODES_INT8) return (size_t)M * (size_t)K;
    if (codes_format == DVDQ_CODES_PACKED4) return (K % 2) ? 0 : (size_t)M * (size_t)K / 2;
    if (codes_format == DVDQ_CODES_FP6) return (K % 128) ? 0 : dvdq::codes_fp6_bytes(M, K);
    return 0;
}

size_t dvdq_qlinear_scale_offset(int64_t M, int64_t K, int codes_format) {
    if (M < 1 || K < 1) return 0;
    if (codes_format == DVDQ_CODES_FP6) return round_up(dvdq::codes_fp6_bytes(M, K), 256);
    const size_t code_bytes = (size_t)M * (size_t)K;
    return round_up(codes_format == DVDQ_CODES_PACKED4 ? code_bytes / 2 : code_bytes, 256);
}

size_t dvdq_qlinear_rowsum_offset(int64_t M, int64_t K, int codes_format) {
    if (M < 1 || K < 1) return 0;
    return dvdq_qlinear_scale_offset(M, K, codes_format) + round_up(sizeof(float) * (size_t)M, 256);
}

size_t dvdq_qlinear_workspace_bytes(int64_t M, int64_t K, int codes_format) {
    if (M < 1 || K < 1) return 0;
    return dvdq_qlinear_rowsum_offset(M, K, codes_format) + round_up(sizeof(int32_t) * (size_t)M, 256);
}

int dvdq_qlinear(const void *x_bf16, const uint8_t *w, const float *w_scale, const int8_t *w_zero,
                 const void *bias_bf16, int64_t M, int64_t N, int64_t K, int had_block, int act_bits,
                 int codes_format, int w_layout, void *y_bf16, void *workspace, size_t workspace_bytes,
                 void *hip_stream) {
    if (!workspace) return DVDQ_ERR_NULL;
    if (M < 1 || K < 1) return DVDQ_ERR_SHAPE;
    if ((reinterpret_cast<uintptr_t>(workspace) & 255u) != 0) return DVDQ_ERR_ALIGN;
    int8_t *codes = static_cast<int8_t *>(workspace);
    float *x_scale = reinterpret_cast<float *>(static_cast<uint8_t *>(workspace) +
                                               dvdq_qlinear_scale_offset(M, K, codes_format));
    int32_t *rowsum = !w_zero ? nullptr
                              : reinterpret_cast<int32_t *>(static_cast<uint8_t *>(workspace) +
                                                            dvdq_qlinear_rowsum_offset(M, K, codes_format));
    int log2b = 0;
    int rc = check_rotate_quant(x_bf16, M, K, had_block, act_bits, codes_format, codes, x_scale, rowsum, &log2b);
    if (rc != DVDQ_OK) return rc;
    rc = check_gemm(codes, x_scale, w, w_scale, w_zero, rowsum, bias_bf16, M, N, K, act_bits, codes_format, w_layout,
                    y_bf16, nullptr);
    if (rc != DVDQ_OK) return rc;
    if (workspace_bytes < dvdq_qlinear_workspace_bytes(M, K, codes_format)) return DVDQ_ERR_WORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    rc = dvdq::launch_rotate_quant(static_cast<const uint16_t *>(x_bf16), M, K, log2b, act_bits, codes_format, 0,
                                   codes, x_scale, rowsum, stream);
    if (rc != DVDQ_OK) return rc;
    if (w_layout == DVDQ_W_NATIVE_FP6)
        return dvdq::launch_w4a4_fp6_gemm(reinterpret_cast<const uint8_t *>(codes), x_scale, w, w_scale, w_zero, rowsum,
                                          static_cast<const uint16_t *>(bias_bf16), M, N, K,
                                          static_cast<uint16_t *>(y_bf16), nullptr, stream);
    return dvdq::launch_w4ax_gemm(codes, x_scale, w, w_scale, w_zero, rowsum,
                                  static_cast<const uint16_t *>(bias_bf16), M, N, K, codes_format, w_layout,
                                  static_cast<uint16_t *>(y_bf16), nullptr, stream);
}

size_t dvdq_static_workspace_bytes(void) { return DVDQ_STATIC_WORKSPACE_BYTES; }

int dvdq_release_stream(void *hip_stream) {
    dvdq::release_sched_slot(static_cast<hipStream_t>(hip_stream));
    return DVDQ_OK;
}

int dvdq_qlinear_static(const void *x_bf16, const uint8_t *w, const float *w_scale, const int8_t *w_zero,
                        const void *bias_bf16, int64_t M, int64_t N, int64_t K, int had_block, int act_bits,
                        int codes_format, int w_layout, void *y_bf16, void *hip_stream) {
    if (M < 1 || K < 1) return DVDQ_ERR_SHAPE;
    if (check_format(codes_format, act_bits) != DVDQ_OK) return DVDQ_ERR_UNSUPPORTED;
    if (codes_format == DVDQ_CODES_FP6 && (K % 128) != 0) return DVDQ_ERR_UNSUPPORTED;
    if (K > 65536 || M > 0x7FFFFFFF) return DVDQ_ERR_UNSUPPORTED;   // (keeps the size below from overflowing)
    const size_t need = dvdq_qlinear_workspace_bytes(M, K, codes_format);
    if (need == 0 || need > (size_t)DVDQ_STATIC_WORKSPACE_BYTES) return DVDQ_ERR_WORKSPACE;
    uint8_t *ws = scratch_ptr();
    if (!ws) return DVDQ_ERR_HIP;
    return dvdq_qlinear(x_bf16, w, w_scale, w_zero, bias_bf16, M, N, K, had_block, act_bits, codes_format, w_layout,
                        y_bf16, ws, (size_t)DVDQ_STATIC_WORKSPACE_BYTES, hip_stream);
}

size_t dvdq_w4_native_bytes(int64_t N, int64_t K) {
    if (N < 1 || K < 1 || (K % 128) != 0) return 0;
    return dvdq::w4_native_bytes(N, K);
}

int dvdq_w4_prepack(const uint8_t *w_canonical, int64_t N, int64_t K, uint8_t *w_native, void *hip_stream) {
    if (!w_canonical || !w_native) return DVDQ_ERR_NULL;
    if (N < 1 || K < 1 || (K % 2) != 0) return DVDQ_ERR_SHAPE;
    if ((K % 128) != 0) return DVDQ_ERR_UNSUPPORTED;
    if (N > 0x7FFFFFFF || K > 0x7FFFFFFF) return DVDQ_ERR_UNSUPPORTED;
    if (!aligned16(w_canonical) || !aligned16(w_native)) return DVDQ_ERR_ALIGN;
    return dvdq::launch_w4_prepack(w_canonical, N, K, w_native, static_cast<hipStream_t>(hip_stream));
}

size_t dvdq_w4_native_fp6_bytes(int64_t N, int64_t K) {
    if (N < 1 || K < 1 || (K % 128) != 0) return 0;
    return dvdq::w4_native_fp6_bytes(N, K);
}

int dvdq_w4_prepack_fp6(const uint8_t *w_canonical, int64_t N, int64_t K, uint8_t *w_native, void *hip_stream) {
    if (!w_canonical || !w_native) return DVDQ_ERR_NULL;
    if (N < 1 || K < 1 || (K % 2) != 0) return DVDQ_ERR_SHAPE;
    if ((K % 128) != 0) return DVDQ_ERR_UNSUPPORTED;
    if (N > 0x7FFFFFFF || K > 0x7FFFFFFF) return DVDQ_ERR_UNSUPPORTED;
    if (!aligned16(w_canonical) || !aligned16(w_native)) return DVDQ_ERR_ALIGN;
    return dvdq::launch_w4_prepack_fp6(w_canonical, N, K, w_native, static_cast<hipStream_t>(hip_stream));
}

int dvdq_bgr_quantize(const float *w, int64_t N, int64_t K, int n_steps, int max_refine, double eps, int search,
                      uint8_t *w_packed, float *w_scale, int8_t *w_zero, double *row_error, void *hip_stream) {
    if (!w || !w_packed || !w_scale || !w_zero) return DVDQ_ERR_NULL;
    if (N < 1 || K < 2 || (K % 2) != 0 || n_steps < 1 || max_refine < 0 || !(eps >= 0.0)) return DVDQ_ERR_SHAPE;
    if (search != DVDQ_BGR_LISTING && search != DVDQ_BGR_BEST_OF_ALL) return DVDQ_ERR_UNSUPPORTED;
    if (search == DVDQ_BGR_LISTING && n_steps < 3) return DVDQ_ERR_SHAPE;   // i = 1 must leave a non-empty range
    if (K > 32768 || N > 0x7FFFFFFF) return DVDQ_ERR_UNSUPPORTED;   // the row is kept in LDS
    if (!aligned16(w) || !aligned16(w_packed) || !aligned16(w_scale) || !aligned16(w_zero) ||
        (row_error && !aligned16(row_error)))
        return DVDQ_ERR_ALIGN;
    return dvdq::launch_bgr(w, N, K, n_steps, max_refine, eps, search, w_packed, w_scale, w_zero, row_error,
                            static_cast<hipStream_t>(hip_stream));
}

size_t dvdq_gbs_workspace_bytes(void) { return dvdq::gbs_workspace_bytes(); }

int dvdq_gbs_reset(void *state, int initial_bits, void *hip_stream) {
    if (!state) return DVDQ_ERR_NULL;
    if (!bits_ok(initial_bits)) return DVDQ_ERR_UNSUPPORTED;
    if (!aligned16(state)) return DVDQ_ERR_ALIGN;
    return dvdq::launch_gbs_reset(state, initial_bits, static_cast<hipStream_t>(hip_stream));
}

int dvdq_gbs_step(const void *f_t_bf16, const void *f_prev_bf16, int64_t n, float delta, int b_low, int b_high,
                  void *state, void *workspace, size_t workspace_bytes, void *hip_stream) {
    if (!f_t_bf16 || !f_prev_bf16 || !state || !workspace) return DVDQ_ERR_NULL;
    if (n < 1 || !(delta >= 0.f)) return DVDQ_ERR_SHAPE;
    if (!bits_ok(b_low) || !bits_ok(b_high) || b_low > b_high) return DVDQ_ERR_UNSUPPORTED;
    if (workspace_bytes < dvdq::gbs_workspace_bytes()) return DVDQ_ERR_WORKSPACE;
    if (!aligned16(f_t_bf16) || !aligned16(f_prev_bf16) || !aligned16(state) || !aligned16(workspace))
        return DVDQ_ERR_ALIGN;
    return dvdq::launch_gbs_step(static_cast<const uint16_t *>(f_t_bf16), static_cast<const uint16_t *>(f_prev_bf16), n,
                                 (double)delta, b_low, b_high, state, workspace, static_cast<hipStream_t>(hip_stream));
}

const char *dvdq_status_string(int status) {
    switch (status) {
        case DVDQ_OK: return "ok";
        case DVDQ_ERR_NULL: return "a required pointer is NULL";
        case DVDQ_ERR_SHAPE: return "inconsistent shape arguments";
        case DVDQ_ERR_UNSUPPORTED: return "request outside what the kernels implement";
        case DVDQ_ERR_WORKSPACE: return "workspace too small";
        case DVDQ_ERR_ALIGN: return "pointer not sufficiently aligned";
        case DVDQ_ERR_HIP: return "kernel launch failed";
        default: return "unknown status";
    }
}

int dvdq_version(void) { return 230; }

}  // extern "C"

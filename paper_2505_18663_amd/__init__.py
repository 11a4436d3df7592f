"""Python binding of libdvdq (ctypes).  Argument marshalling only: every step of
the quantized linear layer runs in the HIP kernels behind the C ABI declared in
``include/dvdq.h``.  PyTorch supplies device memory and streams, nothing else.

There is no CPU fallback: if ``libdvdq.so`` has not been built
(``python -m paper_2505_18663_amd.build``) importing a function works but the first
call raises ``DvdqLibraryMissing``.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

__all__ = [
    "DvdqError", "DvdqLibraryMissing", "lib", "library_path", "version", "status_string",
    "rotate_quant", "rotate_quant_blockwise", "w4ax_gemm", "qlinear", "qlinear_static", "static_workspace_bytes", "qlinear_workspace_bytes", "qlinear_scale_offset", "qlinear_rowsum_offset", "workspace_rowsum",
    "w4_prepack", "w4_native_bytes", "w4_prepack_fp6", "w4_native_fp6_bytes", "codes_bytes", "bgr_quantize", "GbsController", "bench_copy", "bench_mfma_i8", "bench_mfma_fp6", "bench_set_gemm_variant", "bench_set_gemm_schedule", "bench_fill_tile_counters", "bench_set_gemm_grid_limit", "release_stream",
    "W_CANONICAL", "W_NATIVE", "W_NATIVE_FP6", "CODES_INT8", "CODES_PACKED4", "CODES_FP6", "BGR_LISTING", "BGR_BEST_OF_ALL", "EXPORTED_SYMBOLS",
]

W_CANONICAL, W_NATIVE, W_NATIVE_FP6 = 0, 1, 2
CODES_INT8, CODES_PACKED4, CODES_FP6 = 0, 1, 2
BGR_LISTING, BGR_BEST_OF_ALL = 0, 1

EXPORTED_SYMBOLS = (
    "dvdq_rotate_quant", "dvdq_rotate_quant_blockwise", "dvdq_w4ax_gemm", "dvdq_qlinear", "dvdq_qlinear_workspace_bytes",
    "dvdq_qlinear_scale_offset", "dvdq_qlinear_rowsum_offset", "dvdq_qlinear_static", "dvdq_static_workspace_bytes", "dvdq_w4_prepack", "dvdq_w4_native_bytes", "dvdq_w4_prepack_fp6",
    "dvdq_w4_native_fp6_bytes", "dvdq_codes_bytes", "dvdq_status_string",
    "dvdq_version", "dvdq_gbs_workspace_bytes", "dvdq_gbs_reset", "dvdq_gbs_step", "dvdq_bgr_quantize", "dvdq_bench_copy", "dvdq_bench_mfma_i8", "dvdq_bench_mfma_fp6", "dvdq_bench_set_gemm_variant", "dvdq_bench_set_gemm_schedule", "dvdq_bench_fill_tile_counters", "dvdq_bench_set_gemm_grid_limit", "dvdq_release_stream",
)

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libdvdq.so")
_lib = None


class DvdqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: dvdq status {status} ({status_string(status)})")


class DvdqLibraryMissing(RuntimeError):
    pass


def library_path() -> str:
    return _LIB_PATH


def lib() -> C.CDLL:
    """Load libdvdq.so (once) and declare the C prototypes."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise DvdqLibraryMissing(
            f"{_LIB_PATH} not found: build it with `python -m paper_2505_18663_amd.build` "
            "(hipcc, gfx950).  There is no fallback path.")
    L = C.CDLL(_LIB_PATH)
    i64, i32, vp, sz = C.c_int64, C.c_int, C.c_void_p, C.c_size_t
    L.dvdq_rotate_quant.argtypes = [vp, i64, i64, i32, i32, i32, vp, vp, vp, vp]
    L.dvdq_rotate_quant_blockwise.argtypes = [vp, i64, i64, i32, i32, i32, vp, vp, vp, vp]
    L.dvdq_rotate_quant_blockwise.restype = i32
    L.dvdq_w4ax_gemm.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, i32, i32, i32, vp, vp, vp]
    L.dvdq_qlinear.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i32, i32, i32, i32, vp, vp, sz, vp]
    L.dvdq_qlinear_static.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i32, i32, i32, i32, vp, vp]
    L.dvdq_qlinear_static.restype = i32
    L.dvdq_static_workspace_bytes.argtypes = []
    L.dvdq_static_workspace_bytes.restype = sz
    L.dvdq_qlinear_rowsum_offset.argtypes = [i64, i64, i32]
    L.dvdq_qlinear_workspace_bytes.argtypes = [i64, i64, i32]
    L.dvdq_qlinear_scale_offset.argtypes = [i64, i64, i32]
    L.dvdq_w4_prepack.argtypes = [vp, i64, i64, vp, vp]
    L.dvdq_w4_native_bytes.argtypes = [i64, i64]
    L.dvdq_w4_prepack_fp6.argtypes = [vp, i64, i64, vp, vp]
    L.dvdq_w4_prepack_fp6.restype = i32
    L.dvdq_w4_native_fp6_bytes.argtypes = [i64, i64]
    L.dvdq_w4_native_fp6_bytes.restype = sz
    L.dvdq_codes_bytes.argtypes = [i64, i64, i32]
    L.dvdq_codes_bytes.restype = sz
    L.dvdq_status_string.argtypes = [i32]
    L.dvdq_version.argtypes = []
    L.dvdq_gbs_workspace_bytes.argtypes = []
    L.dvdq_gbs_workspace_bytes.restype = sz
    L.dvdq_gbs_reset.argtypes = [vp, i32, vp]
    L.dvdq_gbs_reset.restype = i32
    L.dvdq_gbs_step.argtypes = [vp, vp, i64, C.c_float, i32, i32, vp, vp, sz, vp]
    L.dvdq_gbs_step.restype = i32
    L.dvdq_bgr_quantize.argtypes = [vp, i64, i64, i32, i32, C.c_double, i32, vp, vp, vp, vp, vp]
    L.dvdq_bgr_quantize.restype = i32
    L.dvdq_bench_copy.argtypes = [vp, vp, sz, vp]
    L.dvdq_bench_mfma_i8.argtypes = [i32, i32, vp, C.POINTER(C.c_double), vp]
    L.dvdq_bench_mfma_fp6.argtypes = [i32, i32, vp, C.POINTER(C.c_double), vp]
    L.dvdq_bench_mfma_fp6.restype = i32
    L.dvdq_bench_set_gemm_variant.argtypes = [i32]
    L.dvdq_bench_set_gemm_variant.restype = i32
    L.dvdq_bench_set_gemm_schedule.argtypes = [i32]
    L.dvdq_bench_set_gemm_schedule.restype = i32
    L.dvdq_bench_fill_tile_counters.argtypes = [C.c_uint32, C.c_void_p]
    L.dvdq_bench_fill_tile_counters.restype = i32
    L.dvdq_bench_set_gemm_grid_limit.argtypes = [i32]
    L.dvdq_bench_set_gemm_grid_limit.restype = i32
    L.dvdq_release_stream.argtypes = [C.c_void_p]
    L.dvdq_release_stream.restype = i32
    for f in ("dvdq_rotate_quant", "dvdq_rotate_quant_blockwise", "dvdq_w4ax_gemm", "dvdq_qlinear", "dvdq_w4_prepack", "dvdq_version",
              "dvdq_bench_copy", "dvdq_bench_mfma_i8"):
        getattr(L, f).restype = i32
    for f in ("dvdq_qlinear_workspace_bytes", "dvdq_qlinear_scale_offset", "dvdq_qlinear_rowsum_offset",
              "dvdq_w4_native_bytes"):
        getattr(L, f).restype = sz
    L.dvdq_status_string.restype = C.c_char_p
    _lib = L
    return L


def version() -> int:
    return lib().dvdq_version()


def status_string(status: int) -> str:
    return lib().dvdq_status_string(int(status)).decode()


# ------------------------------------------------------------------ marshalling helpers
def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _need(t, dtype, shape, name):
    if not isinstance(t, torch.Tensor) or not t.is_cuda:
        raise TypeError(f"{name}: expected a CUDA/HIP tensor")
    if t.dtype != dtype:
        raise TypeError(f"{name}: expected dtype {dtype}, got {t.dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name}: must be contiguous")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name}: expected shape {tuple(shape)}, got {tuple(t.shape)}")
    return t


def _check(rc, where):
    if rc != 0:
        raise DvdqError(rc, where)


# ------------------------------------------------------------------ the layer
def _codes_spec(M: int, K: int, codes_format: int):
    """(dtype, shape) of the tensor that carries the activation codes."""
    if codes_format == CODES_PACKED4:
        return torch.uint8, (M, K // 2)
    if codes_format == CODES_FP6:   # opaque block layout, see include/dvdq.h
        return torch.uint8, (lib().dvdq_codes_bytes(M, K, CODES_FP6),)
    return torch.int8, (M, K)


def codes_bytes(M: int, K: int, codes_format: int) -> int:
    return lib().dvdq_codes_bytes(M, K, codes_format)


def rotate_quant(x, had_block: int, act_bits: int, codes=None, x_scale=None, stream=None,
                 codes_format: int = CODES_INT8, code_rowsum=None, want_rowsum: bool = False):
    """x: bf16 [M, K] -> (codes int8 [M, K] or packed uint8 [M, K/2], x_scale fp32 [M]); with
    want_rowsum (or code_rowsum given) also the per-token code sums int32 [M].  See dvdq_rotate_quant."""
    L = lib()
    _need(x, torch.bfloat16, None, "x")
    M, K = x.shape
    cdtype, cshape = _codes_spec(M, K, codes_format)
    if codes is None:
        codes = torch.empty(cshape, dtype=cdtype, device=x.device)
    if x_scale is None:
        x_scale = torch.empty((M,), dtype=torch.float32, device=x.device)
    _need(codes, cdtype, cshape, "codes")
    _need(x_scale, torch.float32, (M,), "x_scale")
    if want_rowsum and code_rowsum is None:
        code_rowsum = torch.empty((M,), dtype=torch.int32, device=x.device)
    if code_rowsum is not None:
        _need(code_rowsum, torch.int32, (M,), "code_rowsum")
    _check(L.dvdq_rotate_quant(_ptr(x), M, K, had_block, act_bits, codes_format, _ptr(codes), _ptr(x_scale),
                               _ptr(code_rowsum), _stream(stream)), "dvdq_rotate_quant")
    return (codes, x_scale) if code_rowsum is None else (codes, x_scale, code_rowsum)


def rotate_quant_blockwise(x, had_block: int, act_bits: int, group: int, values=None, x_scale=None,
                           want_rowsum: bool = False, stream=None):
    """Block-wise scaled quantizer: x bf16 [M, K] -> (values int8 [M, K], x_scale fp32 [M][, rowsum int32 [M]]).
    Feed the result to w4ax_gemm with act_bits=8.  See dvdq_rotate_quant_blockwise."""
    L = lib()
    _need(x, torch.bfloat16, None, "x")
    M, K = x.shape
    if values is None:
        values = torch.empty((M, K), dtype=torch.int8, device=x.device)
    if x_scale is None:
        x_scale = torch.empty((M,), dtype=torch.float32, device=x.device)
    _need(values, torch.int8, (M, K), "values")
    _need(x_scale, torch.float32, (M,), "x_scale")
    rs = torch.empty((M,), dtype=torch.int32, device=x.device) if want_rowsum else None
    _check(L.dvdq_rotate_quant_blockwise(_ptr(x), M, K, had_block, act_bits, group, _ptr(values), _ptr(x_scale),
                                         _ptr(rs), _stream(stream)), "dvdq_rotate_quant_blockwise")
    return (values, x_scale, rs) if want_rowsum else (values, x_scale)


def _check_weight_buffer(L, w, w_layout: int, N: int, K: int):
    """The C ABI cannot know how large the weight buffer is; the kernels read dvdq_w4_native*_bytes(N, K)
    bytes of a native buffer (N padded to 256 rows), so an undersized one must be refused here."""
    if w_layout == W_CANONICAL:
        if tuple(w.shape) != (N, K // 2):
            raise ValueError(f"w: expected shape {(N, K // 2)}, got {tuple(w.shape)}")
        return
    if w_layout not in (W_NATIVE, W_NATIVE_FP6):
        return   # the library reports the unknown layout
    need = L.dvdq_w4_native_bytes(N, K) if w_layout == W_NATIVE else L.dvdq_w4_native_fp6_bytes(N, K)
    if need == 0:
        raise ValueError(f"w: no native layout for N={N}, K={K} (K must be a multiple of 128)")
    if w.numel() < need:
        raise ValueError(f"w: native buffer holds {w.numel()} bytes, the layout needs {need}")


def w4ax_gemm(codes, x_scale, w, w_scale, act_bits: int, w_layout: int = W_CANONICAL, bias=None,
              y=None, acc_out=None, want_acc: bool = False, stream=None, codes_format: int = CODES_INT8,
              w_zero=None, code_rowsum=None, K=None):
    """codes int8 [M, K] (or packed uint8 [M, K/2], or the opaque FP6 buffer: then pass K), w uint8 packed
    INT4 [N, K/2] (or native) -> y bf16 [M, N].  With want_acc (or acc_out given) also returns the int32
    accumulators."""
    L = lib()
    if codes_format == CODES_FP6:
        _need(codes, torch.uint8, None, "codes")
        if K is None:
            raise ValueError("K is required with FP6 codes")
        M = x_scale.shape[0]
        if codes.numel() < L.dvdq_codes_bytes(M, K, CODES_FP6):
            raise ValueError("codes: FP6 buffer too small")
    elif codes_format == CODES_PACKED4:
        _need(codes, torch.uint8, None, "codes")
        M, K = codes.shape[0], 2 * codes.shape[1]
    else:
        _need(codes, torch.int8, None, "codes")
        M, K = codes.shape
    _need(w_scale, torch.float32, None, "w_scale")
    N = w_scale.shape[0]
    _need(x_scale, torch.float32, (M,), "x_scale")
    _need(w, torch.uint8, None, "w")
    _check_weight_buffer(L, w, w_layout, N, K)
    if bias is not None:
        _need(bias, torch.bfloat16, (N,), "bias")
    if w_zero is not None:
        _need(w_zero, torch.int8, (N,), "w_zero")
        _need(code_rowsum, torch.int32, (M,), "code_rowsum")
    if y is None:
        y = torch.empty((M, N), dtype=torch.bfloat16, device=codes.device)
    _need(y, torch.bfloat16, (M, N), "y")
    if want_acc and acc_out is None:
        acc_out = torch.empty((M, N), dtype=torch.int32, device=codes.device)
    if acc_out is not None:
        _need(acc_out, torch.int32, (M, N), "acc_out")
    _check(L.dvdq_w4ax_gemm(_ptr(codes), _ptr(x_scale), _ptr(w), _ptr(w_scale), _ptr(w_zero), _ptr(code_rowsum),
                            _ptr(bias), M, N, K, act_bits, codes_format, w_layout, _ptr(y), _ptr(acc_out),
                            _stream(stream)), "dvdq_w4ax_gemm")
    return (y, acc_out) if acc_out is not None else y


def qlinear_workspace_bytes(M: int, K: int, codes_format: int = CODES_INT8) -> int:
    return lib().dvdq_qlinear_workspace_bytes(M, K, codes_format)


def qlinear_scale_offset(M: int, K: int, codes_format: int = CODES_INT8) -> int:
    return lib().dvdq_qlinear_scale_offset(M, K, codes_format)


def qlinear_rowsum_offset(M: int, K: int, codes_format: int = CODES_INT8) -> int:
    return lib().dvdq_qlinear_rowsum_offset(M, K, codes_format)


def qlinear(x, w, w_scale, had_block: int, act_bits: int, w_layout: int = W_CANONICAL, bias=None,
            y=None, workspace=None, stream=None, codes_format: int = CODES_INT8, w_zero=None):
    """The whole layer.  Returns (y bf16 [M, N], workspace uint8); the workspace holds the
    codes at offset 0 and the token scales at qlinear_scale_offset(M, K, codes_format)."""
    L = lib()
    _need(x, torch.bfloat16, None, "x")
    M, K = x.shape
    _need(w_scale, torch.float32, None, "w_scale")
    N = w_scale.shape[0]
    _need(w, torch.uint8, None, "w")
    _check_weight_buffer(L, w, w_layout, N, K)
    if bias is not None:
        _need(bias, torch.bfloat16, (N,), "bias")
    if w_zero is not None:
        _need(w_zero, torch.int8, (N,), "w_zero")
    if y is None:
        y = torch.empty((M, N), dtype=torch.bfloat16, device=x.device)
    _need(y, torch.bfloat16, (M, N), "y")
    need = L.dvdq_qlinear_workspace_bytes(M, K, codes_format)
    if workspace is None:
        workspace = torch.empty((need,), dtype=torch.uint8, device=x.device)
    _need(workspace, torch.uint8, None, "workspace")
    _check(L.dvdq_qlinear(_ptr(x), _ptr(w), _ptr(w_scale), _ptr(w_zero), _ptr(bias), M, N, K, had_block, act_bits,
                          codes_format, w_layout, _ptr(y), _ptr(workspace), workspace.numel(), _stream(stream)),
           "dvdq_qlinear")
    return y, workspace


def static_workspace_bytes() -> int:
    return lib().dvdq_static_workspace_bytes()


def qlinear_static(x, w, w_scale, had_block: int, act_bits: int, w_layout: int = W_CANONICAL, bias=None, y=None,
                   stream=None, codes_format: int = CODES_INT8, w_zero=None):
    """The whole layer with the library's own fixed workspace (no allocation inside the call; `y` must be
    given if the caller may not allocate either).  Returns y bf16 [M, N]."""
    L = lib()
    _need(x, torch.bfloat16, None, "x")
    M, K = x.shape
    _need(w_scale, torch.float32, None, "w_scale")
    N = w_scale.shape[0]
    _need(w, torch.uint8, None, "w")
    _check_weight_buffer(L, w, w_layout, N, K)
    if bias is not None:
        _need(bias, torch.bfloat16, (N,), "bias")
    if w_zero is not None:
        _need(w_zero, torch.int8, (N,), "w_zero")
    if y is None:
        y = torch.empty((M, N), dtype=torch.bfloat16, device=x.device)
    _need(y, torch.bfloat16, (M, N), "y")
    _check(L.dvdq_qlinear_static(_ptr(x), _ptr(w), _ptr(w_scale), _ptr(w_zero), _ptr(bias), M, N, K, had_block,
                                 act_bits, codes_format, w_layout, _ptr(y), _stream(stream)), "dvdq_qlinear_static")
    return y


def workspace_views(workspace, M: int, K: int, codes_format: int = CODES_INT8):
    """(codes int8 [M, K] or packed uint8 [M, K/2], x_scale fp32 [M]) views into a qlinear workspace."""
    off = qlinear_scale_offset(M, K, codes_format)
    cdtype, cshape = _codes_spec(M, K, codes_format)
    n_el = 1
    for d in cshape:
        n_el *= d
    codes = workspace[:n_el].view(cdtype).view(cshape)
    scale = workspace[off:off + 4 * M].view(torch.float32)
    return codes, scale


def workspace_rowsum(workspace, M: int, K: int, codes_format: int = CODES_INT8):
    """int32 [M] view of the token code sums in a qlinear workspace (written when w_zero is given)."""
    off = qlinear_rowsum_offset(M, K, codes_format)
    return workspace[off:off + 4 * M].view(torch.int32)


def w4_native_bytes(N: int, K: int) -> int:
    return lib().dvdq_w4_native_bytes(N, K)


def w4_prepack(w_canonical, w_native=None, stream=None):
    """uint8 [N, K/2] canonical -> opaque native buffer for the GEMM kernel (offline, once)."""
    L = lib()
    _need(w_canonical, torch.uint8, None, "w_canonical")
    N, K2 = w_canonical.shape
    K = 2 * K2
    need = L.dvdq_w4_native_bytes(N, K)
    if w_native is None:
        w_native = torch.empty((max(need, 1),), dtype=torch.uint8, device=w_canonical.device)
    _need(w_native, torch.uint8, None, "w_native")
    if w_native.numel() < need:
        raise ValueError("w_native too small")
    _check(L.dvdq_w4_prepack(_ptr(w_canonical), N, K, _ptr(w_native), _stream(stream)), "dvdq_w4_prepack")
    return w_native


def w4_native_fp6_bytes(N: int, K: int) -> int:
    return lib().dvdq_w4_native_fp6_bytes(N, K)


def w4_prepack_fp6(w_canonical, w_native=None, stream=None):
    """uint8 [N, K/2] canonical -> opaque FP6 native buffer for the W4A4 GEMM on the FP6 matrix path."""
    L = lib()
    _need(w_canonical, torch.uint8, None, "w_canonical")
    N, K2 = w_canonical.shape
    K = 2 * K2
    need = L.dvdq_w4_native_fp6_bytes(N, K)
    if w_native is None:
        w_native = torch.empty((max(need, 1),), dtype=torch.uint8, device=w_canonical.device)
    _need(w_native, torch.uint8, None, "w_native")
    if w_native.numel() < need:
        raise ValueError("w_native too small")
    _check(L.dvdq_w4_prepack_fp6(_ptr(w_canonical), N, K, _ptr(w_native), _stream(stream)), "dvdq_w4_prepack_fp6")
    return w_native


def bgr_quantize(w, n_steps: int = 100, max_refine: int = 10, eps: float = 0.0, want_error: bool = False, stream=None,
                 search: int = BGR_LISTING):
    """Offline INT4 weight quantizer (Bounded-init Grid Refinement).  w: fp32 [N, K] ->
    (w_packed uint8 [N, K/2] canonical, w_scale fp32 [N], w_zero int8 [N][, row_error fp64 [N]]).
    search: BGR_LISTING (Alg. 1 as printed) or BGR_BEST_OF_ALL (superset search, never worse than MinMax)."""
    L = lib()
    _need(w, torch.float32, None, "w")
    N, K = w.shape
    w_packed = torch.empty((N, K // 2), dtype=torch.uint8, device=w.device)
    w_scale = torch.empty((N,), dtype=torch.float32, device=w.device)
    w_zero = torch.empty((N,), dtype=torch.int8, device=w.device)
    err = torch.empty((N,), dtype=torch.float64, device=w.device) if want_error else None
    _check(L.dvdq_bgr_quantize(_ptr(w), N, K, n_steps, max_refine, float(eps), int(search), _ptr(w_packed), _ptr(w_scale),
                               _ptr(w_zero), _ptr(err), _stream(stream)), "dvdq_bgr_quantize")
    return (w_packed, w_scale, w_zero, err) if want_error else (w_packed, w_scale, w_zero)


# ------------------------------------------------------------------ delta-GBS controller
class GbsController:
    """Device-side state of delta-Guided Bit Switching plus the two C calls.  `step` enqueues the
    update; `bits()` reads the one scalar back (synchronizes)."""

    def __init__(self, delta: float, b_low: int = 4, b_high: int = 8, device="cuda:0", stream=None):
        self.delta, self.b_low, self.b_high = float(delta), int(b_low), int(b_high)
        self.state = torch.zeros((16,), dtype=torch.uint8, device=device)
        self.workspace = torch.empty((lib().dvdq_gbs_workspace_bytes(),), dtype=torch.uint8, device=device)
        self.reset(stream=stream)

    def reset(self, stream=None):
        _check(lib().dvdq_gbs_reset(_ptr(self.state), self.b_high, _stream(stream)), "dvdq_gbs_reset")

    def step(self, f_t, f_prev, stream=None):
        _need(f_t, torch.bfloat16, None, "f_t")
        _need(f_prev, torch.bfloat16, tuple(f_t.shape), "f_prev")
        _check(lib().dvdq_gbs_step(_ptr(f_t), _ptr(f_prev), f_t.numel(), self.delta, self.b_low, self.b_high,
                                   _ptr(self.state), _ptr(self.workspace), self.workspace.numel(), _stream(stream)),
               "dvdq_gbs_step")

    def read(self):
        """(running sum, last relative L1, bits for the next step) -- synchronizes."""
        raw = self.state.cpu().numpy()
        return float(raw[:8].view("<f8")[0]), float(raw[8:12].view("<f4")[0]), int(raw[12:16].view("<i4")[0])

    def bits(self) -> int:
        return self.read()[2]


# ------------------------------------------------------------------ calibration helpers
def bench_copy(src, dst, stream=None):
    nbytes = src.numel() * src.element_size()
    _check(lib().dvdq_bench_copy(_ptr(src), _ptr(dst), nbytes, _stream(stream)), "dvdq_bench_copy")


def bench_mfma_i8(iters: int, sink, stream=None, data: int = 0) -> float:
    """data 0: constant operands (issue-limited rate); 1: random 4-bit codes (the rate under the layer's kind of data)"""
    ops = C.c_double(0.0)
    _check(lib().dvdq_bench_mfma_i8(iters, int(data), _ptr(sink), C.byref(ops), _stream(stream)), "dvdq_bench_mfma_i8")
    return ops.value


def bench_mfma_fp6(iters: int, sink, stream=None, data: int = 0) -> float:
    ops = C.c_double(0.0)
    _check(lib().dvdq_bench_mfma_fp6(iters, int(data), _ptr(sink), C.byref(ops), _stream(stream)), "dvdq_bench_mfma_fp6")
    return ops.value


def bench_set_gemm_variant(variant: int) -> None:
    _check(lib().dvdq_bench_set_gemm_variant(int(variant)), "dvdq_bench_set_gemm_variant")


def bench_set_gemm_schedule(schedule: int) -> None:
    """0: fixed tile shares; -1: the library's own choice (tiles drawn from counters)."""
    _check(lib().dvdq_bench_set_gemm_schedule(int(schedule)), "dvdq_bench_set_gemm_schedule")


def bench_set_gemm_grid_limit(workgroups: int) -> None:
    """At most `workgroups` workgroups per persistent GEMM launch (0: fill the chip).  Same results."""
    _check(lib().dvdq_bench_set_gemm_grid_limit(int(workgroups)), "dvdq_bench_set_gemm_grid_limit")


def bench_fill_tile_counters(value: int, stream=None) -> None:
    """Robustness tests: overwrite every tile-counter word of the current GPU with `value` (in stream order)."""
    _check(lib().dvdq_bench_fill_tile_counters(C.c_uint32(value & 0xFFFFFFFF), _stream(stream)), "dvdq_bench_fill_tile_counters")


def release_stream(stream) -> None:
    """Forget `stream` (a torch.cuda.Stream) before it is destroyed: its tile-counter slot can serve another stream."""
    _check(lib().dvdq_release_stream(C.c_void_p(stream.cuda_stream)), "dvdq_release_stream")

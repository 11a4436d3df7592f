"""numpy-facing loader for the CPU oracle (``dvdq_oracle.c``).

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this module;
only tests, the smoke check and the benchmark's CPU-baseline leg do.  The C file
is compiled with plain gcc (-O2, OpenMP over token rows, no fast-math, no FMA
contraction) into ``oracle/libdvdq_oracle.so`` the first time it is needed or
when the source is newer than the library.

Every wrapper below only marshals arrays; the arithmetic lives in the C file,
where each function cites the passage of the method it restates.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dvdq_oracle.c")
_LIB = os.path.join(_HERE, "libdvdq_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  Returns the library path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call([
            "gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
            "-fPIC", "-shared", "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm",
        ])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = C.CDLL(build())
        i64, i32, vp = C.c_int64, C.c_int, C.c_void_p
        lib.dvdq_oracle_hadamard.argtypes = [i32, vp]
        lib.dvdq_oracle_rotate.argtypes = [vp, i64, i64, i32, vp]
        lib.dvdq_oracle_quantize.argtypes = [vp, i64, i64, i32, vp, vp]
        lib.dvdq_oracle_quantize_blockwise.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp]
        lib.dvdq_oracle_quantize_blockwise.restype = i32
        lib.dvdq_oracle_rotate_quant.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp]
        lib.dvdq_oracle_unpack_w4.argtypes = [vp, i64, i64, vp]
        lib.dvdq_oracle_pack_w4.argtypes = [vp, i64, i64, vp]
        lib.dvdq_oracle_unpack_a4.argtypes = [vp, i64, i64, vp]
        lib.dvdq_oracle_pack_a4.argtypes = [vp, i64, i64, vp]
        lib.dvdq_oracle_unpack_fp6.argtypes = [vp, i64, i64, vp]
        lib.dvdq_oracle_pack_fp6.argtypes = [vp, i64, i64, vp]
        lib.dvdq_oracle_int_gemm.argtypes = [vp, vp, i64, i64, i64, vp]
        lib.dvdq_oracle_epilogue.argtypes = [vp, vp, vp, vp, i64, i64, vp]
        lib.dvdq_oracle_w4ax_gemm.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, vp, vp]
        lib.dvdq_oracle_qlinear.argtypes = [vp, vp, vp, vp, i64, i64, i64, i32, i32, vp, vp, vp, vp]
        lib.dvdq_oracle_f64_to_bf16.argtypes = [vp, i64, vp]
        lib.dvdq_oracle_rel_l1.argtypes = [vp, vp, i64]
        lib.dvdq_oracle_rel_l1.restype = C.c_double
        lib.dvdq_oracle_gbs_update.argtypes = [C.c_double, C.c_double, i32, i32, C.POINTER(C.c_double)]
        lib.dvdq_oracle_gbs_update.restype = i32
        lib.dvdq_oracle_bgr_refine_step.argtypes = [vp, i64, i32, vp, i32, vp, vp, vp, vp]
        lib.dvdq_oracle_minmax_quant.argtypes = [vp, i64, i64, i32, vp, vp, vp, vp]
        lib.dvdq_oracle_bgr.argtypes = [vp, i64, i64, i32, i32, i32, C.c_double, i32, vp, vp, vp, vp]
        lib.dvdq_oracle_w4ax_gemm_zp.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, vp, vp, vp]
        for f in ("bgr_refine_step", "minmax_quant", "bgr", "w4ax_gemm_zp"):
            getattr(lib, "dvdq_oracle_" + f).restype = i32
        for f in ("hadamard", "rotate", "quantize", "rotate_quant", "w4ax_gemm", "qlinear"):
            getattr(lib, "dvdq_oracle_" + f).restype = i32
        for f in ("unpack_w4", "pack_w4", "unpack_a4", "pack_a4", "unpack_fp6", "pack_fp6", "int_gemm", "epilogue", "f64_to_bf16"):
            getattr(lib, "dvdq_oracle_" + f).restype = None
        _lib = lib
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _arr(a, dtype, ndim=None):
    a = np.ascontiguousarray(a, dtype=dtype)
    if ndim is not None and a.ndim != ndim:
        raise ValueError(f"expected {ndim}-d array, got shape {a.shape}")
    return a


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"oracle {what} failed with code {rc}")


def num_threads() -> int:
    """Threads the OpenMP loops will use (for the benchmark's report)."""
    n = os.environ.get("OMP_NUM_THREADS")
    return int(n) if n else (os.cpu_count() or 1)


def hadamard(B: int) -> np.ndarray:
    H = np.empty((B, B), dtype=np.float64)
    _check(_load().dvdq_oracle_hadamard(B, _p(H)), "hadamard")
    return H


def rotate(x_bf16: np.ndarray, had_block: int) -> np.ndarray:
    x = _arr(x_bf16, np.uint16, 2)
    M, K = x.shape
    out = np.empty((M, K), dtype=np.float64)
    _check(_load().dvdq_oracle_rotate(_p(x), M, K, had_block, _p(out)), "rotate")
    return out


def quantize(xrot: np.ndarray, act_bits: int):
    xr = _arr(xrot, np.float64, 2)
    M, K = xr.shape
    codes = np.empty((M, K), dtype=np.int8)
    scale = np.empty(M, dtype=np.float32)
    _check(_load().dvdq_oracle_quantize(_p(xr), M, K, act_bits, _p(codes), _p(scale)), "quantize")
    return codes, scale


def quantize_blockwise(xrot: np.ndarray, act_bits: int, group: int):
    """Block-wise scaled codes in the int8 container.  Returns (values int8 [M, K], x_scale f32 [M] (already
    divided by 2^emax), exps uint8 [M, K/group])."""
    xr = _arr(xrot, np.float64, 2)
    M, K = xr.shape
    v = np.empty((M, K), dtype=np.int8)
    scale = np.empty(M, dtype=np.float32)
    exps = np.empty((M, K // max(group, 1)), dtype=np.uint8)
    _check(_load().dvdq_oracle_quantize_blockwise(_p(xr), M, K, act_bits, group, _p(v), _p(scale), _p(exps)),
           "quantize_blockwise")
    return v, scale, exps


def rotate_quant(x_bf16: np.ndarray, had_block: int, act_bits: int, return_rotated: bool = False):
    x = _arr(x_bf16, np.uint16, 2)
    M, K = x.shape
    codes = np.empty((M, K), dtype=np.int8)
    scale = np.empty(M, dtype=np.float32)
    xr = np.empty((M, K), dtype=np.float64) if return_rotated else None
    _check(_load().dvdq_oracle_rotate_quant(_p(x), M, K, had_block, act_bits, _p(codes), _p(scale), _p(xr)),
           "rotate_quant")
    return (codes, scale, xr) if return_rotated else (codes, scale)


def unpack_w4(w_packed: np.ndarray) -> np.ndarray:
    w = _arr(w_packed, np.uint8, 2)
    N, K2 = w.shape
    out = np.empty((N, 2 * K2), dtype=np.int8)
    _load().dvdq_oracle_unpack_w4(_p(w), N, 2 * K2, _p(out))
    return out


def pack_w4(codes: np.ndarray) -> np.ndarray:
    c = _arr(codes, np.int8, 2)
    N, K = c.shape
    if K % 2:
        raise ValueError("K must be even")
    out = np.empty((N, K // 2), dtype=np.uint8)
    _load().dvdq_oracle_pack_w4(_p(c), N, K, _p(out))
    return out


def unpack_a4(packed: np.ndarray) -> np.ndarray:
    """Packed 4-bit activation codes uint8 [M, K/2] -> int8 [M, K]."""
    p = _arr(packed, np.uint8, 2)
    M, K2 = p.shape
    if K2 % 4:
        raise ValueError("K must be a multiple of 8")
    out = np.empty((M, 2 * K2), dtype=np.int8)
    _load().dvdq_oracle_unpack_a4(_p(p), M, 2 * K2, _p(out))
    return out


def pack_a4(codes: np.ndarray) -> np.ndarray:
    """int8 [M, K] codes in [-8, 7] -> packed uint8 [M, K/2]."""
    c = _arr(codes, np.int8, 2)
    M, K = c.shape
    if K % 8:
        raise ValueError("K must be a multiple of 8")
    out = np.empty((M, K // 2), dtype=np.uint8)
    _load().dvdq_oracle_pack_a4(_p(c), M, K, _p(out))
    return out


def pack_fp6(codes: np.ndarray) -> np.ndarray:
    """int8 [M, K] codes in [-15, 15] -> the FP6 container of the library's C header (uint8, flat): rows padded
    to a multiple of 32 with zero codes, K a multiple of 128 (layout: see dvdq_oracle_pack_fp6)."""
    c = _arr(codes, np.int8, 2)
    M, K = c.shape
    if K % 128:
        raise ValueError("K must be a multiple of 128")
    if np.abs(c.astype(np.int16)).max(initial=0) > 15:
        raise ValueError("codes out of the E2M3 integer range")
    out = np.empty((M + 31) // 32 * 32 * (K // 128) * 96, dtype=np.uint8)
    _load().dvdq_oracle_pack_fp6(_p(c), M, K, _p(out))
    return out


def unpack_fp6(buf: np.ndarray, M: int, K: int) -> np.ndarray:
    """Inverse of pack_fp6: the first M rows as int8 [M, K]."""
    if K % 128:
        raise ValueError("K must be a multiple of 128")
    b = _arr(buf, np.uint8, 1)
    if b.size < (M + 31) // 32 * 32 * (K // 128) * 96:
        raise ValueError("buffer too small")
    out = np.empty((M, K), dtype=np.int8)
    _load().dvdq_oracle_unpack_fp6(_p(b), M, K, _p(out))
    return out


def int_gemm(codes: np.ndarray, w_codes: np.ndarray) -> np.ndarray:
    q, w = _arr(codes, np.int8, 2), _arr(w_codes, np.int8, 2)
    (M, K), (N, K2) = q.shape, w.shape
    if K != K2:
        raise ValueError("K mismatch")
    acc = np.empty((M, N), dtype=np.int64)
    _load().dvdq_oracle_int_gemm(_p(q), _p(w), M, N, K, _p(acc))
    return acc


def epilogue(acc: np.ndarray, x_scale: np.ndarray, w_scale: np.ndarray, bias_bf16=None) -> np.ndarray:
    a = _arr(acc, np.int64, 2)
    M, N = a.shape
    xs, ws = _arr(x_scale, np.float32, 1), _arr(w_scale, np.float32, 1)
    b = None if bias_bf16 is None else _arr(bias_bf16, np.uint16, 1)
    if xs.size != M or ws.size != N or (b is not None and b.size != N):
        raise ValueError("scale/bias length mismatch")
    y = np.empty((M, N), dtype=np.uint16)
    _load().dvdq_oracle_epilogue(_p(a), _p(xs), _p(ws), _p(b), M, N, _p(y))
    return y


def w4ax_gemm(codes, x_scale, w_packed, w_scale, bias_bf16=None, return_acc: bool = False):
    q = _arr(codes, np.int8, 2)
    w = _arr(w_packed, np.uint8, 2)
    (M, K), N = q.shape, w.shape[0]
    if w.shape[1] * 2 != K:
        raise ValueError("K mismatch")
    xs, ws = _arr(x_scale, np.float32, 1), _arr(w_scale, np.float32, 1)
    b = None if bias_bf16 is None else _arr(bias_bf16, np.uint16, 1)
    y = np.empty((M, N), dtype=np.uint16)
    acc = np.empty((M, N), dtype=np.int64) if return_acc else None
    _check(_load().dvdq_oracle_w4ax_gemm(_p(q), _p(xs), _p(w), _p(ws), _p(b), M, N, K, _p(y), _p(acc)),
           "w4ax_gemm")
    return (y, acc) if return_acc else y


def qlinear(x_bf16, w_packed, w_scale, had_block: int, act_bits: int, bias_bf16=None):
    """Whole layer.  Returns dict(y=bf16 bits, codes, x_scale, acc)."""
    x = _arr(x_bf16, np.uint16, 2)
    w = _arr(w_packed, np.uint8, 2)
    (M, K), N = x.shape, w.shape[0]
    if w.shape[1] * 2 != K:
        raise ValueError("K mismatch")
    ws = _arr(w_scale, np.float32, 1)
    b = None if bias_bf16 is None else _arr(bias_bf16, np.uint16, 1)
    y = np.empty((M, N), dtype=np.uint16)
    codes = np.empty((M, K), dtype=np.int8)
    scale = np.empty(M, dtype=np.float32)
    acc = np.empty((M, N), dtype=np.int64)
    _check(_load().dvdq_oracle_qlinear(_p(x), _p(w), _p(ws), _p(b), M, N, K, had_block, act_bits,
                                       _p(y), _p(codes), _p(scale), _p(acc)), "qlinear")
    return dict(y=y, codes=codes, x_scale=scale, acc=acc)


def f64_to_bf16(a: np.ndarray) -> np.ndarray:
    v = _arr(a, np.float64)
    out = np.empty(v.shape, dtype=np.uint16)
    _load().dvdq_oracle_f64_to_bf16(_p(v), v.size, _p(out))
    return out


def rel_l1(f_t_bf16: np.ndarray, f_prev_bf16: np.ndarray) -> float:
    """||F_t - F_{t-1}||_1 / ||F_{t-1}||_1 on bf16 bit patterns (any shape), fp64 sums."""
    a, b = _arr(f_t_bf16, np.uint16), _arr(f_prev_bf16, np.uint16)
    if a.shape != b.shape:
        raise ValueError("shape mismatch")
    return float(_load().dvdq_oracle_rel_l1(_p(a), _p(b), a.size))


def gbs_update(l1: float, delta: float, b_low: int, b_high: int, acc: float):
    """One controller update.  Returns (bits for the next step, new running sum)."""
    c_acc = C.c_double(acc)
    bits = _load().dvdq_oracle_gbs_update(float(l1), float(delta), b_low, b_high, C.byref(c_acc))
    return bits, c_acc.value


# ------------------------------------------------------------------ offline weight quantizer (Sec. 3.1)
def minmax_quant(w: np.ndarray, bits: int = 4):
    """Plain per-row MinMax: returns (codes uint8 [N, K] in [0, 2^b-1], delta f64 [N], zero int32 [N], err f64 [N])."""
    a = _arr(w, np.float32, 2)
    N, K = a.shape
    q = np.empty((N, K), dtype=np.uint8)
    d = np.empty(N, dtype=np.float64)
    z = np.empty(N, dtype=np.int32)
    e = np.empty(N, dtype=np.float64)
    _check(_load().dvdq_oracle_minmax_quant(_p(a), N, K, bits, _p(q), _p(d), _p(z), _p(e)), "minmax_quant")
    return q, d, z, e


def bgr_refine_step(w_row: np.ndarray, q: np.ndarray, z: int, bits: int = 4):
    """One refinement round on one row.  Returns (delta', z', q', err') or None when undefined."""
    a = _arr(w_row, np.float32, 1)
    qq = _arr(q, np.uint8, 1)
    if a.size != qq.size:
        raise ValueError("length mismatch")
    d = C.c_double(0.0)
    zn = C.c_int(0)
    e = C.c_double(0.0)
    qn = np.empty_like(qq)
    rc = _load().dvdq_oracle_bgr_refine_step(_p(a), a.size, bits, _p(qq), int(z), C.byref(d), C.byref(zn), _p(qn),
                                             C.byref(e))
    return None if rc != 0 else (d.value, zn.value, qn, e.value)


BGR_LISTING, BGR_BEST_OF_ALL = 0, 1


def bgr(w: np.ndarray, bits: int = 4, n_steps: int = 100, max_refine: int = 10, eps: float = 0.0,
        search: int = BGR_LISTING):
    """Bounded-init Grid Refinement per row; `search` = BGR_LISTING (Alg. 1 as printed: starts i = 1, 2, ...,
    a start's result is its last refined grid) or BGR_BEST_OF_ALL (superset search from i = 0, every grid competes).
    Returns (codes uint8 [N, K], delta f64 [N], zero int32 [N], err f64 [N])."""
    a = _arr(w, np.float32, 2)
    N, K = a.shape
    q = np.empty((N, K), dtype=np.uint8)
    d = np.empty(N, dtype=np.float64)
    z = np.empty(N, dtype=np.int32)
    e = np.empty(N, dtype=np.float64)
    _check(_load().dvdq_oracle_bgr(_p(a), N, K, bits, n_steps, max_refine, float(eps), int(search), _p(q), _p(d),
                                   _p(z), _p(e)), "bgr")
    return q, d, z, e


def w4ax_gemm_zp(codes, x_scale, w_packed, w_scale, w_zero, bias_bf16=None, return_acc: bool = False,
                 return_rowsum: bool = False):
    """GEMM + epilogue with signed per-channel weight zero-points (int8 [N])."""
    q = _arr(codes, np.int8, 2)
    w = _arr(w_packed, np.uint8, 2)
    (M, K), N = q.shape, w.shape[0]
    if w.shape[1] * 2 != K:
        raise ValueError("K mismatch")
    xs, ws, wz = _arr(x_scale, np.float32, 1), _arr(w_scale, np.float32, 1), _arr(w_zero, np.int8, 1)
    if xs.size != M or ws.size != N or wz.size != N:
        raise ValueError("scale / zero length mismatch")
    b = None if bias_bf16 is None else _arr(bias_bf16, np.uint16, 1)
    y = np.empty((M, N), dtype=np.uint16)
    acc = np.empty((M, N), dtype=np.int64) if return_acc else None
    rs = np.empty(M, dtype=np.int64) if return_rowsum else None
    _check(_load().dvdq_oracle_w4ax_gemm_zp(_p(q), _p(xs), _p(w), _p(ws), _p(wz), _p(b), M, N, K, _p(y), _p(acc), _p(rs)),
           "w4ax_gemm_zp")
    out = (y,)
    if return_acc:
        out += (acc,)
    if return_rowsum:
        out += (rs,)
    return out if len(out) > 1 else y

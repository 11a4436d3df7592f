"""The C-ABI library: it loads, exports every symbol the headers declare, and its
host-side argument checks answer before anything touches a GPU.  CPU-only (no
compute call is made here)."""
import ctypes as C
import glob
import os
import re

import pytest

import paper_2505_18663_amd as dvdq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    names = set()
    for h in glob.glob(os.path.join(ROOT, "include", "*.h")):
        text = re.sub(r"/\*.*?\*/", "", open(h).read(), flags=re.S)
        names |= set(re.findall(r"\b(dvdq_[a-z0-9_]+)\s*\(", text))
    return names


def test_library_loads_and_exports_every_declared_symbol():
    L = dvdq.lib()
    decl = declared_symbols()
    assert decl, "no declarations found"
    for name in decl:
        assert hasattr(L, name), f"{name} declared in include/ but not exported"
    assert decl == set(dvdq.EXPORTED_SYMBOLS)
    assert dvdq.version() >= 100
    assert dvdq.status_string(0) == "ok" and "NULL" in dvdq.status_string(1)


FAKE = C.c_void_p(0x1000)       # non-NULL, 16-byte aligned; never dereferenced: every call below fails validation
ODD = C.c_void_p(0x1008)


def test_rotate_quant_argument_errors():
    f = dvdq.lib().dvdq_rotate_quant
    assert f(None, 4, 256, 256, 4, 0, FAKE, FAKE, None, None) == 1
    assert f(FAKE, 4, 256, 256, 4, 0, None, FAKE, None, None) == 1
    assert f(FAKE, 0, 256, 256, 4, 0, FAKE, FAKE, None, None) == 2          # M < 1
    assert f(FAKE, 4, 252, 4, 4, 0, FAKE, FAKE, None, None) == 2            # K not a multiple of 8
    assert f(FAKE, 4, 768, 512, 4, 0, FAKE, FAKE, None, None) == 2          # block does not divide K
    assert f(FAKE, 4, 768, 96, 4, 0, FAKE, FAKE, None, None) == 2           # block not a power of two
    assert f(FAKE, 4, 2048, 1024, 4, 0, FAKE, FAKE, None, None) == 3        # block > 512
    assert f(FAKE, 4, 256, 256, 5, 0, FAKE, FAKE, None, None) == 3          # bits
    assert f(FAKE, 4, 131072, 256, 4, 0, FAKE, FAKE, None, None) == 3       # K too large
    assert f(ODD, 4, 256, 256, 4, 0, FAKE, FAKE, None, None) == 5
    assert f(FAKE, 4, 256, 256, 6, 1, FAKE, FAKE, None, None) == 3       # packed container holds 4-bit codes only
    assert f(FAKE, 4, 256, 256, 4, 7, FAKE, FAKE, None, None) == 3       # unknown container
    assert f(FAKE, 4, 256, 256, 6, 2, FAKE, FAKE, None, None) == 3       # the FP6 container holds 4-bit codes only
    assert f(FAKE, 4, 192, 64, 4, 2, FAKE, FAKE, None, None) == 3        # and whole 128-channel slices


def test_rotate_quant_blockwise_argument_errors():
    f = dvdq.lib().dvdq_rotate_quant_blockwise
    assert f(None, 4, 1536, 256, 4, 128, FAKE, FAKE, None, None) == 1
    assert f(FAKE, 4, 1536, 256, 4, 1024, FAKE, FAKE, None, None) == 2     # group does not divide K
    assert f(FAKE, 4, 1536, 256, 4, 64, FAKE, FAKE, None, None) == 3       # group size not built
    assert f(FAKE, 4, 1536, 256, 8, 128, FAKE, FAKE, None, None) == 3      # no headroom for 8-bit codes
    assert f(FAKE, 4, 1536, 256, 4, 128, ODD, FAKE, None, None) == 5


def test_gemm_argument_errors():
    f = dvdq.lib().dvdq_w4ax_gemm
    ok = dict(M=4, N=8, K=64)
    assert f(None, FAKE, FAKE, FAKE, None, None, None, 4, 8, 64, 4, 0, 0, FAKE, None, None) == 1
    assert f(FAKE, FAKE, FAKE, FAKE, None, None, None, 4, 8, 64, 4, 0, 0, None, None, None) == 1
    assert f(FAKE, FAKE, FAKE, FAKE, None, None, None, 4, 0, 64, 4, 0, 0, FAKE, None, None) == 2
    assert f(FAKE, FAKE, FAKE, FAKE, None, None, None, 4, 8, 80, 4, 0, 0, FAKE, None, None) == 2     # K % 32
    assert f(FAKE, FAKE, FAKE, FAKE, None, None, None, 4, 8, 64, 3, 0, 0, FAKE, None, None) == 3
    assert f(FAKE, FAKE, FAKE, FAKE, None, None, None, 4, 8, 64, 4, 0, 7, FAKE, None, None) == 3     # layout
    assert f(FAKE, FAKE, FAKE, FAKE, None, None, None, 4, 8, 64 * 4096, 8, 0, 0, FAKE, None, None) == 3   # accumulator bound
    assert f(FAKE, FAKE, FAKE, FAKE, None, None, None, 4, 8, 192, 4, 0, 1, FAKE, None, None) == 3    # native layout needs K % 128 == 0
    assert f(FAKE, FAKE, ODD, FAKE, None, None, None, 4, 8, 64, 4, 0, 0, FAKE, None, None) == 5
    assert f(FAKE, FAKE, FAKE, FAKE, None, None, ODD, 4, 8, 64, 4, 0, 0, FAKE, None, None) == 5
    assert f(FAKE, FAKE, FAKE, FAKE, None, None, None, 4, 8, 128, 4, 1, 0, FAKE, None, None) == 3   # packed codes need the native layout
    assert f(FAKE, FAKE, FAKE, FAKE, None, None, None, 4, 8, 128, 8, 1, 1, FAKE, None, None) == 3   # packed codes are 4-bit
    assert f(FAKE, FAKE, FAKE, FAKE, None, None, None, 4, 8, 128 * 2048, 4, 1, 1, FAKE, None, None) == 3   # accumulator bound, 256 * acc
    assert f(FAKE, FAKE, FAKE, FAKE, FAKE, None, None, 4, 8, 128, 4, 0, 1, FAKE, None, None) == 1   # zero-points need the code sums
    assert f(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, 4, 8, 64, 4, 0, 0, FAKE, None, None) == 3    # zero-points: native layout only
    assert f(FAKE, FAKE, FAKE, FAKE, ODD, FAKE, None, 4, 8, 128, 4, 0, 1, FAKE, None, None) == 5
    assert f(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, 4, 8, 128 * 600, 8, 0, 1, FAKE, None, None) == 3   # bound with |w - z| <= 16
    assert ok


def test_qlinear_workspace_and_argument_errors():
    L = dvdq.lib()
    M, K = 32760, 1536
    off = dvdq.qlinear_scale_offset(M, K, dvdq.CODES_INT8)
    need = dvdq.qlinear_workspace_bytes(M, K, dvdq.CODES_INT8)
    assert off >= M * K and off % 256 == 0 and need >= off + 4 * M
    off4 = dvdq.qlinear_scale_offset(M, K, dvdq.CODES_PACKED4)
    assert M * K // 2 <= off4 < M * K // 2 + 256 and off4 % 256 == 0
    assert dvdq.qlinear_workspace_bytes(M, K, dvdq.CODES_PACKED4) >= off4 + 4 * M
    rs_off = dvdq.qlinear_rowsum_offset(M, K, dvdq.CODES_INT8)
    assert rs_off >= off + 4 * M and rs_off % 256 == 0 and need >= rs_off + 4 * M
    assert dvdq.qlinear_workspace_bytes(0, K, 0) == 0
    f = L.dvdq_qlinear
    assert f(FAKE, FAKE, FAKE, None, None, M, 64, K, 256, 4, 0, 0, FAKE, None, need, None) == 1
    assert f(FAKE, FAKE, FAKE, None, None, M, 64, K, 256, 4, 0, 0, FAKE, C.c_void_p(0x1010), need, None) == 5
    assert f(FAKE, FAKE, FAKE, None, None, M, 64, K, 256, 4, 0, 0, FAKE, C.c_void_p(0x1100), need - 1, None) == 4
    assert f(FAKE, FAKE, FAKE, None, None, M, 64, K, 1024, 4, 0, 0, FAKE, C.c_void_p(0x1100), need, None) == 2   # 1024 does not divide 1536
    assert f(FAKE, FAKE, FAKE, None, None, 8, 64, 2048, 1024, 4, 0, 0, FAKE, C.c_void_p(0x1100), 1 << 20, None) == 3
    assert f(None, FAKE, FAKE, None, None, M, 64, K, 256, 4, 0, 0, FAKE, C.c_void_p(0x1100), need, None) == 1


def test_prepack_argument_errors_and_size():
    L = dvdq.lib()
    assert dvdq.w4_native_bytes(4608, 1536) >= 4608 * 1536 // 2
    assert dvdq.w4_native_bytes(8, 96) == 0 and dvdq.w4_native_bytes(8, 192) == 0
    assert L.dvdq_w4_prepack(None, 8, 64, FAKE, None) == 1
    assert L.dvdq_w4_prepack(FAKE, 8, 95, FAKE, None) == 2
    assert L.dvdq_w4_prepack(FAKE, 8, 192, FAKE, None) == 3
    assert L.dvdq_w4_prepack(FAKE, 8, 128, ODD, None) == 5


def test_static_workspace_argument_errors():
    L = dvdq.lib()
    assert L.dvdq_static_workspace_bytes() == 64 << 20
    f = L.dvdq_qlinear_static
    assert f(FAKE, FAKE, FAKE, None, None, 0, 8, 256, 256, 4, 0, 1, FAKE, None) == 2              # M < 1
    assert f(FAKE, FAKE, FAKE, None, None, 8, 8, 256, 256, 6, 1, 1, FAKE, None) == 3              # packed codes are 4-bit
    assert f(FAKE, FAKE, FAKE, None, None, 1 << 20, 8, 4096, 256, 4, 0, 1, FAKE, None) == 4       # beyond the fixed array


def test_bgr_argument_errors():
    f = dvdq.lib().dvdq_bgr_quantize
    assert f(None, 8, 64, 100, 10, 0.0, 0, FAKE, FAKE, FAKE, None, None) == 1
    assert f(FAKE, 8, 64, 100, 10, 0.0, 0, FAKE, FAKE, None, None, None) == 1
    assert f(FAKE, 0, 64, 100, 10, 0.0, 0, FAKE, FAKE, FAKE, None, None) == 2
    assert f(FAKE, 8, 63, 100, 10, 0.0, 0, FAKE, FAKE, FAKE, None, None) == 2        # K odd
    assert f(FAKE, 8, 64, 0, 10, 0.0, 0, FAKE, FAKE, FAKE, None, None) == 2          # no search steps
    assert f(FAKE, 8, 64, 100, -1, 0.0, 0, FAKE, FAKE, FAKE, None, None) == 2
    assert f(FAKE, 8, 64, 100, 10, -1.0, 0, FAKE, FAKE, FAKE, None, None) == 2
    assert f(FAKE, 8, 65536, 100, 10, 0.0, 0, FAKE, FAKE, FAKE, None, None) == 3     # row does not fit LDS
    assert f(FAKE, 8, 64, 100, 10, 0.0, 0, ODD, FAKE, FAKE, None, None) == 5
    assert f(FAKE, 8, 64, 100, 10, 0.0, 0, FAKE, FAKE, FAKE, ODD, None) == 5
    assert f(FAKE, 8, 64, 100, 10, 0.0, 2, FAKE, FAKE, FAKE, None, None) == 3     # unknown search mode
    assert f(FAKE, 8, 64, 2, 10, 0.0, 0, FAKE, FAKE, FAKE, None, None) == 2       # the listing's i = 1 needs 3 steps
    assert f(FAKE, 8, 64, 2, 10, 0.0, 1, ODD, FAKE, FAKE, None, None) == 5        # (fine for the superset search)


def test_gbs_argument_errors():
    L = dvdq.lib()
    ws = L.dvdq_gbs_workspace_bytes()
    assert ws >= 16
    assert L.dvdq_gbs_reset(None, 8, None) == 1
    assert L.dvdq_gbs_reset(FAKE, 5, None) == 3
    assert L.dvdq_gbs_reset(ODD, 8, None) == 5
    f = L.dvdq_gbs_step
    assert f(None, FAKE, 64, 0.1, 4, 8, FAKE, FAKE, ws, None) == 1
    assert f(FAKE, FAKE, 0, 0.1, 4, 8, FAKE, FAKE, ws, None) == 2
    assert f(FAKE, FAKE, 64, -1.0, 4, 8, FAKE, FAKE, ws, None) == 2
    assert f(FAKE, FAKE, 64, 0.1, 8, 4, FAKE, FAKE, ws, None) == 3
    assert f(FAKE, FAKE, 64, 0.1, 4, 8, FAKE, FAKE, ws - 1, None) == 4
    assert f(FAKE, ODD, 64, 0.1, 4, 8, FAKE, FAKE, ws, None) == 5


def test_bench_helpers_argument_errors():
    L = dvdq.lib()
    assert L.dvdq_bench_copy(None, FAKE, 64, None) == 1
    assert L.dvdq_bench_copy(FAKE, FAKE, 24, None) == 2
    assert L.dvdq_bench_mfma_i8(0, 0, FAKE, None, None) == 2
    assert L.dvdq_bench_mfma_i8(4, 0, None, None, None) == 1
    assert L.dvdq_bench_mfma_i8(4, 2, FAKE, None, None) == 3
    assert L.dvdq_bench_mfma_fp6(0, 1, FAKE, None, None) == 2
    assert L.dvdq_bench_mfma_fp6(4, 1, None, None, None) == 1
    assert L.dvdq_bench_mfma_fp6(4, -1, FAKE, None, None) == 3
    assert L.dvdq_bench_set_gemm_grid_limit(-8) == 3
    assert L.dvdq_bench_set_gemm_grid_limit(0) == 0
    assert L.dvdq_bench_set_gemm_schedule(2) == 3


def test_binding_refuses_cpu_tensors():
    import torch
    x = torch.zeros((4, 256), dtype=torch.bfloat16)
    with pytest.raises(TypeError):
        dvdq.rotate_quant(x, 256, 4)

"""GPU parity of the asymmetric-weight path: per-token code sums from the quantizer, and the
GEMM epilogue that removes the weight zero-points (DeQuant of Sec. 3.1 inside the layer).
Integer work: bit-exact against the oracle."""
import numpy as np
import pytest
import torch

import dvdq_inputs as di
import oracle
import paper_2505_18663_amd as dvdq
from parity import check_y

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def to_bf16(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).to(DEV)


def bits_of(t):
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def rand_x(rng, M, K):
    x = rng.standard_normal((M, K)).astype(np.float32) * np.exp(rng.normal(0, 0.5, (M, 1))).astype(np.float32)
    x += 0.3 * rng.standard_normal((M, 1)).astype(np.float32)          # a row offset, so the code sums are not ~0
    return di.f32_to_bf16_bits(x)


@pytest.mark.parametrize("M,K,B,bits,packed", [
    (1, 8, 1, 4, False), (7, 96, 32, 6, False), (130, 256, 256, 4, True), (257, 1536, 256, 8, False),
    (33, 1536, 256, 4, True), (6, 13824, 512, 4, True), (6, 13824, 512, 6, False), (4, 65536, 512, 8, False),
    (17, 264, 8, 4, True), (1027, 3072, 256, 4, False),
])
def test_quantizer_code_sums_are_exact(M, K, B, bits, packed):
    rng = np.random.default_rng(M + K + bits)
    x_dev = to_bf16(rand_x(rng, M, K))
    fmt = dvdq.CODES_PACKED4 if packed else dvdq.CODES_INT8
    codes, scale, rs = dvdq.rotate_quant(x_dev, B, bits, codes_format=fmt, want_rowsum=True)
    codes2, scale2 = dvdq.rotate_quant(x_dev, B, bits, codes_format=fmt)
    torch.cuda.synchronize()
    assert torch.equal(codes, codes2) and torch.equal(scale, scale2), "asking for the sums must not change the codes"
    c = codes.cpu().numpy()
    if packed:
        c = oracle.unpack_a4(c)
    assert np.array_equal(rs.cpu().numpy().astype(np.int64), c.astype(np.int64).sum(axis=1))
    assert np.abs(rs.cpu().numpy()).max() > 0


@pytest.mark.parametrize("M,N,K,bits,packed,use_bias", [
    (128, 256, 256, 4, False, False),
    (128, 256, 256, 4, True, True),
    (300, 520, 384, 8, False, True),       # ragged in M and N
    (37, 50, 512, 6, False, False),        # N % 8 != 0
    (513, 260, 1536, 4, True, False),
    (256, 768, 13824, 4, True, True),
    (256, 768, 13824, 8, False, False),    # largest code sums of the workloads' shapes
    (1, 1, 128, 4, True, False),
])
def test_gemm_with_weight_zero_points(M, N, K, bits, packed, use_bias):
    rng = np.random.default_rng(M + 3 * N + 5 * K + bits)
    qmax = 2 ** (bits - 1) - 1
    codes = rng.integers(-qmax, qmax + 1, (M, K)).astype(np.int8)
    codes[:, : K // 2] = np.abs(codes[:, : K // 2])        # large code sums
    wc = rng.integers(-8, 8, (N, K)).astype(np.int8)
    wz = rng.integers(-8, 8, N).astype(np.int8)
    xs = np.exp(rng.normal(-2, 1, M)).astype(np.float32)
    ws = np.exp(rng.normal(-5, 0.5, N)).astype(np.float32)
    bias = di.f32_to_bf16_bits(rng.standard_normal(N).astype(np.float32)) if use_bias else None
    bias_dev = None if bias is None else to_bf16(bias)
    wp = di.pack_w4(wc)
    w_native = dvdq.w4_prepack(dev(wp))
    fmt = dvdq.CODES_PACKED4 if packed else dvdq.CODES_INT8
    codes_dev = dev(oracle.pack_a4(codes)) if packed else dev(codes)
    rs = dev(codes.astype(np.int32).sum(axis=1).astype(np.int32))
    kw = dict(bias=bias_dev, codes_format=fmt, w_zero=dev(wz), code_rowsum=rs)
    y, acc = dvdq.w4ax_gemm(codes_dev, dev(xs), w_native, dev(ws), bits, dvdq.W_NATIVE, want_acc=True, **kw)
    y2 = dvdq.w4ax_gemm(codes_dev, dev(xs), w_native, dev(ws), bits, dvdq.W_NATIVE, **kw)
    torch.cuda.synchronize()
    y_ref, acc_ref = oracle.w4ax_gemm_zp(codes, xs, wp, ws, wz, bias, return_acc=True)
    assert np.array_equal(acc.cpu().numpy().astype(np.int64), acc_ref), "zero-point-corrected accumulators must be exact"
    check_y(bits_of(y), y_ref, f"zp gemm M{M} N{N} K{K}", bias)
    assert torch.equal(y2, y)
    # zero zero-points reproduce the symmetric path bit for bit
    y0 = dvdq.w4ax_gemm(codes_dev, dev(xs), w_native, dev(ws), bits, dvdq.W_NATIVE, bias=bias_dev, codes_format=fmt,
                        w_zero=dev(np.zeros(N, np.int8)), code_rowsum=rs)
    y_sym = dvdq.w4ax_gemm(codes_dev, dev(xs), w_native, dev(ws), bits, dvdq.W_NATIVE, bias=bias_dev, codes_format=fmt)
    assert torch.equal(y0, y_sym)


@pytest.mark.parametrize("idx,packed", [(0, False), (0, True), (1, True)])
def test_qlinear_with_zero_points_is_the_composition(idx, packed):
    wl = di.WORKLOADS[idx]
    M, K, N, B, bits = wl.M, wl.K, wl.N, wl.had_block, wl.act_bits
    rng = np.random.default_rng(idx)
    xb = di.make_x(wl)
    wp, ws, _ = di.make_weights(wl)
    wz = rng.integers(-3, 4, N).astype(np.int8)
    fmt = dvdq.CODES_PACKED4 if packed else dvdq.CODES_INT8
    x_dev, ws_dev, wz_dev = to_bf16(xb), dev(ws), dev(wz)
    w_native = dvdq.w4_prepack(dev(wp))
    y, wsp = dvdq.qlinear(x_dev, w_native, ws_dev, B, bits, dvdq.W_NATIVE, codes_format=fmt, w_zero=wz_dev)
    torch.cuda.synchronize()
    codes, scale = dvdq.workspace_views(wsp, M, K, fmt)
    rs = dvdq.workspace_rowsum(wsp, M, K, fmt)
    c2, s2, rs2 = dvdq.rotate_quant(x_dev, B, bits, codes_format=fmt, want_rowsum=True)
    assert torch.equal(codes, c2) and torch.equal(scale, s2) and torch.equal(rs, rs2)
    y2 = dvdq.w4ax_gemm(c2, s2, w_native, ws_dev, bits, dvdq.W_NATIVE, codes_format=fmt, w_zero=wz_dev, code_rowsum=rs2)
    assert torch.equal(y2, y)
    rows = di.sample_rows(M, 64)
    rows_t = torch.from_numpy(rows).to(DEV)
    cg = codes[rows_t].cpu().numpy()
    cg = oracle.unpack_a4(cg) if packed else cg
    y_ref = oracle.w4ax_gemm_zp(cg, scale[rows_t].cpu().numpy(), wp, ws, wz)
    check_y(bits_of(y[rows_t]), y_ref, wl.name + " zero-points")

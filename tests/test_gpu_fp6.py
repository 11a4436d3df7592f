"""GPU parity of W4A4 on the FP6 matrix path.  4-bit codes are carried as E2M3 bit patterns whose values
are code / 8 exactly, and the fp32 accumulators of the matrix instruction hold the integer sums exactly
(times 1/64), so the bar is the one of an encoding: accumulators equal the oracle's integer GEMM bit for
bit, and outputs equal the INT8 path's bit for bit."""
import numpy as np
import pytest
import torch

import dvdq_inputs as di
import oracle
import paper_2505_18663_amd as dvdq
from parity import check_codes_and_scales, check_y

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def to_bf16(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).to(DEV)


def bits_of(t):
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def gemm_case(rng, M, N, K):
    codes = rng.integers(-7, 8, size=(M, K)).astype(np.int8)
    wc = rng.integers(-8, 8, size=(N, K)).astype(np.int8)
    xs = np.exp(rng.normal(-2, 1, M)).astype(np.float32)
    ws = np.exp(rng.normal(-5, 0.5, N)).astype(np.float32)
    return codes, wc, xs, ws


def test_fp6_weight_prepack_holds_the_oracle_encoding():
    """the prepacked weights are the oracle's FP6 container of the same codes (N padded to 256 rows,
    slices outermost instead of row blocks)"""
    rng = np.random.default_rng(1)
    N, K = 300, 384
    wc = rng.integers(-8, 8, size=(N, K)).astype(np.int8)
    native = dvdq.w4_prepack_fp6(dev(di.pack_w4(wc))).cpu().numpy()
    assert native.size == dvdq.w4_native_fp6_bytes(N, K) == 512 * K * 6 // 8
    padded = np.zeros((512, K), dtype=np.int8)
    padded[:N] = wc
    ref = oracle.pack_fp6(padded).reshape(512 // 32, K // 128, 3072).transpose(1, 0, 2)   # -> [slice][block]
    assert np.array_equal(native.reshape(K // 128, 512 // 32, 3072), ref)


@pytest.mark.parametrize("schedule,variant", [(-1, -1), (0, -1), (-1, 1), (-1, 2), (0, 2)])
@pytest.mark.parametrize("M,N,K,use_bias", [
    (1, 1, 128, False),          # one row, one channel, one K slice
    (128, 256, 256, True),       # exactly one interior tile
    (300, 520, 384, False),      # ragged in M and N
    (513, 260, 1536, True),
    (37, 50, 512, True),         # N % 8 != 0: scalar store path
    (1000, 1024, 640, False),    # 32 tiles
    (4100, 2056, 384, True),     # 17 x 9 tiles of 256 x 256, ragged in M and N
    (256, 768, 13824, False),    # deepest K of the workloads
])
def test_fp6_gemm_int32_exact(M, N, K, use_bias, schedule, variant):
    rng = np.random.default_rng(M + 7 * N + 13 * K)
    codes, wc, xs, ws = gemm_case(rng, M, N, K)
    wp = di.pack_w4(wc)
    bias = di.f32_to_bf16_bits(rng.standard_normal(N).astype(np.float32)) if use_bias else None
    bias_dev = None if bias is None else to_bf16(bias)
    w6 = dvdq.w4_prepack_fp6(dev(wp))
    c6 = dev(oracle.pack_fp6(codes))
    assert c6.numel() == dvdq.codes_bytes(M, K, dvdq.CODES_FP6)
    dvdq.bench_set_gemm_schedule(schedule)
    dvdq.bench_set_gemm_variant(variant)   # 1: 128 x 256 tiles, two workgroups per compute unit; 2: 256 x 256 tiles, one
    try:
        y, acc = dvdq.w4ax_gemm(c6, dev(xs), w6, dev(ws), 4, dvdq.W_NATIVE_FP6, bias=bias_dev, want_acc=True,
                                codes_format=dvdq.CODES_FP6, K=K)
        y2 = dvdq.w4ax_gemm(c6, dev(xs), w6, dev(ws), 4, dvdq.W_NATIVE_FP6, bias=bias_dev, codes_format=dvdq.CODES_FP6, K=K)
        torch.cuda.synchronize()
    finally:
        dvdq.bench_set_gemm_schedule(-1)
        dvdq.bench_set_gemm_variant(-1)
    y_ref, acc_ref = oracle.w4ax_gemm(codes, xs, wp, ws, bias, return_acc=True)
    assert np.array_equal(acc.cpu().numpy().astype(np.int64), acc_ref), "accumulators must be bit-exact"
    check_y(bits_of(y), y_ref, f"fp6 gemm M{M} N{N} K{K}", bias)
    assert torch.equal(y2, y), "interior and per-element epilogues must agree"
    y8 = dvdq.w4ax_gemm(dev(codes), dev(xs), dvdq.w4_prepack(dev(wp)), dev(ws), 4, dvdq.W_NATIVE, bias=bias_dev)
    assert torch.equal(y8, y), "the matrix path must not change the outputs"


@pytest.mark.parametrize("M,N,K,use_bias", [(300, 520, 384, True), (1024, 512, 1536, False), (37, 50, 512, True)])
def test_fp6_gemm_with_zero_points(M, N, K, use_bias):
    rng = np.random.default_rng(M + N + K)
    codes, wc, xs, ws = gemm_case(rng, M, N, K)
    wp = di.pack_w4(wc)
    wz = rng.integers(-8, 8, N).astype(np.int8)
    rowsum = codes.astype(np.int32).sum(axis=1).astype(np.int32)
    bias = di.f32_to_bf16_bits(rng.standard_normal(N).astype(np.float32)) if use_bias else None
    bias_dev = None if bias is None else to_bf16(bias)
    kw = dict(bias=bias_dev, w_zero=dev(wz), code_rowsum=dev(rowsum))
    y, acc = dvdq.w4ax_gemm(dev(oracle.pack_fp6(codes)), dev(xs), dvdq.w4_prepack_fp6(dev(wp)), dev(ws), 4, dvdq.W_NATIVE_FP6,
                            want_acc=True, codes_format=dvdq.CODES_FP6, K=K, **kw)
    y2 = dvdq.w4ax_gemm(dev(oracle.pack_fp6(codes)), dev(xs), dvdq.w4_prepack_fp6(dev(wp)), dev(ws), 4, dvdq.W_NATIVE_FP6,
                        codes_format=dvdq.CODES_FP6, K=K, **kw)
    y8, acc8 = dvdq.w4ax_gemm(dev(codes), dev(xs), dvdq.w4_prepack(dev(wp)), dev(ws), 4, dvdq.W_NATIVE, want_acc=True, **kw)
    torch.cuda.synchronize()
    acc_ref = oracle.int_gemm(codes, wc) - wz.astype(np.int64)[None, :] * rowsum.astype(np.int64)[:, None]
    assert np.array_equal(acc.cpu().numpy().astype(np.int64), acc_ref)
    assert torch.equal(acc, acc8) and torch.equal(y, y8) and torch.equal(y, y2)


def test_fp6_is_refused_where_it_does_not_apply():
    M, N, K = 64, 256, 256
    xs, ws = torch.ones(M, device=DEV), torch.ones(N, device=DEV)
    w6 = torch.zeros(dvdq.w4_native_fp6_bytes(N, K), dtype=torch.uint8, device=DEV)
    c6 = torch.zeros(dvdq.codes_bytes(M, K, dvdq.CODES_FP6), dtype=torch.uint8, device=DEV)
    with pytest.raises(dvdq.DvdqError):   # 6-bit codes do not fit
        dvdq.w4ax_gemm(c6, xs, w6, ws, 6, dvdq.W_NATIVE_FP6, codes_format=dvdq.CODES_FP6, K=K)
    with pytest.raises(dvdq.DvdqError):   # FP6 codes against INT4 native weights
        dvdq.w4ax_gemm(c6, xs, w6, ws, 4, dvdq.W_NATIVE, codes_format=dvdq.CODES_FP6, K=K)
    c8 = torch.zeros((M, K), dtype=torch.int8, device=DEV)
    with pytest.raises(dvdq.DvdqError):   # int8 codes against FP6 weights
        dvdq.w4ax_gemm(c8, xs, w6, ws, 4, dvdq.W_NATIVE_FP6)


def rand_x(rng, M, K):
    x = rng.standard_normal((M, K)).astype(np.float32) * np.exp(rng.normal(0, 0.5, (M, 1))).astype(np.float32)
    x[:, rng.choice(K, size=max(1, K // 100), replace=False)] *= 50.0
    return di.f32_to_bf16_bits(x)


@pytest.mark.parametrize("M,K,B", [
    (1, 128, 1), (3, 128, 128), (7, 384, 32), (130, 256, 256), (33, 768, 256), (257, 1536, 256), (64, 3072, 256),
    (31, 512, 512), (6, 13824, 512), (17, 640, 8), (4, 65536, 512), (1027, 1536, 256), (40, 2560, 512),
    (70, 13824, 512), (45, 32768, 512), (70, 8192, 256),   # rows of many units: runs of 8, 4 and 2 rows staged per wave
])
def test_rotate_quant_fp6_decodes_to_the_int8_codes(M, K, B):
    rng = np.random.default_rng(M * 17 + K + B)
    xb = rand_x(rng, M, K)
    x_dev = to_bf16(xb)
    c6, scale6, rs6 = dvdq.rotate_quant(x_dev, B, 4, codes_format=dvdq.CODES_FP6, want_rowsum=True)
    codes8, scale8, rs8 = dvdq.rotate_quant(x_dev, B, 4, want_rowsum=True)
    torch.cuda.synchronize()
    assert c6.dtype == torch.uint8 and c6.numel() == dvdq.codes_bytes(M, K, dvdq.CODES_FP6)
    decoded = oracle.unpack_fp6(c6.cpu().numpy(), M, K)
    assert np.array_equal(decoded, codes8.cpu().numpy()), "both containers must carry the same codes"
    assert torch.equal(scale6, scale8) and torch.equal(rs6, rs8)
    codes_r, scale_r, xr = oracle.rotate_quant(xb, B, 4, return_rotated=True)
    check_codes_and_scales(decoded, scale6.cpu().numpy(), codes_r, scale_r, xr, 4, f"fp6 M{M} K{K} B{B}",
                           allow_fp32_ties=B <= 8)


def test_rotate_quant_fp6_leaves_neighbouring_memory_alone():
    M, K = 37, 1536
    need = dvdq.codes_bytes(M, K, dvdq.CODES_FP6)
    buf = torch.full((need + 512,), 0xA5, dtype=torch.uint8, device=DEV)
    codes = buf[256:256 + need]
    dvdq.rotate_quant(to_bf16(rand_x(np.random.default_rng(5), M, K)), 256, 4, codes=codes, codes_format=dvdq.CODES_FP6)
    torch.cuda.synchronize()
    assert bool((buf[:256] == 0xA5).all()) and bool((buf[256 + need:] == 0xA5).all())
    # rows 37..63 of the second block are padding: never written
    blk = buf[256:256 + need].cpu().numpy().reshape(2, K // 128, 6, 32, 16)
    assert (blk[1, :, :, 5:, :] == 0xA5).all() and not (blk[1, :, :, :5, :] == 0xA5).all()


@pytest.mark.parametrize("idx", [0, 1, 3, 4])
def test_qlinear_on_the_fp6_path_matches_the_int8_path(idx):
    wl = di.WORKLOADS[idx]
    M, K, N, B = wl.M, wl.K, wl.N, wl.had_block
    assert wl.act_bits == 4
    print(f"[{wl.name}] inputs", flush=True)
    xb = di.make_x(wl)
    wp, ws, _ = di.make_weights(wl)
    x_dev, ws_dev = to_bf16(xb), dev(ws)
    print(f"[{wl.name}] qlinear fp6 M={M} K={K} N={N}", flush=True)
    y, wsp = dvdq.qlinear(x_dev, dvdq.w4_prepack_fp6(dev(wp)), ws_dev, B, 4, dvdq.W_NATIVE_FP6, codes_format=dvdq.CODES_FP6)
    y8, wsp8 = dvdq.qlinear(x_dev, dvdq.w4_prepack(dev(wp)), ws_dev, B, 4, dvdq.W_NATIVE)
    torch.cuda.synchronize()
    assert wsp.numel() == dvdq.qlinear_workspace_bytes(M, K, dvdq.CODES_FP6) < wsp8.numel()
    assert torch.equal(y, y8)
    c6, scale = dvdq.workspace_views(wsp, M, K, dvdq.CODES_FP6)
    codes8, scale8 = dvdq.workspace_views(wsp8, M, K)
    assert torch.equal(scale, scale8)
    # first 256 + last 256 rows (the ragged last tile) + 64 from the middle, as in the INT8 full-size test
    rows = di.sample_rows(M, 256)
    if M > 512:
        rows = np.unique(np.concatenate([rows, np.random.default_rng(M).choice(np.arange(256, M - 256), 64, replace=False)]))
    rows_t = torch.from_numpy(rows).to(DEV)
    decoded = oracle.unpack_fp6(c6.cpu().numpy(), M, K)[rows]
    assert np.array_equal(decoded, codes8[rows_t].cpu().numpy())
    codes_r, scale_r, xr = oracle.rotate_quant(np.ascontiguousarray(xb[rows]), B, 4, return_rotated=True)
    scale_g = scale[rows_t].cpu().numpy()
    check_codes_and_scales(decoded, scale_g, codes_r, scale_r, xr, 4, wl.name + " fp6")
    check_y(bits_of(y[rows_t]), oracle.w4ax_gemm(decoded, scale_g, wp, ws), wl.name + " fp6")

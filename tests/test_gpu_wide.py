"""The 4-wave / 128 x 128-wave-tile GEMM kernels (accumulators in AGPRs) against the two-waves-per-SIMD kernels
and the oracle.  Both run the same integer contraction and the same epilogue arithmetic, so outputs and
accumulators must agree bit for bit: over single tiles, edge tiles, one K slice, N not a multiple of 8, more
tiles than workgroups, bias, zero-points, the accumulator hook, drawn and fixed tile shares."""
import numpy as np
import pytest
import torch

import oracle
import paper_2505_18663_amd as dvdq

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
WIDE_INT8, WIDE_FP6 = 5, 3     # tile-variant numbers of the wide kernels on the two matrix paths


@pytest.fixture(autouse=True)
def _library_defaults():
    yield
    dvdq.bench_set_gemm_schedule(-1)
    dvdq.bench_set_gemm_variant(-1)
    dvdq.bench_set_gemm_grid_limit(0)


def _case(M, K, N, bits, seed, fp6):
    rng = np.random.default_rng(seed)
    qmax = 2 ** (bits - 1) - 1
    codes = rng.integers(-qmax, qmax + 1, (M, K)).astype(np.int8)
    wc = rng.integers(-8, 8, (N, K)).astype(np.int8)
    wp = oracle.pack_w4(wc)
    xs = (rng.random(M) + 0.01).astype(np.float32)
    ws = (rng.random(N) * 0.01 + 1e-3).astype(np.float32)
    wz = rng.integers(-8, 8, N).astype(np.int8)
    bias = torch.from_numpy(rng.standard_normal(N).astype(np.float32)).to(DEV).to(torch.bfloat16)
    d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    if fp6:
        c_dev, w_dev = d(oracle.pack_fp6(codes)), dvdq.w4_prepack_fp6(d(wp))
        kw = dict(codes_format=dvdq.CODES_FP6, K=K)
        lay = dvdq.W_NATIVE_FP6
    else:
        c_dev, w_dev = d(codes), dvdq.w4_prepack(d(wp))
        kw, lay = {}, dvdq.W_NATIVE
    rs = d(codes.astype(np.int32).sum(axis=1).astype(np.int32))
    return dict(codes=codes, wc=wc, c_dev=c_dev, w_dev=w_dev, xs=d(xs), ws=d(ws), wz=d(wz), rs=rs, bias=bias, kw=kw,
                lay=lay, bits=bits)


def _run(c, variant, schedule=-1, **extra):
    dvdq.bench_set_gemm_variant(variant)
    dvdq.bench_set_gemm_schedule(schedule)
    out = dvdq.w4ax_gemm(c["c_dev"], c["xs"], c["w_dev"], c["ws"], c["bits"], c["lay"], **c["kw"], **extra)
    torch.cuda.synchronize()
    return out


SHAPES = [
    # M, K, N, bits
    (128, 128, 256, 4),        # one tile, one K slice
    (256, 256, 256, 4),        # one full (interior) tile
    (100, 256, 200, 8),        # one edge tile
    (1000, 384, 776, 6),       # 4 x 4 tiles, ragged in M and N
    (700, 512, 1030, 4),       # N not a multiple of 8: per-element path on every tile
    (2048, 1536, 1024, 4),     # 32 interior tiles, 12 slices
    (8192, 256, 8192, 4),      # 1024 tiles: four per workgroup, two K slices
    (5000, 640, 2304, 6),      # 20 x 9 tiles, ragged M
    (513, 128, 264, 4),        # one K slice, several tiles (fixed shares only)
]


@pytest.mark.parametrize("fp6", [False, True])
@pytest.mark.parametrize("M,K,N,bits", SHAPES)
def test_wide_kernel_matches_the_two_wave_kernel_and_the_oracle(M, K, N, bits, fp6):
    if fp6 and bits != 4:
        bits = 4
    print(f"wide M{M} K{K} N{N} b{bits} fp6={fp6}", flush=True)
    c = _case(M, K, N, bits, M + N + K, fp6)
    wide = WIDE_FP6 if fp6 else WIDE_INT8
    y_ref, acc_ref = _run(c, -1, want_acc=True)
    y_ref2 = _run(c, -1)
    acc_or = oracle.int_gemm(c["codes"], c["wc"])
    assert np.array_equal(acc_ref.cpu().numpy().astype(np.int64), acc_or)
    for schedule in (0, -1):
        y, acc = _run(c, wide, schedule, want_acc=True)
        assert np.array_equal(acc.cpu().numpy().astype(np.int64), acc_or), f"accumulators, schedule {schedule}"
        assert torch.equal(y.view(torch.int16), y_ref.view(torch.int16)), f"outputs (hook path), schedule {schedule}"
        y2 = _run(c, wide, schedule)
        assert torch.equal(y2.view(torch.int16), y_ref2.view(torch.int16)), f"outputs, schedule {schedule}"
        assert torch.equal(y2.view(torch.int16), y.view(torch.int16))


@pytest.mark.parametrize("fp6", [False, True])
def test_wide_kernel_bias_and_zero_points(fp6):
    for (M, K, N, bits) in [(600, 384, 520, 6), (2048, 512, 1024, 4), (300, 256, 1030, 4)]:
        if fp6:
            bits = 4
        c = _case(M, K, N, bits, 77 + M, fp6)
        wide = WIDE_FP6 if fp6 else WIDE_INT8
        for extra in (dict(bias=c["bias"]), dict(w_zero=c["wz"], code_rowsum=c["rs"]),
                      dict(bias=c["bias"], w_zero=c["wz"], code_rowsum=c["rs"])):
            y_ref, acc_ref = _run(c, -1, want_acc=True, **extra)
            y, acc = _run(c, wide, want_acc=True, **extra)
            assert torch.equal(acc, acc_ref) and torch.equal(y.view(torch.int16), y_ref.view(torch.int16)), (M, K, N, list(extra))
            y2_ref, y2 = _run(c, -1, **extra), _run(c, wide, **extra)
            assert torch.equal(y2.view(torch.int16), y2_ref.view(torch.int16)), (M, K, N, list(extra))
        if "w_zero" in extra:
            acc_or = oracle.int_gemm(c["codes"], c["wc"]) - c["codes"].astype(np.int64).sum(axis=1)[:, None] * c["wz"].cpu().numpy().astype(np.int64)[None, :]
            assert np.array_equal(acc.cpu().numpy().astype(np.int64), acc_or)


@pytest.mark.parametrize("fp6", [False, True])
def test_wide_kernel_many_launches_in_a_row(fp6):
    """the tile counters must be back at zero after every kernel; two shapes alternate on one stream"""
    a = _case(4100, 512, 2056, 4, 3, fp6)
    b = _case(700, 256, 520, 4, 4, fp6)
    wide = WIDE_FP6 if fp6 else WIDE_INT8
    ya_ref, yb_ref = _run(a, -1), _run(b, -1)
    dvdq.bench_set_gemm_variant(wide)
    ya, yb = torch.empty_like(ya_ref), torch.empty_like(yb_ref)
    for it in range(40):
        ya.zero_()
        yb.zero_()
        dvdq.w4ax_gemm(a["c_dev"], a["xs"], a["w_dev"], a["ws"], 4, a["lay"], y=ya, **a["kw"])
        dvdq.w4ax_gemm(b["c_dev"], b["xs"], b["w_dev"], b["ws"], 4, b["lay"], y=yb, **b["kw"])
        if it % 10 == 9:
            torch.cuda.synchronize()
            assert torch.equal(ya.view(torch.int16), ya_ref.view(torch.int16)), f"iteration {it}"
            assert torch.equal(yb.view(torch.int16), yb_ref.view(torch.int16)), f"iteration {it}"


@pytest.mark.parametrize("fp6", [False, True])
@pytest.mark.parametrize("K", [128, 256, 384, 640, 1152])
def test_wide_kernel_with_few_workgroups_walking_many_tiles(K, fp6):
    """8 and 24 workgroups for 20 x 5 tiles: every workgroup goes through several tiles in a row (tile draws or fixed
    shares, the load pipeline across tile boundaries, the epilogue's staging buffer) at one to nine K slices per tile"""
    c = _case(5000, K, 1160, 4, 500 + K, fp6)
    wide = WIDE_FP6 if fp6 else WIDE_INT8
    extra = dict(bias=c["bias"]) if K % 256 else {}
    y_ref = _run(c, -1, **extra)
    for limit in (8, 24):
        dvdq.bench_set_gemm_grid_limit(limit)
        for schedule in (0, -1):
            print(f"wide K{K} fp6={fp6} workgroups {limit} schedule {schedule}", flush=True)
            y = _run(c, wide, schedule, **extra)
            assert torch.equal(y.view(torch.int16), y_ref.view(torch.int16)), (K, limit, schedule)
    dvdq.bench_set_gemm_grid_limit(0)


@pytest.mark.parametrize("K", [1152, 1280])
def test_default_dispatch_around_the_fp6_wide_kernel_threshold(K):
    """512 tiles of 256 x 256 (two rounds of them on the chip): below ten K slices the library takes the 8-wave FP6
    kernel by itself, from ten on the wide one.  Whatever it takes must equal both kernels forced, bit for bit, and
    the integer contraction of the oracle on a sample of token rows."""
    M, N = 4096, 8192
    print(f"dispatch threshold K{K}", flush=True)
    c = _case(M, K, N, 4, 9000 + K, True)
    y_default, acc = _run(c, -1, want_acc=True)
    rows = np.r_[0:24, 2040:2056, M - 24:M]
    acc_or = oracle.int_gemm(c["codes"][rows], c["wc"])
    assert np.array_equal(acc.cpu().numpy()[rows].astype(np.int64), acc_or)
    y_plain = _run(c, -1)
    assert torch.equal(y_plain.view(torch.int16), y_default.view(torch.int16))
    for variant in (1, 2, WIDE_FP6):
        y = _run(c, variant)
        assert torch.equal(y.view(torch.int16), y_plain.view(torch.int16)), f"variant {variant}"

"""Tile scheduling of the native-layout GEMM.  The persistent workgroups either draw their tiles from
per-stream counters in device memory (default) or take fixed equal shares (while a stream is being
captured, or forced through the benchmark hook).  Which workgroup computes a tile must not show in
the result: outputs are compared bit for bit between the two modes, over shapes with fewer tiles than
workgroups, edge tiles, every tile variant, many launches in a row (no launch may depend on what the
one before left in the counters), counters overwritten with garbage between launches, and launches on
several streams at once (one counter slot per stream)."""
import pytest
import torch

import paper_2505_18663_amd as dvdq

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(autouse=True)
def _library_defaults():
    yield
    dvdq.bench_set_gemm_schedule(-1)
    dvdq.bench_set_gemm_variant(-1)


def _operands(M, K, N, bits, packed, seed):
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    qmax = 2 ** (bits - 1) - 1
    codes = torch.randint(-qmax, qmax + 1, (M, K), device=DEV, dtype=torch.int8, generator=g)
    if packed:   # byte b of a group of 8 channels = code[8g+b] | code[8g+b+4] << 4
        c = codes.view(M, K // 8, 2, 4).to(torch.int16) & 0xF
        codes = (c[:, :, 0, :] | (c[:, :, 1, :] << 4)).to(torch.uint8).view(M, K // 2).contiguous()
    xs = torch.rand((M,), device=DEV, generator=g) + 0.01
    w = dvdq.w4_prepack(torch.randint(0, 256, (N, K // 2), device=DEV, dtype=torch.uint8, generator=g))
    ws = torch.rand((N,), device=DEV, generator=g) * 0.01 + 1e-3
    return codes, xs, w, ws


def _gemm(ops, bits, packed, y=None, stream=None, want_acc=False):
    codes, xs, w, ws = ops
    fmt = dvdq.CODES_PACKED4 if packed else dvdq.CODES_INT8
    return dvdq.w4ax_gemm(codes, xs, w, ws, bits, dvdq.W_NATIVE, y=y, codes_format=fmt, stream=stream, want_acc=want_acc)


SHAPES = [
    # M, K, N, bits, packed
    (128, 128, 256, 4, True),        # one tile, one K slice
    (100, 256, 200, 8, False),       # one edge tile
    (1000, 384, 776, 6, False),      # 8 x 4 tiles: fewer than workgroups, ragged in M and N
    (3000, 512, 1030, 4, True),      # N not a multiple of 8: per-element path on every tile
    (8192, 1024, 4096, 4, True),     # 1024 tiles: two per workgroup
    (20000, 640, 2304, 4, False),    # 157 x 9 tiles, uneven shares, ragged M
]


@pytest.mark.parametrize("M,K,N,bits,packed", SHAPES)
def test_drawn_and_fixed_shares_give_identical_outputs(M, K, N, bits, packed):
    ops = _operands(M, K, N, bits, packed, seed=M + N)
    dvdq.bench_set_gemm_schedule(0)
    y_fixed = _gemm(ops, bits, packed)                            # interior tiles take the staged epilogue
    y2_fixed, acc_fixed = _gemm(ops, bits, packed, want_acc=True)  # the accumulator hook: per-element epilogue
    dvdq.bench_set_gemm_schedule(-1)
    y_drawn = _gemm(ops, bits, packed)
    y2_drawn, acc_drawn = _gemm(ops, bits, packed, want_acc=True)
    torch.cuda.synchronize()
    assert torch.equal(acc_fixed, acc_drawn)
    assert torch.equal(y_fixed.view(torch.int16), y_drawn.view(torch.int16))
    assert torch.equal(y2_fixed.view(torch.int16), y2_drawn.view(torch.int16))
    assert torch.equal(y_fixed.view(torch.int16), y2_fixed.view(torch.int16))


@pytest.mark.parametrize("variant", [1, 2, 3, 4])
@pytest.mark.parametrize("packed", [False, True])
def test_every_tile_variant_agrees_between_the_two_modes(variant, packed):
    M, K, N, bits = 5000, 768, 1536, 4
    ops = _operands(M, K, N, bits, packed, seed=variant)
    dvdq.bench_set_gemm_variant(variant)
    dvdq.bench_set_gemm_schedule(0)
    y_fixed = _gemm(ops, bits, packed)
    dvdq.bench_set_gemm_schedule(-1)
    y_drawn = _gemm(ops, bits, packed)
    torch.cuda.synchronize()
    assert torch.equal(y_fixed.view(torch.int16), y_drawn.view(torch.int16))


def test_many_launches_in_a_row_on_one_stream():
    """200 launches in a row on one stream, alternating between two shapes: a launch that counted on from
    where the one before stopped would skip or repeat tiles."""
    a = _operands(4096, 512, 2048, 4, True, seed=1)
    b = _operands(700, 256, 520, 6, False, seed=2)
    dvdq.bench_set_gemm_schedule(0)
    ya_ref, yb_ref = _gemm(a, 4, True), _gemm(b, 6, False)
    dvdq.bench_set_gemm_schedule(-1)
    ya, yb = torch.empty_like(ya_ref), torch.empty_like(yb_ref)
    for it in range(100):
        ya.zero_()
        yb.zero_()
        _gemm(a, 4, True, y=ya)
        _gemm(b, 6, False, y=yb)
        if it % 10 == 9:
            torch.cuda.synchronize()
            assert torch.equal(ya.view(torch.int16), ya_ref.view(torch.int16)), f"iteration {it}"
            assert torch.equal(yb.view(torch.int16), yb_ref.view(torch.int16)), f"iteration {it}"


def test_launches_on_several_streams_do_not_share_counters():
    ops = [_operands(6000 + 512 * i, 512, 1536, 4, True, seed=10 + i) for i in range(4)]
    dvdq.bench_set_gemm_schedule(0)
    refs = [_gemm(o, 4, True) for o in ops]
    dvdq.bench_set_gemm_schedule(-1)
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream() for _ in ops]
    outs = [torch.zeros_like(r) for r in refs]
    for rep in range(20):
        for s, o, y in zip(streams, ops, outs):
            with torch.cuda.stream(s):
                _gemm(o, 4, True, y=y, stream=s)
    torch.cuda.synchronize()
    for i, (y, r) in enumerate(zip(outs, refs)):
        assert torch.equal(y.view(torch.int16), r.view(torch.int16)), f"stream {i}"


def _fp6_operands(M, K, N, seed):
    import oracle
    rng = __import__("numpy").random.default_rng(seed)
    codes = rng.integers(-7, 8, (M, K)).astype("int8")
    c6 = torch.from_numpy(oracle.pack_fp6(codes)).to(DEV)
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    xs = torch.rand((M,), device=DEV, generator=g) + 0.01
    w = dvdq.w4_prepack_fp6(torch.randint(0, 256, (N, K // 2), device=DEV, dtype=torch.uint8, generator=g))
    ws = torch.rand((N,), device=DEV, generator=g) * 0.01 + 1e-3
    return c6, xs, w, ws, K


def _fp6_gemm(ops, y=None, stream=None):
    c6, xs, w, ws, K = ops
    return dvdq.w4ax_gemm(c6, xs, w, ws, 4, dvdq.W_NATIVE_FP6, y=y, codes_format=dvdq.CODES_FP6, K=K, stream=stream)


@pytest.mark.parametrize("variant", [1, 2])
def test_fp6_kernel_counters_and_streams(variant):
    """the FP6 matrix path's kernel draws tiles the same way: both tile variants, many launches in a row on
    one stream and launches on several streams at once, against fixed shares"""
    a = _fp6_operands(4100, 512, 2056, seed=3)     # 17 x 9 tiles of 256 x 256 (33 x 9 of 128 x 256), ragged
    b = _fp6_operands(700, 256, 520, seed=4)
    dvdq.bench_set_gemm_variant(variant)
    dvdq.bench_set_gemm_schedule(0)
    ya_ref, yb_ref = _fp6_gemm(a), _fp6_gemm(b)
    dvdq.bench_set_gemm_schedule(-1)
    ya, yb = torch.empty_like(ya_ref), torch.empty_like(yb_ref)
    for it in range(60):
        ya.zero_()
        yb.zero_()
        _fp6_gemm(a, y=ya)
        _fp6_gemm(b, y=yb)
        if it % 10 == 9:
            torch.cuda.synchronize()
            assert torch.equal(ya.view(torch.int16), ya_ref.view(torch.int16)), f"iteration {it}"
            assert torch.equal(yb.view(torch.int16), yb_ref.view(torch.int16)), f"iteration {it}"
    streams = [torch.cuda.Stream() for _ in range(3)]
    outs = [torch.zeros_like(ya_ref) for _ in streams]
    torch.cuda.synchronize()
    for rep in range(10):
        for s, y in zip(streams, outs):
            with torch.cuda.stream(s):
                _fp6_gemm(a, y=y, stream=s)
    torch.cuda.synchronize()
    for i, y in enumerate(outs):
        assert torch.equal(y.view(torch.int16), ya_ref.view(torch.int16)), f"stream {i}"


@pytest.mark.parametrize("value", [0xFFFFF, 0xFFFFFFFF, 0x7FF00003, 0xFFF80000, 1])
def test_gemms_do_not_depend_on_what_the_tile_counters_hold(value):
    """Every counter word overwritten (as a launch that never finished, or a stray write, would leave it) before
    each of several launches: the two-wave INT8 kernel, the wide INT8 kernel, both FP6 kernels, and the fused
    layer, whose quantizer kernel is what clears the counters."""
    s = torch.cuda.Stream()
    i8 = _operands(4096, 512, 2048, 4, True, seed=21)
    wide = _operands(2100, 384, 1300, 4, False, seed=22)
    f6 = _fp6_operands(4100, 512, 2056, seed=23)
    dvdq.bench_set_gemm_schedule(0)
    ref_i8 = _gemm(i8, 4, True)
    dvdq.bench_set_gemm_variant(5)
    ref_wide = _gemm(wide, 4, False)
    dvdq.bench_set_gemm_variant(3)
    ref_f6w = _fp6_gemm(f6)
    dvdq.bench_set_gemm_variant(-1)
    ref_f6 = _fp6_gemm(f6)
    g = torch.Generator(device=DEV)
    g.manual_seed(24)
    x = torch.randn((3000, 512), device=DEV, generator=g).to(torch.bfloat16)
    ref_layer, _ = dvdq.qlinear(x, f6[2], f6[3], 256, 4, dvdq.W_NATIVE_FP6, codes_format=dvdq.CODES_FP6)
    dvdq.bench_set_gemm_schedule(-1)
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        for rep in range(3):
            dvdq.bench_fill_tile_counters(value, stream=s)
            y_layer, _ = dvdq.qlinear(x, f6[2], f6[3], 256, 4, dvdq.W_NATIVE_FP6, codes_format=dvdq.CODES_FP6, stream=s)
            dvdq.bench_fill_tile_counters(value, stream=s)
            y = _gemm(i8, 4, True, stream=s)
            dvdq.bench_fill_tile_counters(value + rep, stream=s)
            dvdq.bench_set_gemm_variant(5)
            yw = _gemm(wide, 4, False, stream=s)
            dvdq.bench_fill_tile_counters(value, stream=s)
            dvdq.bench_set_gemm_variant(3)
            y6w = _fp6_gemm(f6, stream=s)
            dvdq.bench_set_gemm_variant(-1)
            dvdq.bench_fill_tile_counters(value ^ 5, stream=s)
            y6 = _fp6_gemm(f6, stream=s)
            s.synchronize()
            assert torch.equal(y.view(torch.int16), ref_i8.view(torch.int16)), f"int8, round {rep}"
            assert torch.equal(yw.view(torch.int16), ref_wide.view(torch.int16)), f"wide int8, round {rep}"
            assert torch.equal(y6w.view(torch.int16), ref_f6w.view(torch.int16)), f"wide fp6, round {rep}"
            assert torch.equal(y6.view(torch.int16), ref_f6.view(torch.int16)), f"fp6, round {rep}"
            assert torch.equal(y_layer.view(torch.int16), ref_layer.view(torch.int16)), f"fused layer, round {rep}"
    dvdq.release_stream(s)


def test_a_released_stream_can_be_used_again():
    ops = _operands(3000, 256, 1024, 4, True, seed=31)
    dvdq.bench_set_gemm_schedule(0)
    ref = _gemm(ops, 4, True)
    dvdq.bench_set_gemm_schedule(-1)
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream() for _ in range(3)]
    for rep in range(3):
        for s in streams:
            with torch.cuda.stream(s):
                y = _gemm(ops, 4, True, stream=s)
            s.synchronize()
            assert torch.equal(y.view(torch.int16), ref.view(torch.int16))
            dvdq.release_stream(s)
            dvdq.release_stream(s)   # unknown by now: no-op

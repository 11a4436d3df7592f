"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element
by element, on the same seeded inputs.  Bars are the ones stated in tests/parity.py.
Small cases span several tiles and ragged tails; the full-size cases live in
test_gpu_fullsize.py."""
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
    return t.detach().cpu().view(torch.int16).numpy().view(np.uint16)


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def rand_x(rng, M, K, outliers=True):
    x = rng.standard_normal((M, K)).astype(np.float32) * np.exp(rng.normal(0, 0.5, (M, 1))).astype(np.float32)
    if outliers and K >= 16:
        ch = rng.choice(K, size=max(1, K // 100), replace=False)
        x[:, ch] *= 50.0
    return di.f32_to_bf16_bits(x)


# ------------------------------------------------------------------ rotate + quantize
def run_rq(xb, B, bits, label):
    codes_g, scale_g = dvdq.rotate_quant(to_bf16(xb), B, bits)
    torch.cuda.synchronize()
    codes_r, scale_r, xr = oracle.rotate_quant(xb, B, bits, return_rotated=True)
    # blocks of 1 to 8 channels leave bf16 inputs (nearly) unmixed: exact ties at fp32 resolution come in clusters
    return check_codes_and_scales(codes_g.cpu().numpy(), scale_g.cpu().numpy(), codes_r, scale_r, xr, bits, label,
                                  allow_fp32_ties=B <= 8)


def test_rotate_quant_tiny_config():
    wl = di.WORKLOADS[0]
    stats = run_rq(di.make_x(wl), wl.had_block, wl.act_bits, wl.name)
    print(stats)


@pytest.mark.parametrize("M,K,B,bits", [
    (1, 8, 1, 4), (3, 8, 8, 4), (5, 64, 2, 6), (5, 64, 4, 8), (7, 96, 32, 4), (9, 128, 128, 6),
    (130, 256, 256, 4), (33, 768, 256, 4), (257, 1536, 256, 6), (65, 1536, 256, 8), (64, 3072, 256, 4),
    (31, 512, 512, 4), (19, 1024, 512, 6), (6, 13824, 512, 4), (5, 4096, 256, 4), (3, 16384, 512, 8),
    (17, 264, 8, 4), (12, 1280, 256, 4), (4, 65536, 512, 4), (4, 2560, 64, 4), (1027, 1536, 256, 4),
])
def test_rotate_quant_shapes(M, K, B, bits):
    rng = np.random.default_rng(M * 131 + K + B + bits)
    stats = run_rq(rand_x(rng, M, K), B, bits, f"M{M} K{K} B{B} b{bits}")
    assert stats["mismatches"] - stats.get("fp32_ties", 0) <= stats["budget"]


@pytest.mark.parametrize("bits,qmax", [(4, 7), (6, 31), (8, 127)])
def test_rotate_quant_on_grid_is_bit_exact(bits, qmax):
    """No rotation, values c * 2^p with some |c| = qmax: codes == c and scale == 2^p exactly."""
    rng = np.random.default_rng(bits)
    M, K = 37, 1024
    c = rng.integers(-qmax, qmax + 1, size=(M, K))
    c[:, 11] = qmax * rng.choice([-1, 1], size=M)
    p = rng.integers(-6, 6, size=M)
    xb = di.f32_to_bf16_bits((c * (2.0 ** p)[:, None]).astype(np.float32))
    codes, scale = dvdq.rotate_quant(to_bf16(xb), 1, bits)
    assert np.array_equal(codes.cpu().numpy(), c.astype(np.int8))
    assert np.array_equal(scale.cpu().numpy(), (2.0 ** p).astype(np.float32))


def test_rotate_quant_ties_go_to_even_and_zero_rows():
    row = np.array([7, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.5, -3.5, 6.5, 0, 0, 0, 0, 0, 0], dtype=np.float32) * 0.25
    x = np.zeros((3, 16), dtype=np.float32)
    x[0] = row
    x[2] = -row
    codes, scale = dvdq.rotate_quant(to_bf16(di.f32_to_bf16_bits(x)), 1, 4)
    codes, scale = codes.cpu().numpy(), scale.cpu().numpy()
    expect = np.array([7, 0, 2, 2, 0, -2, -2, 4, -4, 6, 0, 0, 0, 0, 0, 0], dtype=np.int8)
    assert np.array_equal(codes[0], expect) and np.array_equal(codes[2], -expect)
    assert not codes[1].any() and scale[1] == 0.0 and scale[0] == 0.25


def test_rotate_quant_hadamard_structure_exact():
    """Impulses and constants have exactly representable transforms: codes are +-qmax patterns
    of the natural-order Hadamard rows, bit-exact."""
    B = 256
    X = np.zeros((4, 512), dtype=np.float32)
    X[0, 3] = 1.0            # impulse in block 0 -> row 3 of H in block 0, zeros in block 1
    X[1, 256 + 77] = -2.0    # impulse in block 1
    X[2, :256] = 1.0         # constant -> sqrt(B) e_0
    X[3, 5] = 1.0
    X[3, 300] = 1.0
    xb = di.f32_to_bf16_bits(X)
    codes_g, scale_g = dvdq.rotate_quant(to_bf16(xb), B, 4)
    codes_r, scale_r = oracle.rotate_quant(xb, B, 4)
    assert np.array_equal(codes_g.cpu().numpy(), codes_r)
    assert np.array_equal(scale_g.cpu().numpy(), scale_r)


# ------------------------------------------------------------------ GEMM
def rand_gemm_inputs(rng, M, N, K, bits):
    qmax = 2 ** (bits - 1) - 1
    codes = rng.integers(-qmax, qmax + 1, size=(M, K)).astype(np.int8)
    wc = rng.integers(-7, 8, size=(N, K)).astype(np.int8)
    xs = np.exp(rng.normal(-2, 1, M)).astype(np.float32)
    ws = np.exp(rng.normal(-5, 0.5, N)).astype(np.float32)
    return codes, wc, xs, ws


@pytest.mark.parametrize("M,N,K,bits,layout,use_bias", [
    (128, 256, 256, 4, "canonical", False),
    (128, 256, 256, 4, "native", True),
    (1, 1, 64, 4, "canonical", False),
    (37, 50, 128, 6, "canonical", True),       # N % 4 != 0: scalar store path
    (300, 520, 384, 8, "native", False),       # ragged in M and N, several tiles
    (300, 520, 192, 8, "canonical", False),    # K not a multiple of 128: canonical layout only
    (513, 260, 1536, 4, "native", True),
    (256, 768, 13824, 4, "native", False),     # deepest K of the workloads
    (70, 300, 704, 8, "canonical", True),
    (90, 130, 32, 4, "canonical", False),      # K multiples of 32 that are not multiples of 64: half a last slice
    (200, 260, 96, 6, "canonical", True),
    (33, 513, 1120, 8, "canonical", False),
])
def test_gemm_int32_exact_and_bf16_epilogue(M, N, K, bits, layout, use_bias):
    rng = np.random.default_rng(M + 7 * N + 13 * K + bits)
    codes, wc, xs, ws = rand_gemm_inputs(rng, M, N, K, bits)
    wp = di.pack_w4(wc)
    bias = di.f32_to_bf16_bits(rng.standard_normal(N).astype(np.float32)) if use_bias else None
    w_dev = dev(wp)
    lay = dvdq.W_CANONICAL
    if layout == "native":
        w_dev = dvdq.w4_prepack(w_dev)
        lay = dvdq.W_NATIVE
    y, acc = dvdq.w4ax_gemm(dev(codes), dev(xs), w_dev, dev(ws), bits, lay,
                            bias=None if bias is None else to_bf16(bias), want_acc=True)
    torch.cuda.synchronize()
    y_ref, acc_ref = oracle.w4ax_gemm(codes, xs, wp, ws, bias, return_acc=True)
    assert np.array_equal(acc.cpu().numpy().astype(np.int64), acc_ref), "int32 accumulators must be bit-exact"
    stats = check_y(bits_of(y), y_ref, f"gemm M{M} N{N} K{K}", bias)
    # without the parity hook the outputs are the same
    y2 = dvdq.w4ax_gemm(dev(codes), dev(xs), w_dev, dev(ws), bits, lay, bias=None if bias is None else to_bf16(bias))
    assert torch.equal(y2, y)
    print(stats)


def test_gemm_extreme_codes_and_one_hot_weights():
    """Closed forms: saturated operands pin the accumulator width and the -8 nibble;
    one-hot weight rows pin the nibble order and sign extension of both layouts."""
    M, N, K = 64, 64, 13824
    codes = np.full((M, K), 127, dtype=np.int8)
    wc = np.full((N, K), -8, dtype=np.int8)
    wc[1::2] = 7
    ones_m, ones_n = np.ones(M, np.float32), np.ones(N, np.float32)
    for lay in (dvdq.W_CANONICAL, dvdq.W_NATIVE):
        w_dev = dev(di.pack_w4(wc))
        if lay == dvdq.W_NATIVE:
            w_dev = dvdq.w4_prepack(w_dev)
        _, acc = dvdq.w4ax_gemm(dev(codes), dev(ones_m), w_dev, dev(ones_n), 8, lay, want_acc=True)
        acc = acc.cpu().numpy()
        assert np.all(acc[:, 0::2] == -8 * 127 * K) and np.all(acc[:, 1::2] == 7 * 127 * K)
    # the longest contraction the accumulator bound admits for 8-bit codes (16 * 127 * 8 * K < 2^31)
    M, N, K = 40, 72, 131072
    codes = np.full((M, K), 127, dtype=np.int8)
    codes[1::2] = -127
    wc = np.full((N, K), -8, dtype=np.int8)
    wc[1::2] = 7
    w_dev = dvdq.w4_prepack(dev(di.pack_w4(wc)))
    _, acc = dvdq.w4ax_gemm(dev(codes), dev(np.ones(M, np.float32)), w_dev, dev(np.ones(N, np.float32)), 8, dvdq.W_NATIVE,
                            want_acc=True)
    expect = np.outer(np.where(np.arange(M) % 2 == 0, 127, -127), np.where(np.arange(N) % 2 == 0, -8, 7)).astype(np.int64) * K
    assert np.array_equal(acc.cpu().numpy().astype(np.int64), expect)
    rng = np.random.default_rng(3)
    K = 256
    q = rng.integers(-31, 32, size=(40, K)).astype(np.int8)
    k0 = rng.permutation(K)[:96]
    w1 = np.zeros((96, K), dtype=np.int8)
    w1[np.arange(96), k0] = np.where(np.arange(96) % 2 == 0, 1, -1)
    for lay in (dvdq.W_CANONICAL, dvdq.W_NATIVE):
        w_dev = dev(di.pack_w4(w1))
        if lay == dvdq.W_NATIVE:
            w_dev = dvdq.w4_prepack(w_dev)
        _, acc = dvdq.w4ax_gemm(dev(q), dev(np.ones(40, np.float32)), w_dev, dev(np.ones(96, np.float32)), 6, lay,
                                want_acc=True)
        expect = q[:, k0].astype(np.int32) * np.where(np.arange(96) % 2 == 0, 1, -1)[None, :]
        assert np.array_equal(acc.cpu().numpy(), expect)


# ------------------------------------------------------------------ the whole layer
@pytest.mark.parametrize("idx", [0])
def test_qlinear_tiny_config_compositional(idx):
    """codes / scales from the workspace against the oracle (flip budget); Y against the
    oracle's GEMM + epilogue applied to the GPU's own codes and scales (1 bf16 ulp);
    and the fused call equals the two separate calls bit for bit."""
    wl = di.WORKLOADS[idx]
    xb = di.make_x(wl)
    wp, ws, _ = di.make_weights(wl)
    x_dev, w_dev, ws_dev = to_bf16(xb), dev(wp), dev(ws)
    for lay in (dvdq.W_CANONICAL, dvdq.W_NATIVE):
        wd = dvdq.w4_prepack(w_dev) if lay == dvdq.W_NATIVE else w_dev
        y, wsp = dvdq.qlinear(x_dev, wd, ws_dev, wl.had_block, wl.act_bits, lay)
        torch.cuda.synchronize()
        codes_g, scale_g = dvdq.workspace_views(wsp, wl.M, wl.K)
        codes_g, scale_g = codes_g.cpu().numpy(), scale_g.cpu().numpy()
        ref = oracle.qlinear(xb, wp, ws, wl.had_block, wl.act_bits)
        xr = oracle.rotate(xb, wl.had_block)
        check_codes_and_scales(codes_g, scale_g, ref["codes"], ref["x_scale"], xr, wl.act_bits, wl.name)
        y_ref = oracle.w4ax_gemm(codes_g, scale_g, wp, ws)
        check_y(bits_of(y), y_ref, wl.name)
        c2, s2 = dvdq.rotate_quant(x_dev, wl.had_block, wl.act_bits)
        y2 = dvdq.w4ax_gemm(c2, s2, wd, ws_dev, wl.act_bits, lay)
        assert torch.equal(y2, y)
        if np.array_equal(codes_g, ref["codes"]) and np.array_equal(scale_g, ref["x_scale"]):
            check_y(bits_of(y), ref["y"], wl.name + " direct")


@pytest.mark.parametrize("M,K,N,B,bits", [(77, 96, 130, 32, 4), (300, 1120, 200, 32, 6), (64, 160, 64, 1, 8)])
def test_qlinear_with_k_a_multiple_of_32_only(M, K, N, B, bits):
    """the whole layer where K is no multiple of 64 (weights in the canonical layout): as above"""
    rng = np.random.default_rng(M + K + N)
    xb = rand_x(rng, M, K)
    _, wc, _, ws = rand_gemm_inputs(rng, M, N, K, bits)
    wp = di.pack_w4(wc)
    x_dev, w_dev, ws_dev = to_bf16(xb), dev(wp), dev(ws)
    y, wsp = dvdq.qlinear(x_dev, w_dev, ws_dev, B, bits, dvdq.W_CANONICAL)
    torch.cuda.synchronize()
    codes_g, scale_g = dvdq.workspace_views(wsp, M, K)
    codes_g, scale_g = codes_g.cpu().numpy(), scale_g.cpu().numpy()
    ref = oracle.qlinear(xb, wp, ws, B, bits)
    check_codes_and_scales(codes_g, scale_g, ref["codes"], ref["x_scale"], oracle.rotate(xb, B), bits, f"K{K}",
                           allow_fp32_ties=B <= 8)
    check_y(bits_of(y), oracle.w4ax_gemm(codes_g, scale_g, wp, ws), f"K{K}")

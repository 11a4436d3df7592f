"""GPU parity of the packed 4-bit activation-code container (two codes per byte between
the quantizer and the GEMM).  It is an encoding, so the bar is bit-exactness: the packed
bytes decode (with the oracle's decoder) to the very codes the int8 container holds, the
accumulators equal the oracle's integer GEMM, and outputs equal the int8 path bit for bit."""
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


def rand_x(rng, M, K):
    x = rng.standard_normal((M, K)).astype(np.float32) * np.exp(rng.normal(0, 0.5, (M, 1))).astype(np.float32)
    if K >= 16:
        x[:, rng.choice(K, size=max(1, K // 100), replace=False)] *= 50.0
    return di.f32_to_bf16_bits(x)


@pytest.mark.parametrize("M,K,B", [
    (1, 8, 1), (3, 8, 8), (7, 96, 32), (130, 256, 256), (33, 768, 256), (257, 1536, 256), (64, 3072, 256),
    (31, 512, 512), (6, 13824, 512), (17, 264, 8), (4, 65536, 512), (1027, 1536, 256),
])
def test_rotate_quant_packed_decodes_to_the_int8_codes(M, K, B):
    rng = np.random.default_rng(M * 17 + K + B)
    xb = rand_x(rng, M, K)
    x_dev = to_bf16(xb)
    packed, scale_p = dvdq.rotate_quant(x_dev, B, 4, codes_format=dvdq.CODES_PACKED4)
    codes8, scale8 = dvdq.rotate_quant(x_dev, B, 4)
    torch.cuda.synchronize()
    assert packed.dtype == torch.uint8 and tuple(packed.shape) == (M, K // 2)
    decoded = oracle.unpack_a4(packed.cpu().numpy())
    assert np.array_equal(decoded, codes8.cpu().numpy()), "both containers must carry the same codes"
    assert torch.equal(scale_p, scale8)
    codes_r, scale_r, xr = oracle.rotate_quant(xb, B, 4, return_rotated=True)
    check_codes_and_scales(decoded, scale_p.cpu().numpy(), codes_r, scale_r, xr, 4, f"packed M{M} K{K} B{B}",
                           allow_fp32_ties=B <= 8)


def test_rotate_quant_packed_leaves_neighbouring_memory_alone():
    """the packed store writes exactly M*K/2 bytes"""
    M, K = 5, 1536
    buf = torch.full((M * K // 2 + 512,), 0xA5, dtype=torch.uint8, device=DEV)
    codes = buf[256:256 + M * K // 2].view(M, K // 2)
    xb = rand_x(np.random.default_rng(5), M, K)
    dvdq.rotate_quant(to_bf16(xb), 256, 4, codes=codes, codes_format=dvdq.CODES_PACKED4)
    torch.cuda.synchronize()
    assert bool((buf[:256] == 0xA5).all()) and bool((buf[256 + M * K // 2:] == 0xA5).all())


def gemm_case(rng, M, N, K, full_range=False):
    lo = -8 if full_range else -7
    codes = rng.integers(lo, 8, size=(M, K)).astype(np.int8)
    wc = rng.integers(-8, 8, size=(N, K)).astype(np.int8)
    xs = np.exp(rng.normal(-2, 1, M)).astype(np.float32)
    ws = np.exp(rng.normal(-5, 0.5, N)).astype(np.float32)
    return codes, wc, xs, ws


@pytest.mark.parametrize("variant", [-1, 1, 2, 3, 4])
@pytest.mark.parametrize("M,N,K,use_bias", [
    (1, 1, 128, False),          # one K slice: the shallow-K fallback
    (128, 256, 256, True),
    (300, 520, 384, False),      # ragged in M and N; exactly 3 K slices (deepest ring's minimum)
    (513, 260, 1536, True),
    (37, 50, 512, True),         # N % 8 != 0: scalar store path
    (256, 768, 13824, False),    # deepest K of the workloads
])
def test_gemm_packed_codes_int32_exact(M, N, K, use_bias, variant):
    rng = np.random.default_rng(M + 7 * N + 13 * K)
    codes, wc, xs, ws = gemm_case(rng, M, N, K, full_range=(M == 300))
    wp = di.pack_w4(wc)
    bias = di.f32_to_bf16_bits(rng.standard_normal(N).astype(np.float32)) if use_bias else None
    bias_dev = None if bias is None else to_bf16(bias)
    w_native = dvdq.w4_prepack(dev(wp))
    packed = dev(oracle.pack_a4(codes))
    dvdq.bench_set_gemm_variant(variant)
    try:
        y, acc = dvdq.w4ax_gemm(packed, dev(xs), w_native, dev(ws), 4, dvdq.W_NATIVE, bias=bias_dev, want_acc=True,
                                codes_format=dvdq.CODES_PACKED4)
        y2 = dvdq.w4ax_gemm(packed, dev(xs), w_native, dev(ws), 4, dvdq.W_NATIVE, bias=bias_dev,
                            codes_format=dvdq.CODES_PACKED4)
        torch.cuda.synchronize()
    finally:
        dvdq.bench_set_gemm_variant(-1)
    y_ref, acc_ref = oracle.w4ax_gemm(codes, xs, wp, ws, bias, return_acc=True)
    assert np.array_equal(acc.cpu().numpy().astype(np.int64), acc_ref), "int32 accumulators must be bit-exact"
    check_y(bits_of(y), y_ref, f"packed gemm M{M} N{N} K{K} v{variant}", bias)
    assert torch.equal(y2, y)
    y8 = dvdq.w4ax_gemm(dev(codes), dev(xs), w_native, dev(ws), 4, dvdq.W_NATIVE, bias=bias_dev)
    assert torch.equal(y8, y), "the container must not change the outputs"


@pytest.mark.parametrize("idx", [0, 1, 3, 4])
def test_qlinear_with_packed_codes_matches_the_int8_container(idx):
    wl = di.WORKLOADS[idx]
    M, K, N, B = wl.M, wl.K, wl.N, wl.had_block
    assert wl.act_bits == 4
    print(f"[{wl.name}] inputs", flush=True)
    xb = di.make_x(wl)
    wp, ws, _ = di.make_weights(wl)
    x_dev, ws_dev = to_bf16(xb), dev(ws)
    w_native = dvdq.w4_prepack(dev(wp))
    print(f"[{wl.name}] qlinear packed M={M} K={K} N={N}", flush=True)
    y, wsp = dvdq.qlinear(x_dev, w_native, ws_dev, B, 4, dvdq.W_NATIVE, codes_format=dvdq.CODES_PACKED4)
    y8, wsp8 = dvdq.qlinear(x_dev, w_native, ws_dev, B, 4, dvdq.W_NATIVE)
    torch.cuda.synchronize()
    assert wsp.numel() == dvdq.qlinear_workspace_bytes(M, K, dvdq.CODES_PACKED4) < wsp8.numel()
    assert torch.equal(y, y8)
    packed, scale = dvdq.workspace_views(wsp, M, K, dvdq.CODES_PACKED4)
    codes8, scale8 = dvdq.workspace_views(wsp8, M, K)
    assert torch.equal(scale, scale8)
    rows = di.sample_rows(M, 128)
    rows_t = torch.from_numpy(rows).to(DEV)
    decoded = oracle.unpack_a4(packed[rows_t].cpu().numpy())
    assert np.array_equal(decoded, codes8[rows_t].cpu().numpy())
    # and against the oracle, on the row sample
    xs_rows = np.ascontiguousarray(xb[rows])
    codes_r, scale_r, xr = oracle.rotate_quant(xs_rows, B, 4, return_rotated=True)
    scale_g = scale[rows_t].cpu().numpy()
    check_codes_and_scales(decoded, scale_g, codes_r, scale_r, xr, 4, wl.name + " packed")
    y_ref = oracle.w4ax_gemm(decoded, scale_g, wp, ws)
    check_y(bits_of(y[rows_t]), y_ref, wl.name + " packed")

"""GPU parity of the block-wise scaled quantizer (power-of-two group steps folded into int8 values)
and of the layer built on it.  Bars as stated in parity.check_blockwise."""
import numpy as np
import pytest
import torch

import dvdq_inputs as di
import oracle
import paper_2505_18663_amd as dvdq
from parity import check_blockwise, check_y

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def to_bf16(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).to(DEV)


def bits_of(t):
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def rand_x(rng, M, K):
    """tokens with loud and quiet stretches of channels, outlier channels, and a spread of token scales"""
    x = rng.standard_normal((M, K)).astype(np.float32) * np.exp(rng.normal(0, 0.5, (M, 1))).astype(np.float32)
    prof = np.exp(rng.normal(0, 1.2, (1, max(1, K // 128)))).astype(np.float32).repeat(128, axis=1)[:, :K]
    x *= prof
    x[:, rng.choice(K, size=max(1, K // 100), replace=False)] *= 30.0
    return di.f32_to_bf16_bits(x)


@pytest.mark.parametrize("M,K,B,bits,group", [
    (128, 256, 256, 4, 128), (130, 512, 256, 4, 256), (33, 1536, 256, 4, 512), (257, 1536, 256, 4, 128),
    (65, 1536, 256, 6, 128), (64, 3072, 256, 4, 256), (31, 1024, 512, 4, 128), (6, 13824, 512, 4, 512),
    (6, 13824, 512, 6, 128), (5, 4096, 64, 4, 128), (3, 1280, 256, 4, 128), (1027, 1536, 256, 4, 256),
    (4, 65536, 512, 4, 512),
])
def test_blockwise_quantizer_matches_the_oracle(M, K, B, bits, group):
    rng = np.random.default_rng(M * 31 + K + bits + group)
    xb = rand_x(rng, M, K)
    values, scale, rs = dvdq.rotate_quant_blockwise(to_bf16(xb), B, bits, group, want_rowsum=True)
    torch.cuda.synchronize()
    xr = oracle.rotate(xb, B)
    v_ref, s_ref, e_ref = oracle.quantize_blockwise(xr, bits, group)
    vg = values.cpu().numpy()
    stats = check_blockwise(vg, scale.cpu().numpy(), v_ref, s_ref, e_ref, xr, bits, group, f"M{M} K{K} B{B} b{bits} g{group}")
    if K >= 4 * B:   # (within one Hadamard block the rotation evens the groups out)
        assert e_ref.max() > 0, "the inputs must exercise finer group steps"
    assert np.array_equal(rs.cpu().numpy().astype(np.int64), vg.astype(np.int64).sum(axis=1))
    print(stats)


def test_blockwise_layer_is_closer_to_the_float_layer():
    """quantizer (block-wise) + GEMM (act_bits = 8 on the int8 values): outputs equal the oracle's GEMM on
    the GPU's own values, and the layer error against the float layer drops below the per-token one."""
    M, K, N, B = 192, 1536, 320, 256          # six Hadamard blocks of unequal energy
    rng = np.random.default_rng(21)
    xb = rand_x(rng, M, K)
    wc = rng.integers(-7, 8, (N, K)).astype(np.int8)
    ws = np.exp(rng.normal(-5, 0.3, N)).astype(np.float32)
    wp = di.pack_w4(wc)
    x_dev, ws_dev = to_bf16(xb), dev(ws)
    w_native = dvdq.w4_prepack(dev(wp))
    values, scale = dvdq.rotate_quant_blockwise(x_dev, B, 4, 128)
    y = dvdq.w4ax_gemm(values, scale, w_native, ws_dev, 8, dvdq.W_NATIVE)
    y_tok, _ = dvdq.qlinear(x_dev, w_native, ws_dev, B, 4, dvdq.W_NATIVE)
    torch.cuda.synchronize()
    y_ref = oracle.w4ax_gemm(values.cpu().numpy(), scale.cpu().numpy(), wp, ws)
    check_y(bits_of(y), y_ref, "blockwise layer")
    w_deq = wc.astype(np.float64) * ws.astype(np.float64)[:, None]
    y_float = oracle.rotate(xb, B) @ w_deq.T
    err_blk = np.linalg.norm(y.float().cpu().numpy().astype(np.float64) - y_float)
    err_tok = np.linalg.norm(y_tok.float().cpu().numpy().astype(np.float64) - y_float)
    print(dict(err_blockwise=err_blk, err_per_token=err_tok))
    assert err_blk < err_tok

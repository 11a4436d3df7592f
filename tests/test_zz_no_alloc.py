"""dvdq_qlinear_static (the entry point for callers that cannot allocate: the library's own fixed
workspace) against dvdq_qlinear with a caller workspace, through the C ABI.  Same kernels, so the
outputs must be bit-identical; two calls in a row, the second with a smaller input (the array keeps
the first call's contents)."""
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


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def make_case(seed, M, K, N):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((M, K)).astype(np.float32) * np.exp(rng.normal(0, 0.5, (M, 1))).astype(np.float32)
    x[:, rng.choice(K, size=max(1, K // 100), replace=False)] *= 50.0
    wc = rng.integers(-7, 8, (N, K)).astype(np.int8)
    ws = np.exp(rng.normal(-4, 0.3, N)).astype(np.float32)
    return di.f32_to_bf16_bits(x), oracle.pack_w4(wc), ws


@pytest.mark.parametrize("container", ["int8", "packed4", "fp6"])
def test_static_workspace_matches_caller_workspace_on_two_calls_in_a_row(container):
    fmt, layout, prepack = {
        "int8": (dvdq.CODES_INT8, dvdq.W_NATIVE, dvdq.w4_prepack),
        "packed4": (dvdq.CODES_PACKED4, dvdq.W_NATIVE, dvdq.w4_prepack),
        "fp6": (dvdq.CODES_FP6, dvdq.W_NATIVE_FP6, dvdq.w4_prepack_fp6),
    }[container]
    B, bits = 256, 4
    for call, (M, K, N) in enumerate([(1000, 1536, 520), (130, 768, 264)]):   # the second is smaller
        print(f"static workspace, {container}, call {call}: M{M} K{K} N{N}", flush=True)
        xb, wp, ws = make_case(100 + call, M, K, N)
        x_dev, w_dev, ws_dev = to_bf16(xb), prepack(dev(wp)), dev(ws)
        y_ref, wsp = dvdq.qlinear(x_dev, w_dev, ws_dev, B, bits, layout, codes_format=fmt)
        y = torch.empty_like(y_ref)
        out = dvdq.qlinear_static(x_dev, w_dev, ws_dev, B, bits, layout, y=y, codes_format=fmt)
        torch.cuda.synchronize()
        assert out is y and torch.equal(y, y_ref), "outputs differ from the caller-workspace entry point"
        if container == "int8":   # and, once, straight against the oracle on the GPU's own codes and scales
            codes, scale = dvdq.workspace_views(wsp, M, K)
            y_or = oracle.w4ax_gemm(codes.cpu().numpy(), scale.cpu().numpy(), wp, ws)
            check_y(y.cpu().contiguous().view(torch.int16).numpy().view(np.uint16), y_or, f"static call {call}")


def test_static_workspace_with_zero_points_and_bias():
    M, K, N, B = 300, 512, 264, 256
    rng = np.random.default_rng(7)
    xb, wp, ws = make_case(7, M, K, N)
    wz = dev(rng.integers(-8, 8, N).astype(np.int8))
    bias = torch.from_numpy(rng.standard_normal(N).astype(np.float32)).to(DEV).to(torch.bfloat16)
    x_dev, w_dev, ws_dev = to_bf16(xb), dvdq.w4_prepack(dev(wp)), dev(ws)
    y_ref, _ = dvdq.qlinear(x_dev, w_dev, ws_dev, B, 6, dvdq.W_NATIVE, bias=bias, w_zero=wz)
    y = dvdq.qlinear_static(x_dev, w_dev, ws_dev, B, 6, dvdq.W_NATIVE, bias=bias, w_zero=wz)
    torch.cuda.synchronize()
    assert torch.equal(y, y_ref)


def test_static_workspace_rejects_requests_beyond_its_size():
    cap = dvdq.static_workspace_bytes()
    assert cap == 64 << 20
    L = dvdq.lib()
    K = 4096
    M = cap // K + 1                     # int8 container: M * K bytes of codes alone exceed the array
    assert dvdq.qlinear_workspace_bytes(M, K) > cap
    x = torch.zeros((8, K), dtype=torch.bfloat16, device=DEV)     # never read: the call must fail on the host
    w = torch.zeros((256 * K // 2,), dtype=torch.uint8, device=DEV)
    ws = torch.ones((8,), dtype=torch.float32, device=DEV)
    y = torch.zeros((8, 8), dtype=torch.bfloat16, device=DEV)
    rc = L.dvdq_qlinear_static(x.data_ptr(), w.data_ptr(), ws.data_ptr(), None, None, M, 8, K, 256, 4, 0, 1,
                               y.data_ptr(), None)
    assert rc == 4, dvdq.status_string(rc)
    torch.cuda.synchronize()

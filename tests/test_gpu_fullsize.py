"""GPU parity at the full workload sizes through dvdq_qlinear with the native weight layout,
int8 code container, INT8 matrix path (the configuration the benchmark times for W4A6; the
W4A4 workloads on the FP6 matrix path, which the benchmark times for them, are checked at
full size in test_gpu_fp6.py).  The oracle cannot afford all M rows, so it
judges a deterministic row sample (first 256 + last 256 rows, which covers the ragged
last tile, plus 64 rows from the middle); properties that hold at any size are
checked on every row on the GPU."""
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


def sampled_rows(M):
    head_tail = di.sample_rows(M, 256)
    if M <= 512:
        return head_tail
    mid = np.random.default_rng(M).choice(np.arange(256, M - 256), size=64, replace=False)
    return np.unique(np.concatenate([head_tail, mid]))


@pytest.mark.parametrize("idx", [1, 2, 3, 4])
def test_full_size_workload(idx):
    wl = di.WORKLOADS[idx]
    M, K, N, B, bits = wl.M, wl.K, wl.N, wl.had_block, wl.act_bits
    qmax = 2 ** (bits - 1) - 1
    print(f"[{wl.name}] generating inputs", flush=True)
    xb = di.make_x(wl)
    wp, ws, _ = di.make_weights(wl)
    x_dev = to_bf16(xb)
    w_native = dvdq.w4_prepack(torch.from_numpy(wp).to(DEV))
    ws_dev = torch.from_numpy(ws).to(DEV)

    print(f"[{wl.name}] dvdq_qlinear M={M} K={K} N={N}", flush=True)
    y, wsp = dvdq.qlinear(x_dev, w_native, ws_dev, B, bits, dvdq.W_NATIVE)
    torch.cuda.synchronize()
    codes_dev, scale_dev = dvdq.workspace_views(wsp, M, K)

    # ---- properties on every row (GPU side, cheap)
    row_max = codes_dev.abs().amax(dim=1)
    assert bool(((row_max == qmax) | ((row_max == 0) & (scale_dev == 0))).all()), "a row does not reach +-qmax"
    assert bool((codes_dev.abs() <= qmax).all())
    assert bool(torch.isfinite(scale_dev).all()) and bool((scale_dev >= 0).all())
    assert bool(torch.isfinite(y.float()).all())

    # ---- oracle on the row sample: codes / scales (flip budget), then accumulators and outputs
    rows = sampled_rows(M)
    rows_t = torch.from_numpy(rows).to(DEV)
    xs_rows = np.ascontiguousarray(xb[rows])
    print(f"[{wl.name}] oracle rotate+quantize on {rows.size} rows", flush=True)
    codes_ref, scale_ref, xr = oracle.rotate_quant(xs_rows, B, bits, return_rotated=True)
    codes_g = codes_dev[rows_t].cpu().numpy()
    scale_g = scale_dev[rows_t].cpu().numpy()
    stats = check_codes_and_scales(codes_g, scale_g, codes_ref, scale_ref, xr, bits, wl.name)
    print(f"[{wl.name}] codes: {stats}", flush=True)

    # accumulators through the parity hook at full size, compared on the sample
    _, acc = dvdq.w4ax_gemm(codes_dev, scale_dev, w_native, ws_dev, bits, dvdq.W_NATIVE, want_acc=True)
    torch.cuda.synchronize()
    acc_g = acc[rows_t].cpu().numpy()
    del acc
    print(f"[{wl.name}] oracle int GEMM + epilogue on the sample", flush=True)
    y_ref, acc_ref = oracle.w4ax_gemm(codes_g, scale_g, wp, ws, return_acc=True)
    assert np.array_equal(acc_g.astype(np.int64), acc_ref), "int32 accumulators must be bit-exact"
    ystats = check_y(bits_of(y[rows_t]), y_ref, wl.name)
    print(f"[{wl.name}] outputs: {ystats}", flush=True)

    # the fused call and the accumulator-hook call write the same outputs
    y2 = dvdq.w4ax_gemm(codes_dev, scale_dev, w_native, ws_dev, bits, dvdq.W_NATIVE)
    assert torch.equal(y2, y)


def test_rotate_quant_every_row_of_the_headline_workload():
    """codes and scales of all 32760 rows of the QKV workload against the oracle."""
    wl = di.WORKLOADS[1]
    xb = di.make_x(wl)
    codes_g, scale_g = dvdq.rotate_quant(to_bf16(xb), wl.had_block, wl.act_bits)
    torch.cuda.synchronize()
    codes_g, scale_g = codes_g.cpu().numpy(), scale_g.cpu().numpy()
    step = 4096                                    # bound the fp64 copy of the rotated rows
    total = dict(mismatches=0, elements=0, max_scale_ulp=0, max_boundary_dist_ulps=0.0)
    for r0 in range(0, wl.M, step):
        sl = slice(r0, min(wl.M, r0 + step))
        codes_ref, scale_ref, xr = oracle.rotate_quant(xb[sl], wl.had_block, wl.act_bits, return_rotated=True)
        st = check_codes_and_scales(codes_g[sl], scale_g[sl], codes_ref, scale_ref, xr, wl.act_bits, f"rows {r0}+")
        total["mismatches"] += st["mismatches"]
        total["elements"] += st["elements"]
        total["max_scale_ulp"] = max(total["max_scale_ulp"], st["max_scale_ulp"])
        total["max_boundary_dist_ulps"] = max(total["max_boundary_dist_ulps"], st["max_boundary_dist_ulps"])
    print(total)
    assert total["mismatches"] <= 1e-5 * total["elements"]

"""GPU parity of the offline weight quantizer (Bounded-init Grid Refinement, Sec. 3.1 / Alg. 1)
against the oracle.  Both sides compute in fp64 and differ only in summation order, so grids
and codes are expected to be identical; a row may differ only if the two searches tie to
within rounding, in which case its error must still equal the oracle's (budget below)."""
import numpy as np
import pytest
import torch

import dvdq_inputs as di
import oracle
import paper_2505_18663_amd as dvdq
from parity import check_y

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def gpu_bgr(w, **kw):
    wp, ws, wz, err = dvdq.bgr_quantize(dev(w), want_error=True, **kw)
    torch.cuda.synchronize()
    q = oracle.unpack_w4(wp.cpu().numpy()).astype(np.int16) + 8          # back to the unsigned codes 0..15
    return q.astype(np.uint8), ws.cpu().numpy(), wz.cpu().numpy().astype(np.int32) + 8, err.cpu().numpy()


def compare(w, label, **kw):
    q_g, d_g, z_g, e_g = gpu_bgr(w, **kw)
    q_r, d_r, z_r, e_r = oracle.bgr(w, **kw)
    same = (z_g == z_r) & (d_g == d_r.astype(np.float32)) & np.all(q_g == q_r, axis=1)
    # errors agree to fp64 summation-order noise on every row, identical grid or not
    assert np.all(np.abs(e_g - e_r) <= 1e-9 * np.maximum(e_r, 1e-300)), f"{label}: row errors differ"
    budget = int(np.ceil(0.005 * w.shape[0]))
    assert (~same).sum() <= budget, f"{label}: {(~same).sum()} rows with a different grid (budget {budget})"
    # whatever grid the GPU returned, its codes are the Quant equation on that grid (checked in fp64 here)
    q_expect = np.clip(np.rint(w.astype(np.float64) / d_r[:, None]) + z_g[:, None], 0, 15).astype(np.uint8)
    assert np.array_equal(q_g[same], q_expect[same])
    return dict(rows=w.shape[0], differing=int((~same).sum()), max_rel_err_diff=float(np.max(np.abs(e_g - e_r) / np.maximum(e_r, 1e-300))))


@pytest.mark.parametrize("N,K,kw", [
    (96, 64, {}), (96, 256, {}), (256, 1536, {}), (64, 3072, {}), (24, 13824, {}), (5, 32768, dict(n_steps=20)),
    (96, 1536, dict(n_steps=16, max_refine=0)), (96, 1536, dict(n_steps=40, max_refine=3)),
    (96, 1536, dict(eps=1e-4)), (7, 130, dict(n_steps=7, max_refine=2)),
    (96, 256, dict(search=1)), (128, 1536, dict(search=1)), (96, 1536, dict(search=1, n_steps=16, max_refine=0)),
    (96, 1536, dict(search=1, eps=1e-4)), (24, 13824, dict(search=1)),
])
def test_bgr_matches_the_oracle_on_gaussian_rows(N, K, kw):
    rng = np.random.default_rng(N * 7 + K)
    w = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    w[0] += 0.05                                   # not zero-mean
    w[1, :4] = [0.4, -0.5, 0.45, -0.38]            # outliers
    print(compare(w, f"N{N} K{K} {kw}", **kw))


def test_bgr_special_rows():
    rng = np.random.default_rng(1)
    K = 256
    rows = [np.zeros(K), np.full(K, 0.37), np.full(K, -2.5),                      # constant rows: exact
            0.125 * (rng.integers(0, 16, K) - 3.0),                              # already on a grid: exact
            rng.standard_normal(K) * 0.1 + 5.0,                                  # all positive: zero-point pinned at 0
            np.concatenate([[1.0], np.zeros(K - 1)]),                            # one spike
            rng.standard_t(3, K) * 0.02]                                         # heavy tails
    rows[3][:16] = 0.125 * (np.arange(16) - 3.0)
    w = np.stack(rows).astype(np.float32)
    # exact: constant rows in either search; the on-grid row where plain MinMax (i = 0) is a candidate
    for search, exact in ((dvdq.BGR_BEST_OF_ALL, 4), (dvdq.BGR_LISTING, 3)):
        q_g, d_g, z_g, e_g = gpu_bgr(w, search=search)
        q_r, d_r, z_r, e_r = oracle.bgr(w, search=search)
        assert np.array_equal(z_g, z_r) and np.array_equal(d_g, d_r.astype(np.float32)) and np.array_equal(q_g, q_r)
        assert np.allclose(e_g, e_r, rtol=1e-9, atol=0)
        assert np.all(e_g[:exact] == 0)
        deq = d_g[:exact, None].astype(np.float64) * (q_g[:exact].astype(np.float64) - z_g[:exact, None])
        assert np.array_equal(deq, w[:exact].astype(np.float64))


def test_bgr_weights_through_the_layer():
    """fp32 weights -> BGR on the GPU -> pre-pack -> the whole layer with zero-points; the outputs
    match the oracle's zero-point GEMM on the GPU's own codes, and the layer is closer to the
    float layer than with plain MinMax weights (what the quantizer is for)."""
    wl = di.WORKLOADS[0]
    M, K, N, B = wl.M, wl.K, wl.N, wl.had_block
    rng = np.random.default_rng(11)
    w = (rng.standard_t(5, (N, K)) * 0.02).astype(np.float32)
    xb = di.make_x(wl)
    x_dev = torch.from_numpy(xb.view(np.int16)).view(torch.bfloat16).to(DEV)
    wp, ws, wz = dvdq.bgr_quantize(dev(w))
    y, wsp = dvdq.qlinear(x_dev, dvdq.w4_prepack(wp), ws, B, 8, dvdq.W_NATIVE, w_zero=wz)
    torch.cuda.synchronize()
    codes, scale = dvdq.workspace_views(wsp, M, K)
    y_ref = oracle.w4ax_gemm_zp(codes.cpu().numpy(), scale.cpu().numpy(), wp.cpu().numpy(), ws.cpu().numpy(),
                                wz.cpu().numpy())
    check_y(y.cpu().contiguous().view(torch.int16).numpy().view(np.uint16), y_ref, "bgr layer")
    # against the float layer  (X H)(W)^T  with W taken as already rotated
    xr = oracle.rotate(xb, B)
    y_float = xr @ w.astype(np.float64).T
    q_mm, d_mm, z_mm, _ = oracle.minmax_quant(w)
    w_mm = d_mm[:, None] * (q_mm.astype(np.float64) - z_mm[:, None])
    err_bgr = np.linalg.norm(y.float().cpu().numpy().astype(np.float64) - y_float)
    err_mm = np.linalg.norm(xr @ w_mm.T - y_float)
    assert err_bgr < err_mm

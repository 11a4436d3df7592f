"""Randomized sweep of GEMM shapes (ragged and aligned), code containers, bit-widths, tile variants,
bias and weight zero-points against the oracle: int32 accumulators bit-exact, outputs to the bf16
bar, and the interior (staged) and predicated epilogues bit-identical."""
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


def to_bf16(bits):
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).view(torch.bfloat16).to(DEV)


def bits_of(t):
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_gemm_cases(seed):
    rng = np.random.default_rng(seed)
    for case in range(40):
        M = int(rng.choice([1, 7, 31, 64, 127, 128, 129, 255, 256, 257, 300, 511, 640, 1000]))
        N = int(rng.choice([1, 8, 24, 50, 64, 248, 256, 264, 300, 512, 520, 768, 1032]))
        K = int(rng.choice([128, 256, 384, 512, 1024, 2048]))
        bits = int(rng.choice([4, 6, 8]))
        packed = bool(bits == 4 and rng.random() < 0.5)
        use_bias, use_zero = bool(rng.random() < 0.5), bool(rng.random() < 0.4)
        variant = int(rng.choice([-1, -1, 1, 2, 3, 4]))
        label = f"seed {seed} case {case}: M{M} N{N} K{K} b{bits} packed={packed} bias={use_bias} zero={use_zero} v{variant}"
        print(label, flush=True)
        qmax = 2 ** (bits - 1) - 1
        codes = rng.integers(-qmax, qmax + 1, (M, K)).astype(np.int8)
        wc = rng.integers(-8, 8, (N, K)).astype(np.int8)
        xs = np.exp(rng.normal(-2, 1, M)).astype(np.float32)
        ws = np.exp(rng.normal(-5, 0.5, N)).astype(np.float32)
        bias = di.f32_to_bf16_bits(rng.standard_normal(N).astype(np.float32)) if use_bias else None
        wz = rng.integers(-8, 8, N).astype(np.int8) if use_zero else None
        wp = di.pack_w4(wc)
        w_native = dvdq.w4_prepack(dev(wp))
        fmt = dvdq.CODES_PACKED4 if packed else dvdq.CODES_INT8
        cd = dev(oracle.pack_a4(codes)) if packed else dev(codes)
        kw = dict(bias=None if bias is None else to_bf16(bias), codes_format=fmt)
        if use_zero:
            kw.update(w_zero=dev(wz), code_rowsum=dev(codes.astype(np.int32).sum(axis=1).astype(np.int32)))
        dvdq.bench_set_gemm_variant(variant)
        try:
            y, acc = dvdq.w4ax_gemm(cd, dev(xs), w_native, dev(ws), bits, dvdq.W_NATIVE, want_acc=True, **kw)
            y2 = dvdq.w4ax_gemm(cd, dev(xs), w_native, dev(ws), bits, dvdq.W_NATIVE, **kw)
            torch.cuda.synchronize()
        finally:
            dvdq.bench_set_gemm_variant(-1)
        if use_zero:
            y_ref, acc_ref = oracle.w4ax_gemm_zp(codes, xs, wp, ws, wz, bias, return_acc=True)
        else:
            y_ref, acc_ref = oracle.w4ax_gemm(codes, xs, wp, ws, bias, return_acc=True)
        assert np.array_equal(acc.cpu().numpy().astype(np.int64), acc_ref), label
        check_y(bits_of(y), y_ref, label, bias)
        assert torch.equal(y, y2), label + ": epilogue paths differ"

"""Randomized sweep of GEMM shapes (ragged and aligned), code containers (int8, packed nibbles, FP6
patterns on the FP6 matrix path), bit-widths, tile variants, bias and weight zero-points against the
oracle: int32 accumulators bit-exact, outputs to the bf16 bar, and the interior (staged) and predicated
epilogues bit-identical."""
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
        container = str(rng.choice(["int8", "packed4", "fp6"])) if bits == 4 else "int8"
        packed, fp6 = container == "packed4", container == "fp6"
        use_bias, use_zero = bool(rng.random() < 0.5), bool(rng.random() < 0.4)
        variant = int(rng.choice([-1, -1, 1, 2, 3, 4]))
        label = f"seed {seed} case {case}: M{M} N{N} K{K} b{bits} {container} bias={use_bias} zero={use_zero} v{variant}"
        print(label, flush=True)
        qmax = 2 ** (bits - 1) - 1
        codes = rng.integers(-qmax, qmax + 1, (M, K)).astype(np.int8)
        wc = rng.integers(-8, 8, (N, K)).astype(np.int8)
        xs = np.exp(rng.normal(-2, 1, M)).astype(np.float32)
        ws = np.exp(rng.normal(-5, 0.5, N)).astype(np.float32)
        bias = di.f32_to_bf16_bits(rng.standard_normal(N).astype(np.float32)) if use_bias else None
        wz = rng.integers(-8, 8, N).astype(np.int8) if use_zero else None
        wp = di.pack_w4(wc)
        if fp6:
            w_native, lay, fmt, cd = dvdq.w4_prepack_fp6(dev(wp)), dvdq.W_NATIVE_FP6, dvdq.CODES_FP6, dev(oracle.pack_fp6(codes))
        else:
            w_native, lay = dvdq.w4_prepack(dev(wp)), dvdq.W_NATIVE
            fmt = dvdq.CODES_PACKED4 if packed else dvdq.CODES_INT8
            cd = dev(oracle.pack_a4(codes)) if packed else dev(codes)
        kw = dict(bias=None if bias is None else to_bf16(bias), codes_format=fmt, K=K)
        if use_zero:
            kw.update(w_zero=dev(wz), code_rowsum=dev(codes.astype(np.int32).sum(axis=1).astype(np.int32)))
        dvdq.bench_set_gemm_variant(variant)
        try:
            y, acc = dvdq.w4ax_gemm(cd, dev(xs), w_native, dev(ws), bits, lay, want_acc=True, **kw)
            y2 = dvdq.w4ax_gemm(cd, dev(xs), w_native, dev(ws), bits, lay, **kw)
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


@pytest.mark.parametrize("seed", [21, 22])
def test_random_quantizer_cases(seed):
    from parity import check_blockwise, check_codes_and_scales
    rng = np.random.default_rng(seed)
    for case in range(40):
        K = int(rng.choice([8, 24, 64, 136, 256, 512, 768, 1000, 1536, 2048, 3072, 4104, 8192, 640, 2688]))
        blocks = [b for b in (1, 2, 4, 8, 16, 32, 64, 128, 256, 512) if K % b == 0]
        B = int(rng.choice(blocks))
        M = int(rng.choice([1, 3, 17, 64, 130, 513]))
        bits = int(rng.choice([4, 6, 8]))
        container = str(rng.choice(["int8", "packed4", "fp6"])) if bits == 4 else "int8"
        if K % 128:
            container = "int8" if container == "fp6" else container
        packed, fp6 = container == "packed4", container == "fp6"
        groups = [g for g in (128, 256, 512) if K % g == 0]
        blockwise = bool(bits != 8 and groups and rng.random() < 0.3)
        label = f"seed {seed} case {case}: M{M} K{K} B{B} b{bits} {container} blockwise={blockwise}"
        print(label, flush=True)
        x = rng.standard_normal((M, K)).astype(np.float32) * np.exp(rng.normal(0, 1.0, (M, 1))).astype(np.float32)
        x[:, rng.integers(0, K, max(1, K // 64))] *= 40.0
        xb = di.f32_to_bf16_bits(x)
        xr = oracle.rotate(xb, B)
        if blockwise:
            g = int(rng.choice(groups))
            vals, scale, rs = dvdq.rotate_quant_blockwise(to_bf16(xb), B, bits, g, want_rowsum=True)
            torch.cuda.synchronize()
            v_ref, s_ref, e_ref = oracle.quantize_blockwise(xr, bits, g)
            check_blockwise(vals.cpu().numpy(), scale.cpu().numpy(), v_ref, s_ref, e_ref, xr, bits, g, label,
                            allow_fp32_ties=True)
            codes_np = vals.cpu().numpy()
        else:
            fmt = dvdq.CODES_FP6 if fp6 else (dvdq.CODES_PACKED4 if packed else dvdq.CODES_INT8)
            codes, scale, rs = dvdq.rotate_quant(to_bf16(xb), B, bits, codes_format=fmt, want_rowsum=True)
            torch.cuda.synchronize()
            if fp6:
                codes_np = oracle.unpack_fp6(codes.cpu().numpy(), M, K)
            else:
                codes_np = oracle.unpack_a4(codes.cpu().numpy()) if packed else codes.cpu().numpy()
            c_ref, s_ref = oracle.quantize(xr, bits)
            check_codes_and_scales(codes_np, scale.cpu().numpy(), c_ref, s_ref, xr, bits, label, allow_fp32_ties=True)
        assert np.array_equal(rs.cpu().numpy().astype(np.int64), codes_np.astype(np.int64).sum(axis=1)), label

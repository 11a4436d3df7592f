"""Pins for the CPU oracle: closed forms, hand-derived fixtures, library
special cases, error bounds and brute force -- none of them re-uses the oracle's
own formulae.  A dropped term, wrong sign, wrong index or transposed operand in
``oracle/dvdq_oracle.c`` fails at least one test here.  All CPU-only."""
import os

import numpy as np
import pytest
import scipy.linalg
import torch

import dvdq_inputs as di
import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def bf16(a):
    return di.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))


def read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, *v = line.split()
            out[k] = np.array([float(t) for t in v])
    return out


# ------------------------------------------------------------------ Hadamard
@pytest.mark.parametrize("B", [1, 2, 4, 8, 64, 256, 512])
def test_hadamard_orthogonal_symmetric(B):
    H = oracle.hadamard(B)
    tol = 0.0 if B in (1, 4, 64, 256) else 1e-15   # 1/sqrt(B) is a power of two for even log2(B)
    assert np.max(np.abs(H @ H.T - np.eye(B))) <= tol
    assert np.array_equal(H, H.T)


@pytest.mark.parametrize("B", [2, 16, 256, 512])
def test_hadamard_closed_form_and_library(B):
    """Natural (Sylvester) ordering: H[i,j] = (-1)^popcount(i&j) / sqrt(B)."""
    H = oracle.hadamard(B)
    i, j = np.meshgrid(np.arange(B), np.arange(B), indexing="ij")
    pc = np.array([bin(v).count("1") for v in (i & j).ravel()]).reshape(B, B)
    closed = np.where(pc % 2 == 0, 1.0, -1.0) / np.sqrt(B)
    assert np.array_equal(H, closed)
    assert np.array_equal(H, scipy.linalg.hadamard(B) / np.sqrt(B))


def test_hadamard_rejects_non_power_of_two():
    with pytest.raises(ValueError):
        oracle.hadamard(12)


# ------------------------------------------------------------------ rotation
def test_rotate_worked_example():
    g = read_golden("hadamard4_worked_example.txt")
    xr = oracle.rotate(bf16(g["x"][None, :]), 4)
    assert np.array_equal(xr[0], g["rotated"])


@pytest.mark.parametrize("B", [256, 512])
def test_rotate_impulse_constant_involution_norm(B):
    rng = np.random.default_rng(10)
    # impulse at index i -> row i of H
    idx = [0, 1, 5, B // 2 + 3, B - 1]
    X = np.zeros((len(idx), B), dtype=np.float32)
    for r, i in enumerate(idx):
        X[r, i] = 1.0
    Hlib = scipy.linalg.hadamard(B) / np.sqrt(B)
    assert np.array_equal(oracle.rotate(bf16(X), B), Hlib[idx])
    # constant vector -> sqrt(B) * e_0
    c = oracle.rotate(bf16(np.ones((1, B))), B)[0]
    e0 = np.zeros(B)
    e0[0] = np.sqrt(B)
    assert np.allclose(c, e0, rtol=0, atol=1e-12)
    # norm preservation, and H is an involution (apply twice through exact bf16-representable data)
    x = bf16(rng.standard_normal((7, B)))
    xf = di.bf16_bits_to_f32(x).astype(np.float64)
    xr = oracle.rotate(x, B)
    assert np.allclose(np.linalg.norm(xr, axis=1), np.linalg.norm(xf, axis=1), rtol=1e-12)
    assert np.allclose(xr @ Hlib, xf, rtol=0, atol=1e-12)


def test_rotate_block_diagonal_placement_and_invariance():
    """Blocks of B contiguous channels rotate independently, and rotating both
    operands leaves the product unchanged: (X Hbd)(W Hbd)^T = X W^T."""
    rng = np.random.default_rng(11)
    B, K, M, N = 256, 768, 5, 9
    x = bf16(rng.standard_normal((M, K)))
    w = bf16(rng.standard_normal((N, K)) * 0.02)
    xr, wr = oracle.rotate(x, B), oracle.rotate(w, B)
    Hlib = scipy.linalg.hadamard(B) / np.sqrt(B)
    xf = di.bf16_bits_to_f32(x).astype(np.float64)
    for g in range(K // B):
        assert np.allclose(xr[:, g * B:(g + 1) * B], xf[:, g * B:(g + 1) * B] @ Hlib, rtol=0, atol=1e-12)
    wf = di.bf16_bits_to_f32(w).astype(np.float64)
    ref = xf @ wf.T
    assert np.max(np.abs(xr @ wr.T - ref)) <= 1e-12 * np.max(np.abs(ref)) + 1e-14
    # changing one block of the input only changes that block of the output
    x2 = x.copy()
    x2[:, B:2 * B] = bf16(rng.standard_normal((M, B)))
    xr2 = oracle.rotate(x2, B)
    assert np.array_equal(xr2[:, :B], xr[:, :B]) and np.array_equal(xr2[:, 2 * B:], xr[:, 2 * B:])
    assert not np.array_equal(xr2[:, B:2 * B], xr[:, B:2 * B])


def test_rotate_rejects_bad_block():
    x = bf16(np.ones((1, 96)))
    with pytest.raises(ValueError):
        oracle.rotate(x, 64)      # 64 does not divide 96
    with pytest.raises(ValueError):
        oracle.rotate(x, 48)      # not a power of two


# ------------------------------------------------------------------ quantizer
def test_quant_worked_example():
    g = read_golden("hadamard4_worked_example.txt")
    codes, scale = oracle.rotate_quant(bf16(g["x"][None, :]), 4, 4)
    assert np.array_equal(codes[0], g["codes"].astype(np.int8))
    assert scale[0] == np.float32(g["scale_num"][0] / g["scale_den"][0])


@pytest.mark.parametrize("p", [-9, 0, 5])
def test_quant_ties_to_even(p):
    g = read_golden("rne_ties_a4.txt")
    x = bf16(g["x_over_2p"][None, :] * 2.0 ** p)
    codes, scale = oracle.rotate_quant(x, 1, 4)
    assert scale[0] == np.float32(2.0 ** p)
    assert np.array_equal(codes[0], g["codes"].astype(np.int8))


@pytest.mark.parametrize("bits,qmax", [(4, 7), (6, 31), (8, 127)])
def test_quant_on_grid_roundtrip_exact(bits, qmax):
    """Values already on the grid c * 2^p (some |c| = qmax) come back as c, scale 2^p."""
    rng = np.random.default_rng(bits)
    M, K = 16, 64
    c = rng.integers(-qmax, qmax + 1, size=(M, K))
    c[:, 3] = qmax * rng.choice([-1, 1], size=M)
    p = rng.integers(-6, 6, size=M)
    x = bf16(c * (2.0 ** p)[:, None])          # |c| <= 127 fits bf16's 8 significant bits
    codes, scale = oracle.rotate_quant(x, 1, bits)
    assert np.array_equal(codes, c.astype(np.int8))
    assert np.array_equal(scale, (2.0 ** p).astype(np.float32))


@pytest.mark.parametrize("bits", [4, 6, 8])
def test_quant_range_errorbound_scaleinvariance(bits):
    rng = np.random.default_rng(20 + bits)
    qmax = 2 ** (bits - 1) - 1
    x = rng.standard_normal((33, 512)).astype(np.float32)
    x[:, 7] *= 40.0
    xb = bf16(x)
    codes, scale, xr = oracle.rotate_quant(xb, 256, bits, return_rotated=True)
    # every row reaches +-qmax exactly, never beyond
    assert np.array_equal(np.abs(codes.astype(np.int32)).max(axis=1), np.full(33, qmax))
    # scale is the row abs-max over ALL channels (both blocks) divided by qmax
    amax = np.abs(xr).max(axis=1)
    assert np.all(np.abs(scale.astype(np.float64) * qmax - amax) <= amax * 2.0 ** -23)
    # nearest-grid-point property: |x~ - q*s| <= s/2 (round-to-nearest), up to the fp32 rounding of s
    err = np.abs(xr - codes.astype(np.float64) * scale.astype(np.float64)[:, None])
    assert np.all(err <= 0.5 * scale.astype(np.float64)[:, None] * (1 + 1e-6))
    # doubling the input leaves the codes alone and doubles the scale exactly
    codes2, scale2 = oracle.rotate_quant(bf16(2.0 * di.bf16_bits_to_f32(xb)), 256, bits)
    assert np.array_equal(codes2, codes) and np.array_equal(scale2, 2 * scale)
    # negating the input negates the codes
    codes3, scale3 = oracle.rotate_quant(bf16(-di.bf16_bits_to_f32(xb)), 256, bits)
    assert np.array_equal(codes3, -codes) and np.array_equal(scale3, scale)


def test_quant_zero_row():
    x = bf16(np.zeros((2, 256)))
    x[1, 5] = bf16(np.array([3.0]))[0]
    codes, scale = oracle.rotate_quant(x, 256, 4)
    assert scale[0] == 0.0 and not codes[0].any()
    assert scale[1] > 0 and np.abs(codes[1]).max() == 7


# ------------------------------------------------------------------ packing
def test_pack_unpack_all_pairs_and_generator_agreement():
    lo, hi = np.meshgrid(np.arange(-8, 8), np.arange(-8, 8), indexing="ij")
    codes = np.stack([lo.ravel(), hi.ravel()], axis=1).astype(np.int8).reshape(1, -1)
    packed = oracle.pack_w4(codes)
    assert np.array_equal(oracle.unpack_w4(packed), codes)
    # the input generator has its own (numpy) packer; the oracle's unpacker must invert it
    assert np.array_equal(di.pack_w4(codes), packed)
    # explicit byte values: low nibble = even channel, two's complement
    assert oracle.pack_w4(np.array([[1, -1]], dtype=np.int8))[0, 0] == 0xF1
    assert oracle.pack_w4(np.array([[-7, 7]], dtype=np.int8))[0, 0] == 0x79
    assert np.array_equal(oracle.unpack_w4(np.array([[0x8F]], dtype=np.uint8))[0], [-1, -8])


def test_packed_activation_container_bytes_roundtrip_and_mask_property():
    # hand-derived bytes for one group of 8 channels: byte b = channel b | channel b+4 << 4
    row = np.array([[1, -1, 7, -7, 2, 3, -8, 0]], dtype=np.int8)
    #                 byte0 = 1 | 2<<4, byte1 = 0xF | 3<<4, byte2 = 7 | 8<<4, byte3 = 9 | 0<<4
    assert oracle.pack_a4(row).tolist() == [[0x21, 0x3F, 0x87, 0x09]]
    assert np.array_equal(oracle.unpack_a4(np.array([[0x21, 0x3F, 0x87, 0x09]], dtype=np.uint8)), row)
    # every code value in every one of the 8 positions of a group, two groups per row
    rng = np.random.default_rng(77)
    codes = rng.integers(-8, 8, size=(64, 16)).astype(np.int8)
    for pos in range(16):
        codes[:16, pos] = np.arange(-8, 8)
    packed = oracle.pack_a4(codes)
    assert packed.shape == (64, 8) and np.array_equal(oracle.unpack_a4(packed), codes)
    # the property the container exists for: reading a group as one little-endian 32-bit word p,
    # (p << 4) & 0xF0F0F0F0 and p & 0xF0F0F0F0 are the int8 lanes 16*code of channels 0-3 and 4-7
    p32 = packed.reshape(64, 2, 4).astype(np.uint32)
    word = p32[..., 0] | (p32[..., 1] << 8) | (p32[..., 2] << 16) | (p32[..., 3] << 24)
    lo = ((word << 4) & 0xF0F0F0F0).astype(np.uint32)
    hi = (word & 0xF0F0F0F0).astype(np.uint32)
    lanes = np.stack([(lo >> (8 * b)) & 0xFF for b in range(4)] + [(hi >> (8 * b)) & 0xFF for b in range(4)], axis=-1)
    assert np.array_equal(lanes.astype(np.uint8).view(np.int8).reshape(64, 16).astype(np.int32), 16 * codes.astype(np.int32))


# ------------------------------------------------------------------ integer GEMM
def test_int_gemm_bruteforce_vs_float64():
    rng = np.random.default_rng(30)
    for (M, N, K, qmax) in [(3, 5, 8, 7), (7, 4, 64, 31), (5, 6, 250, 127)]:
        q = rng.integers(-qmax, qmax + 1, size=(M, K)).astype(np.int8)
        w = rng.integers(-8, 8, size=(N, K)).astype(np.int8)
        acc = oracle.int_gemm(q, w)
        ref = q.astype(np.float64) @ w.astype(np.float64).T     # exact below 2^53
        assert np.array_equal(acc.astype(np.float64), ref)
        # pure-python triple loop on the smallest case
        if K == 8:
            for m in range(M):
                for n in range(N):
                    assert acc[m, n] == sum(int(q[m, k]) * int(w[n, k]) for k in range(K))


def test_int_gemm_closed_forms():
    K = 13824
    ones = np.ones((2, K), dtype=np.int8)
    assert np.all(oracle.int_gemm(ones, ones) == K)
    q = np.full((1, K), 127, dtype=np.int8)
    w = np.full((1, K), -7, dtype=np.int8)
    assert oracle.int_gemm(q, w)[0, 0] == -7 * 127 * K
    q = np.full((1, K), 7, dtype=np.int8)
    assert oracle.int_gemm(q, w)[0, 0] == -677376            # 7 * 7 * 13824


def test_one_hot_weights_pin_nibble_order_end_to_end():
    """w[n, k] = delta(k, k0(n)) packed canonically  =>  acc[m, n] = q[m, k0(n)]."""
    rng = np.random.default_rng(31)
    M, K = 4, 64
    k0 = np.array([0, 1, 2, 31, 32, 63])
    w = np.zeros((k0.size, K), dtype=np.int8)
    w[np.arange(k0.size), k0] = 1
    q = rng.integers(-7, 8, size=(M, K)).astype(np.int8)
    y, acc = oracle.w4ax_gemm(q, np.ones(M, np.float32), di.pack_w4(w), np.ones(k0.size, np.float32),
                              return_acc=True)
    assert np.array_equal(acc, q[:, k0].astype(np.int64))
    assert np.array_equal(di.bf16_bits_to_f32(y), q[:, k0].astype(np.float32))
    # negative one-hot pins the sign extension
    y2, acc2 = oracle.w4ax_gemm(q, np.ones(M, np.float32), di.pack_w4(-w), np.ones(k0.size, np.float32),
                                return_acc=True)
    assert np.array_equal(acc2, -q[:, k0].astype(np.int64))


# ------------------------------------------------------------------ epilogue / bf16 rounding
def test_bf16_rounding_against_known_patterns_and_torch():
    v = np.array([1.0, 1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, 1 + 2.0 ** -8 + 2.0 ** -40, -2.5, 0.0, 3.0e38 * 2, 1e-40])
    got = oracle.f64_to_bf16(v)
    #            1.0     tie->even  tie->even(up)  just above tie   -2.5    0     overflow  subnormal
    expect = [0x3F80, 0x3F80, 0x3F82, 0x3F81, 0xC020, 0x0000, 0x7F80, None]
    for g, e in zip(got[:-1], expect[:-1]):
        assert g == e
    # library special case: for float32-representable inputs torch's bf16 cast is the same single RNE
    rng = np.random.default_rng(40)
    f = (rng.standard_normal(20000) * np.exp(rng.uniform(-30, 30, 20000))).astype(np.float32)
    f = np.concatenate([f, np.array([1e-40, -3e-39, 7e-41], dtype=np.float32)])   # bf16 subnormal range
    t = torch.from_numpy(f).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(oracle.f64_to_bf16(f.astype(np.float64)), t)


def test_epilogue_exact_powers_of_two_and_bias():
    acc = np.array([[4, -8, 0], [1, 2, -4]], dtype=np.int64)
    xs = np.array([0.5, 2.0], dtype=np.float32)
    ws = np.array([0.25, 1.0, 8.0], dtype=np.float32)
    y = di.bf16_bits_to_f32(oracle.epilogue(acc, xs, ws))
    assert np.array_equal(y, (acc * xs[:, None] * ws[None, :]).astype(np.float32))
    bias = bf16(np.array([1.0, -2.0, 0.5]))
    yb = di.bf16_bits_to_f32(oracle.epilogue(acc, xs, ws, bias))
    assert np.array_equal(yb, y + np.array([1.0, -2.0, 0.5], dtype=np.float32))


def test_epilogue_within_half_ulp_of_fp64_product():
    rng = np.random.default_rng(41)
    acc = rng.integers(-700000, 700000, size=(8, 16)).astype(np.int64)
    xs = rng.uniform(0.01, 3, 8).astype(np.float32)
    ws = rng.uniform(1e-3, 1e-2, 16).astype(np.float32)
    y = di.bf16_bits_to_f32(oracle.epilogue(acc, xs, ws)).astype(np.float64)
    exact = acc * xs.astype(np.float64)[:, None] * ws.astype(np.float64)[None, :]
    assert np.all(np.abs(y - exact) <= np.abs(exact) * 2.0 ** -8 * (1 + 1e-12))   # half a bf16 ulp, relative bound


# ------------------------------------------------------------------ whole layer
def test_qlinear_is_the_composition_and_tracks_the_float_layer():
    """The one-call oracle equals its steps chained; and against the unquantized
    layer X W^T the error shrinks as activation bits grow and is smaller with the
    rotation than without it on outlier-channel inputs (the qualitative claim of
    Sec. 3.2 about massive outliers)."""
    wl = di.Workload("t", 77, 48, 512, 40, 256, 4, "gauss", 0.5, 0.01, 50.0, 0.02)
    x = di.make_x(wl)
    rng = np.random.default_rng(5)
    w = rng.standard_normal((wl.N, wl.K)) * wl.w_sigma
    xf = di.bf16_bits_to_f32(x).astype(np.float64)
    ref = xf @ w.T
    errs = {}
    for B in (1, 256):
        Hbd = np.kron(np.eye(wl.K // B), scipy.linalg.hadamard(B) / np.sqrt(B)) if B > 1 else np.eye(wl.K)
        wr = w @ Hbd
        ws = (np.abs(wr).max(axis=1) / 7).astype(np.float32)
        wc = np.clip(np.rint(wr / ws[:, None]), -7, 7).astype(np.int8)
        wp = di.pack_w4(wc)
        for bits in (4, 6, 8):
            out = oracle.qlinear(x, wp, ws, B, bits)
            codes, scale = oracle.rotate_quant(x, B, bits)
            y2, acc2 = oracle.w4ax_gemm(codes, scale, wp, ws, return_acc=True)
            assert np.array_equal(out["codes"], codes) and np.array_equal(out["x_scale"], scale)
            assert np.array_equal(out["acc"], acc2) and np.array_equal(out["y"], y2)
            assert np.array_equal(acc2, oracle.int_gemm(codes, oracle.unpack_w4(wp)))
            y = di.bf16_bits_to_f32(out["y"]).astype(np.float64)
            errs[(B, bits)] = np.linalg.norm(y - ref) / np.linalg.norm(ref)
    assert errs[(256, 4)] > errs[(256, 6)] > errs[(256, 8)]
    assert errs[(256, 4)] < 0.8 * errs[(1, 4)]
    assert errs[(256, 8)] < 0.25

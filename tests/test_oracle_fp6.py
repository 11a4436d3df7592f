"""CPU pins of the oracle's FP6 container (oracle.pack_fp6 / unpack_fp6), the encoder and decoder the GPU
tests use to feed and read the FP6 matrix path.  It is pinned to things other than itself: a byte-level
example worked by hand (tests/golden/fp6_container_worked_example.txt), and the E2M3 element format
evaluated field by field with the format's own definition (sign, exponent bias 1, subnormals)."""
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "fp6_container_worked_example.txt")


def e2m3_value(field: int) -> float:
    """value of a 6-bit E2M3 pattern by the format's definition"""
    sign = -1.0 if field & 32 else 1.0
    e, m = (field >> 3) & 3, field & 7
    return sign * (m / 8.0 if e == 0 else 2.0 ** (e - 1) * (1.0 + m / 8.0))


def test_worked_example_bytes():
    rows = channels = None
    codes, expect = [], {}
    for line in open(GOLDEN):
        t = line.split()
        if not t or t[0].startswith("#"):
            continue
        if t[0] == "rows":
            rows = int(t[1])
        elif t[0] == "channels":
            channels = int(t[1])
        elif t[0] == "code":
            codes.append((int(t[1]), int(t[2]), int(t[3])))
        elif t[0] == "byte":
            expect[int(t[1])] = int(t[2], 16)
    c = np.zeros((rows, channels), dtype=np.int8)
    for r, k, v in codes:
        c[r, k] = v
    buf = oracle.pack_fp6(c)
    assert buf.size == rows * channels * 6 // 8
    want = np.zeros(buf.size, dtype=np.uint8)
    for off, val in expect.items():
        want[off] = val
    assert np.array_equal(buf, want)


def test_every_field_has_the_value_code_over_eight():
    """decode the container with nothing but the layout rule and the E2M3 definition"""
    rng = np.random.default_rng(7)
    M, K = 45, 384
    c = rng.integers(-15, 16, (M, K)).astype(np.int8)
    buf = oracle.pack_fp6(c)
    KT = K // 128
    for _ in range(400):
        r, k = int(rng.integers(0, M)), int(rng.integers(0, K))
        kt, kk = divmod(k, 128)
        f, e = 2 * (kk // 64) + (kk % 64) // 32, kk % 32
        bit = 192 * f + 6 * e
        base = ((r // 32) * KT + kt) * 3072 + (r % 32) * 16
        word = 0
        for i in range(2):     # the field may straddle two bytes
            b = bit // 8 + i
            if b < 96:
                word |= int(buf[base + (b // 16) * 512 + b % 16]) << (8 * i)
        field = (word >> (bit % 8)) & 63
        assert e2m3_value(field) * 8 == c[r, k], (r, k)


def test_roundtrip_padding_and_range():
    rng = np.random.default_rng(8)
    for M, K in ((1, 128), (32, 128), (33, 256), (100, 640)):
        c = rng.integers(-15, 16, (M, K)).astype(np.int8)
        buf = oracle.pack_fp6(c)
        assert buf.size == (M + 31) // 32 * 32 * K * 6 // 8
        assert np.array_equal(oracle.unpack_fp6(buf, M, K), c)
        padded = oracle.unpack_fp6(buf, (M + 31) // 32 * 32, K)
        assert not padded[M:].any(), "padding rows hold zero codes"
    with pytest.raises(ValueError):
        oracle.pack_fp6(np.full((1, 128), 16, dtype=np.int8))      # 16 / 8 is not an exact E2M3 integer step
    with pytest.raises(ValueError):
        oracle.pack_fp6(np.zeros((1, 96), dtype=np.int8))


def test_planted_mistakes_are_caught():
    """the pins above fail for plausible mistakes: fragments in plain channel order swapped, sign bit at the
    wrong position, chunk / row order transposed"""
    rng = np.random.default_rng(9)
    c = rng.integers(-7, 8, (32, 128)).astype(np.int8)
    good = oracle.pack_fp6(c)
    # swapped steps within a K half (channel 64 h + 32 s + e -> 64 h + 32 (1 - s) + e)
    swapped = c.reshape(32, 2, 2, 32)[:, :, ::-1, :].reshape(32, 128)
    assert not np.array_equal(oracle.pack_fp6(swapped), good)
    # transposed [chunk][row] -> [row][chunk]
    assert not np.array_equal(good.reshape(6, 32, 16).transpose(1, 0, 2).reshape(-1), good)
    # negative codes must set bit 5 of their field, not two's complement
    one = np.zeros((32, 128), dtype=np.int8)
    one[0, 0] = -1
    assert oracle.pack_fp6(one)[0] == 0b100001

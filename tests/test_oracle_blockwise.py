"""Pins for the oracle's block-wise scaled activation quantizer (a reading of the block-wise variant
of Sec. 3.2: per-token scale times a power-of-two per channel group, folded into int8 values)."""
import os

import numpy as np
import pytest

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def read_gold(name):
    out = {}
    for line in open(os.path.join(GOLD, name)):
        if line.startswith("#") or not line.strip():
            continue
        key, *vals = line.split()
        out[key] = np.array([float(v) for v in vals])
    return out


def rows(seed, M, K, quiet_from=None):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((M, K)) * np.exp(rng.normal(0, 0.5, (M, 1)))
    if quiet_from is not None:
        x[:, quiet_from:] *= 0.05          # channels that are much quieter than the rest of the token
    return x


def test_worked_example():
    g = read_gold("blockwise_worked_example.txt")
    v, s, e = oracle.quantize_blockwise(g["x"][None, :], 4, 4)
    assert s[0] == g["scale"][0] and np.array_equal(e[0], g["exps"].astype(np.uint8))
    assert np.array_equal(v[0], g["values"].astype(np.int8))
    assert np.array_equal(v[0].astype(np.float64) * s[0], g["dequant"])


@pytest.mark.parametrize("bits,emax", [(4, 4), (6, 2), (8, 0)])
def test_structure_exponents_are_maximal_and_nothing_clips(bits, emax):
    qmax = 2 ** (bits - 1) - 1
    G = 32
    x = rows(1, 40, 256, quiet_from=160)
    v, s, e = oracle.quantize_blockwise(x, bits, G)
    assert e.max() <= emax and (emax == 0 or e.max() == emax) and e.min() == 0
    vv = v.astype(np.int64).reshape(40, -1, G)
    sh = (emax - e.astype(np.int64))[:, :, None]
    assert np.all(vv % (1 << sh) == 0)                       # stored value = code * 2^(emax - e)
    q = vv >> sh
    assert np.abs(q).max() <= qmax and np.abs(vv).max() <= 127
    # each token's scale is the per-token scale / 2^emax, and the largest group reaches +-qmax
    _, s_tok = oracle.quantize(x, bits)
    assert np.array_equal(s, (s_tok.astype(np.float64) / 2 ** emax).astype(np.float32))
    assert np.all(np.abs(q).reshape(40, -1).max(axis=1) == qmax)
    # maximal exponent: a group that could have been scaled finer (e < emax) uses more than half the range
    gmax = np.abs(q).max(axis=2)
    assert np.all(gmax[e < emax] >= np.ceil(qmax / 2))
    # error bound: half a group step everywhere
    step = s.astype(np.float64)[:, None, None] * (1 << sh)
    err = np.abs(x.reshape(40, -1, G) - vv * s.astype(np.float64)[:, None, None])
    assert np.all(err <= step / 2 * (1 + 1e-6))


def test_reduces_to_the_per_token_quantizer_when_groups_are_alike_or_one():
    x = rows(2, 16, 128)
    codes, s_tok = oracle.quantize(x, 4)
    v, s, e = oracle.quantize_blockwise(x, 4, 128)            # one group per token
    assert np.all(e == 0) and np.array_equal(v.astype(np.int32), codes.astype(np.int32) * 16)
    assert np.array_equal(s.astype(np.float64) * 16, s_tok.astype(np.float64))
    # groups within a factor of two of the row maximum keep e = 0
    x2 = np.tile(np.array([[1.0, -0.9, 0.8, 0.7, 0.6, -0.95, 0.55, 0.51]]), (3, 1))
    v2, _, e2 = oracle.quantize_blockwise(x2, 4, 2)
    assert np.all(e2 == 0) and np.array_equal(v2, oracle.quantize(x2, 4)[0].astype(np.int32) * 16)


def test_exact_power_of_two_ratio_takes_the_finer_step():
    # group maximum exactly amax / 16: a * 2^4 <= amax holds with equality, so e = 4 and the group reaches +-7
    x = np.array([[7.0, 0, 0, 0, 0.4375, 0, 0, 0, 0.875, -0.5, 0, 0]])
    v, s, e = oracle.quantize_blockwise(x, 4, 4)
    assert e.tolist() == [[0, 4, 3]]
    assert v.tolist() == [[112, 0, 0, 0, 7, 0, 0, 0, 14, -8, 0, 0]]


def test_lower_error_than_per_token_scaling_on_tokens_with_quiet_groups():
    x = rows(3, 64, 1024, quiet_from=512)
    codes, s_tok = oracle.quantize(x, 4)
    v, s, _ = oracle.quantize_blockwise(x, 4, 128)
    d_tok = x - codes * s_tok.astype(np.float64)[:, None]
    d_blk = x - v * s.astype(np.float64)[:, None]
    assert np.linalg.norm(d_blk) < np.linalg.norm(d_tok)
    assert np.linalg.norm(d_blk[:, 512:]) < 0.2 * np.linalg.norm(d_tok[:, 512:])     # the quiet channels gain
    # elementwise never worse than the per-token bound (the group step is never coarser)
    assert np.all(np.abs(x - v * s.astype(np.float64)[:, None]) <= s_tok.astype(np.float64)[:, None] / 2 * (1 + 1e-6))


def test_gemm_on_the_int8_values_is_the_blockwise_sum():
    """y = sum_g s_mg * sum_{k in g} q_mk w_nk * Delta_n, written out group by group in numpy, equals
    the plain integer GEMM on the stored int8 values with the handed-on token scale."""
    rng = np.random.default_rng(4)
    M, N, K, G = 6, 10, 256, 64
    x = rows(5, M, K, quiet_from=128)
    v, s, e = oracle.quantize_blockwise(x, 4, G)
    wc = rng.integers(-7, 8, (N, K)).astype(np.int8)
    ws = np.exp(rng.normal(-4, 0.3, N)).astype(np.float32)
    y, acc = oracle.w4ax_gemm(v, s, oracle.pack_w4(wc), ws, return_acc=True)
    q = v.astype(np.int64).reshape(M, -1, G) >> (4 - e.astype(np.int64))[:, :, None]
    s_g = s.astype(np.float64)[:, None] * 16.0 / 2.0 ** e                     # s_m * 2^-e
    part = np.einsum("mgk,ngk->mgn", q, wc.astype(np.int64).reshape(N, -1, G))  # per-group integer partial sums
    y_blk = (part * s_g[:, :, None]).sum(axis=1) * ws.astype(np.float64)[None, :]
    assert np.array_equal(oracle.f64_to_bf16(y_blk), y)
    assert np.array_equal(acc, (part << (4 - e.astype(np.int64))[:, :, None]).sum(axis=1))


def test_scale_equivariance_zero_rows_and_bad_group():
    x = rows(6, 8, 64, quiet_from=32)
    v, s, e = oracle.quantize_blockwise(x, 4, 16)
    v2, s2, e2 = oracle.quantize_blockwise(x * 4.0, 4, 16)
    assert np.array_equal(v, v2) and np.array_equal(e, e2) and np.array_equal(s * np.float32(4), s2)
    z = np.zeros((2, 32))
    v, s, e = oracle.quantize_blockwise(z, 4, 8)
    assert np.all(v == 0) and np.all(s == 0)
    with pytest.raises(ValueError):
        oracle.quantize_blockwise(x, 4, 24)

"""Pins for the oracle's delta-GBS pieces (Sec. 3.3): the relative L1 change and the
controller update.  CPU-only."""
import os

import numpy as np

import dvdq_inputs as di
import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def bf16(a):
    return di.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))


def test_rel_l1_closed_forms():
    a = bf16([1.0, -2.0, 3.0, 0.5])
    b = bf16([1.0, 2.0, 1.0, -0.5])
    # |0| + |-4| + |2| + |1| = 7 ; |1| + |2| + |1| + |0.5| = 4.5
    assert oracle.rel_l1(a, b) == 7.0 / 4.5
    assert oracle.rel_l1(b, b) == 0.0
    # scaling both tensors leaves the ratio alone; F_t = 2 F_{t-1} gives exactly 1
    assert oracle.rel_l1(bf16([2.0, -4.0, 6.0]), bf16([1.0, -2.0, 3.0])) == 1.0
    assert oracle.rel_l1(bf16([4.0, -8.0, 12.0, 2.0]), bf16([4.0, 8.0, 4.0, -2.0])) == 7.0 / 4.5
    # not symmetric: the denominator is the PREVIOUS output
    assert oracle.rel_l1(bf16([0.0, 0.0]), bf16([1.0, 1.0])) == 1.0
    assert oracle.rel_l1(bf16([1.0, 1.0]), bf16([0.0, 0.0])) == np.inf
    assert oracle.rel_l1(bf16([0.0]), bf16([0.0])) == 0.0


def test_rel_l1_against_numpy_float64():
    rng = np.random.default_rng(0)
    a, b = bf16(rng.standard_normal(100003)), bf16(rng.standard_normal(100003) * 3)
    af, bfl = di.bf16_bits_to_f32(a).astype(np.float64), di.bf16_bits_to_f32(b).astype(np.float64)
    ref = np.abs(af - bfl).sum() / np.abs(bfl).sum()
    assert abs(oracle.rel_l1(a, b) - ref) <= 1e-12 * ref


def test_controller_worked_sequence():
    g = {}
    for line in open(os.path.join(GOLDEN, "gbs_worked_sequence.txt")):
        if line.strip() and not line.startswith("#"):
            k, *v = line.split()
            g[k] = [float(t) for t in v]
    acc, got = 0.0, []
    for l1 in g["l1"]:
        bits, acc = oracle.gbs_update(l1, g["delta"][0], 4, 8, acc)
        got.append(bits)
    assert got == [int(b) for b in g["bits"]]


def test_controller_limits():
    """delta -> 0 keeps every step at b_high, delta -> infinity at b_low (the two ends of the
    threshold sweep the paper discusses)."""
    rng = np.random.default_rng(1)
    l1s = rng.uniform(0.01, 0.2, 50)
    acc = 0.0
    for l1 in l1s:
        bits, acc = oracle.gbs_update(l1, 0.0, 4, 8, acc)
        assert bits == 8 and acc == 0.0
    acc = 0.0
    for l1 in l1s:
        bits, acc = oracle.gbs_update(l1, np.inf, 4, 8, acc)
        assert bits == 4
    assert abs(acc - l1s.sum()) < 1e-12

"""The seeded input generator: shapes, determinism, row-subset consistency and
the structure the workloads are meant to have.  CPU-only."""
import numpy as np

import dvdq_inputs as di


def test_workload_table_matches_the_five_configs():
    shapes = [(w.M, w.K, w.N, w.had_block, w.act_bits) for w in di.WORKLOADS]
    assert shapes == [(128, 256, 256, 256, 4), (32760, 1536, 4608, 256, 4), (32760, 1536, 8960, 256, 6),
                      (118800, 3072, 3072, 256, 4), (32760, 13824, 5120, 512, 4)]
    assert [w.seed for w in di.WORKLOADS] == [0, 1, 2, 3, 4]
    assert 21 * 30 * 52 == 32760 and 33 * 45 * 80 == 118800
    assert di.WORKLOADS[4].K // 512 == 27


def test_bf16_cast_roundtrip_and_rne():
    f = np.array([1.0, 1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, -0.0, 3.140625], dtype=np.float32)
    b = di.f32_to_bf16_bits(f)
    assert list(b) == [0x3F80, 0x3F80, 0x3F82, 0x8000, 0x4049]
    assert np.array_equal(di.f32_to_bf16_bits(di.bf16_bits_to_f32(b)), b)


def test_x_rows_are_a_consistent_view_of_the_full_tensor():
    wl = di.Workload("t", 9, 2500, 512, 8, 256, 4, "gauss", 0.5, 0.01, 50.0, 0.02)
    full = di.make_x(wl)
    assert full.shape == (2500, 512) and full.dtype == np.uint16
    rows = np.array([0, 1, 1023, 1024, 2047, 2048, 2499])
    assert np.array_equal(di.make_x_rows(wl, rows), full[rows])
    assert np.array_equal(di.make_x(wl), full)          # deterministic


def test_outlier_channels_and_token_scales_show_up():
    wl = di.WORKLOADS[0]
    x = di.bf16_bits_to_f32(di.make_x(wl)).astype(np.float64)
    rms = np.sqrt((x ** 2).mean(axis=0))
    assert (rms > 10).sum() == 5                         # 2 % of 256 channels scaled x30
    wl4 = di.Workload("t", 4, 64, 1024, 8, 512, 4, "postgelu", 0.0, 0.005, 80.0, 0.015)
    x4 = di.bf16_bits_to_f32(di.make_x(wl4))
    assert x4.min() >= -0.17 * 80 * (1 + 2.0 ** -8) and (x4 < 0).any()


def test_weights_recipe():
    wl = di.WORKLOADS[0]
    wp, ws, wc = di.make_weights(wl)
    assert wp.shape == (256, 128) and wp.dtype == np.uint8 and ws.shape == (256,) and ws.dtype == np.float32
    assert wc.min() >= -7 and wc.max() <= 7 and np.all(np.abs(wc).max(axis=1) == 7)
    assert np.all(ws > 0)
    lo = (wp & 0xF).astype(np.int8)
    lo = np.where(lo >= 8, lo - 16, lo)
    assert np.array_equal(lo, wc[:, 0::2])


def test_sample_rows_cover_head_and_tail():
    r = di.sample_rows(32760)
    assert r.size == 512 and r[0] == 0 and r[-1] == 32759 and r[255] == 255 and r[256] == 32760 - 256
    assert np.array_equal(di.sample_rows(128), np.arange(128))

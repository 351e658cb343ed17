"""The seeded input generators: reproducible, of the stated shape and distribution, and free
of the method's arithmetic (they only draw numbers)."""
import numpy as np

import tally_inputs as TI


def test_generators_are_reproducible_and_differ_by_configuration():
    a = TI.saxpy_inputs(n=1000, config_index=0)
    b = TI.saxpy_inputs(n=1000, config_index=0)
    c = TI.saxpy_inputs(n=1000, config_index=1)
    assert (a["x"] == b["x"]).all() and (a["y"] == b["y"]).all()
    assert not (a["x"] == c["x"]).all()
    g = TI.gemm_inputs(64, 32, 16, config_index=1, batch=2)
    assert g["A"].shape == (2, 64, 16) and g["Bt"].shape == (2, 32, 16) and g["A"].dtype == np.uint16


def test_preempt_points_are_distinct_sorted_and_inside_the_grid():
    pts = TI.preempt_points(4096, 3, config_index=0)
    assert pts == sorted(set(pts)) and len(pts) == 3 and 1 <= pts[0] and pts[-1] <= 4095


def test_bf16_bits_round_to_nearest_even():
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -2.5], np.float32)
    bits = TI.to_bf16_bits(x)
    # 1 + 2^-8 lies half way between 1 and 1 + 2^-7: ties go to the even mantissa (1.0);
    # 1 + 3*2^-8 lies half way between 1 + 2^-7 and 1 + 2^-6: even is 1 + 2^-6
    assert bits.tolist() == [0x3F80, 0x3F80, 0x3F82, 0xC020]


def test_arrival_processes():
    p = TI.periodic_arrivals_us(1000.0, 5)
    assert p.tolist() == [1000.0, 2000.0, 3000.0, 4000.0, 5000.0]
    a = TI.poisson_arrivals_us(500.0, 20000, config_index=2)
    assert (np.diff(a) > 0).all() and len(a) == 20000
    assert abs(20000 / (a[-1] * 1e-6) - 500.0) < 15.0            # mean rate within 3 %
    gaps = np.diff(a)
    assert abs(gaps.std() / gaps.mean() - 1.0) < 0.05            # exponential gaps: cv = 1
    b = TI.bursty_arrivals_us(1000.0, 20000, config_index=1, burst=10.0, p_on=0.05,
                              mean_segment_us=2000.0)
    assert (np.diff(b) > 0).all() and len(b) == 20000
    assert 700.0 < 20000 / (b[-1] * 1e-6) < 1400.0               # mean rate as asked, roughly
    gb = np.diff(b)
    assert gb.std() / gb.mean() > 1.2                            # burstier than Poisson
    # windows of 2 ms: the busiest carry several times the mean load
    w = np.histogram(b, bins=np.arange(0.0, b[-1], 2000.0))[0]
    assert w.max() > 4 * w.mean()

"""Sec. 3.3 (Eq. 1-4) host arithmetic, checked against the inequality it is derived from."""
import math

import numpy as np

from paper_1811_08596_amd import sensitivity as S


def test_threshold_is_where_twice_the_codec_cost_meets_the_saved_wire_time():
    rng = np.random.default_rng(7)
    for _ in range(200):
        T_m, T_f, T_p, T_s = rng.uniform(5, 500, 4)
        T_comm = rng.uniform(0.1, 30)
        M = rng.uniform(1e6, 1e9)
        k0 = S.min_useful_ratio(T_comm, T_m, T_f, T_p, T_s)
        cost_comp = M * (2 / T_m + 1 / T_f + 1 / T_p + 1 / T_s)                  # Eq. 1
        saved = lambda k: M / T_comm * (1 - 1 / k)                               # Eq. 3
        if math.isinf(k0):
            assert 2 * cost_comp >= M / T_comm                                  # even k -> infinity cannot pay
        else:
            assert k0 > 1
            assert 2 * cost_comp < saved(k0 * 1.001)
            assert 2 * cost_comp > saved(k0 * 0.999)


def test_slow_links_need_little_and_fast_links_much():
    # Sec. 3.3: a slow network pays at a small ratio, a fast one needs a large one or cannot pay at all
    T = dict(T_m=300.0, T_f=100.0, T_p=34.0, T_s=40.0)
    ks = [S.min_useful_ratio(t, **T) for t in (0.1, 1.25, 7.0)]
    assert 1.0 < ks[0] < ks[1] < ks[2]
    assert ks[0] < 1.05
    assert math.isinf(S.min_useful_ratio(1e3, **T))


def test_selection_alone_caps_the_useful_link():
    # with only the selection term, Eq. 4's denominator vanishes at T_comm = T_s / 2: a 12 GB/s selection can never
    # pay above 6 GB/s = 48 Gb/s, and the other terms only lower that (the paper reads 22 Gb/s off its figure)
    big = 1e12
    assert math.isinf(S.min_useful_ratio(6.0, big, big, big, 12.0))
    assert not math.isinf(S.min_useful_ratio(5.99, big, big, big, 12.0))
    assert S.break_even_link(12.0, 12.0) == 6.0


def test_measured_directions_are_the_same_formula():
    c = S.codec_seconds_per_byte(200.0, 90.0, 34.0, 12.0)
    assert S.min_useful_ratio(2.0, 200.0, 90.0, 34.0, 12.0) == S.min_useful_ratio_measured(2.0, 1 / c, 1 / c)

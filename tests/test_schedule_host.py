"""The library's host-side scheduling arithmetic (Algorithm 2, Eqs. 2-14) against the oracle's and
against the numbers the paper prints.  No GPU needed."""
import math

import numpy as np
import pytest

import paper_2003_10735_amd as st
from oracle import schedule as S
from test_oracle_schedule import P


def test_next_stride_matches_oracle_on_a_grid():
    rng = np.random.default_rng(3)
    for _ in range(2000):
        stride = rng.uniform(1, 100)
        metric = rng.uniform(0, 1)
        thr = rng.uniform(0.05, 0.95)
        lo = rng.uniform(1, 16)
        hi = lo + rng.uniform(0, 100)
        a = st.st_next_stride(stride, metric, thr, lo, hi)
        b = S.next_stride(stride, metric, thr, lo, hi)
        assert a == pytest.approx(b, rel=1e-12, abs=1e-12)
    thr = P["threshold"]
    assert st.st_next_stride(10, 0.0, thr, 0, 1e9) == 0.0
    assert st.st_next_stride(10, thr, thr, 0, 1e9) == pytest.approx(10.0, abs=1e-12)
    assert st.st_next_stride(10, 1.0, thr, 0, 1e9) == pytest.approx(20.0, abs=1e-12)
    assert math.isnan(st.st_next_stride(10, 0.5, 1.0, 1, 2))
    assert math.isnan(st.st_next_stride(10, 0.5, 0.5, 3, 2))


def paper_params(**kw):
    d = dict(t_si=P["t_si"], t_sd=P["t_sd"], t_ti=P["t_ti"], t_net=P["t_net"], s_net=P["s_net_mb"] * 8e6,
             min_stride=P["min_stride"], max_stride=P["max_stride"], max_updates=P["max_updates"])
    d.update(kw)
    return d


def test_printed_numbers():
    b = st.st_schedule_bounds(**paper_params())
    assert round(b["throughput_upper"], 2) == P["throughput_upper_fps"]
    assert b["throughput_lower"] > P["throughput_lower_floor_fps"]
    assert st.st_schedule_bounds(**paper_params(max_updates=9))["throughput_lower"] < P["throughput_lower_floor_fps"]
    assert round(b["traffic_lower"] / 1e6, 2) == P["traffic_lower_mbps"]
    assert round(b["traffic_upper"] / 1e6, 1) == P["traffic_upper_mbps"]


def test_bounds_match_oracle_on_random_parameters():
    rng = np.random.default_rng(4)
    for _ in range(500):
        q = dict(t_si=rng.uniform(0.01, 0.5), t_sd=rng.uniform(0.001, 0.05), t_ti=rng.uniform(0.01, 0.2),
                 t_net=rng.uniform(0.01, 1.0), s_net=rng.uniform(1, 1e8), min_stride=float(rng.integers(1, 16)),
                 max_updates=float(rng.integers(0, 20)))
        q["max_stride"] = q["min_stride"] + float(rng.integers(0, 100))
        b = st.st_schedule_bounds(**q)
        lo, hi = S.t_c_bounds(q["t_si"], q["t_ti"], q["t_net"], q["min_stride"])
        ref = dict(t_c_lower=lo, t_c_upper=hi,
                   traffic_lower=S.traffic_lower(q["s_net"], q["t_si"], q["t_sd"], q["t_ti"], q["t_net"], q["max_stride"], q["max_updates"]),
                   traffic_upper=S.traffic_upper(q["s_net"], q["t_si"], q["t_ti"], q["t_net"], q["min_stride"]),
                   throughput_lower=S.throughput_lower(q["t_si"], q["t_sd"], q["t_ti"], q["t_net"], q["min_stride"], q["max_updates"]),
                   throughput_upper=S.throughput_upper(q["t_si"], q["t_ti"], q["t_net"], q["min_stride"], q["max_stride"]))
        for k, v in ref.items():
            assert b[k] == pytest.approx(v, rel=1e-12), k
        n, d, k = 5000.0, 300.0, 90.0
        assert st.st_schedule_total_time(n, d, k, hi, **q) == pytest.approx(
            S.t_total(n, d, k, q["t_si"], q["t_sd"], hi, q["min_stride"]), rel=1e-12)


def test_bad_parameters():
    with pytest.raises(st.StError):
        st.st_schedule_bounds(**paper_params(t_si=0.0))
    with pytest.raises(st.StError):
        st.st_schedule_bounds(**paper_params(max_stride=4.0))
    with pytest.raises(st.StError):
        st.st_schedule_bounds(**paper_params(t_net=float("nan")))

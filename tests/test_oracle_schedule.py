"""Pins of the scheduling oracle: the numbers the paper prints for its own configuration and the
points Algorithm 2's text names."""
import os

import pytest

from oracle import schedule as S

HERE = os.path.dirname(os.path.abspath(__file__))


def printed():
    out = {}
    for line in open(os.path.join(HERE, "golden", "printed_bounds.txt")):
        line = line.split("#")[0].split()
        if len(line) == 2:
            out[line[0]] = float(line[1])
    return out


P = printed()


def test_next_stride_passes_through_the_named_points():
    """Section 4.1 (key frame striding): the ratio connects (0,0), (THRESHOLD,1) and (1,2)."""
    thr = P["threshold"]
    big = 1e9
    assert S.next_stride(10.0, 0.0, thr, 0.0, big) == 0.0
    assert S.next_stride(10.0, thr, thr, 0.0, big) == pytest.approx(10.0, abs=1e-12)
    assert S.next_stride(10.0, 1.0, thr, 0.0, big) == pytest.approx(20.0, abs=1e-12)
    # linear in between, continuous at the threshold
    assert S.next_stride(10.0, thr / 2, thr, 0.0, big) == pytest.approx(5.0, abs=1e-12)
    assert S.next_stride(10.0, (1 + thr) / 2, thr, 0.0, big) == pytest.approx(15.0, abs=1e-12)
    assert S.next_stride(10.0, thr - 1e-12, thr, 0.0, big) == pytest.approx(10.0, abs=1e-9)
    # clamped
    assert S.next_stride(8.0, 0.1, thr, P["min_stride"], P["max_stride"]) == P["min_stride"]
    assert S.next_stride(64.0, 0.99, thr, P["min_stride"], P["max_stride"]) == P["max_stride"]


def test_printed_throughput_bounds():
    up = S.throughput_upper(P["t_si"], P["t_ti"], P["t_net"], P["min_stride"], P["max_stride"])
    assert round(up, 2) == P["throughput_upper_fps"]
    lo8 = S.throughput_lower(P["t_si"], P["t_sd"], P["t_ti"], P["t_net"], P["min_stride"], 8)
    lo9 = S.throughput_lower(P["t_si"], P["t_sd"], P["t_ti"], P["t_net"], P["min_stride"], 9)
    # 8 is the largest MAX_UPDATES whose lower bound stays above 5 FPS, and the gap is within 2 FPS
    assert lo8 > P["throughput_lower_floor_fps"] > lo9
    assert P["max_updates"] == 8 and up - lo8 < 2.0


def test_printed_traffic_bounds():
    s_bits = P["s_net_mb"] * 1e6 * 8
    lo = S.traffic_lower(s_bits, P["t_si"], P["t_sd"], P["t_ti"], P["t_net"], P["max_stride"], P["max_updates"])
    hi = S.traffic_upper(s_bits, P["t_si"], P["t_ti"], P["t_net"], P["min_stride"])
    assert round(lo / 1e6, 2) == P["traffic_lower_mbps"]
    assert round(hi / 1e6, 1) == P["traffic_upper_mbps"]
    assert round(100 * (1 - P["s_net_mb"] / P["s_net_naive_mb"]), 2) == P["reduction_per_key_frame_percent"]


def test_bounds_are_the_general_formulas_at_their_extremes():
    """Eqs. 8, 12, 13, 14 are Eqs. 4 and 9 with the k, d, t_c of Eqs. 5-7 and 10-11."""
    a = dict(t_si=P["t_si"], t_sd=P["t_sd"])
    mn, mx, mu = P["min_stride"], P["max_stride"], P["max_updates"]
    tc_lo, tc_hi = S.t_c_bounds(P["t_si"], P["t_ti"], P["t_net"], mn)
    n = 6400.0
    s = 1.0
    assert S.traffic(n, n / mx * mu, n / mx, s, a["t_si"], a["t_sd"], tc_hi, mn) == pytest.approx(
        S.traffic_lower(s, P["t_si"], P["t_sd"], P["t_ti"], P["t_net"], mx, mu), rel=1e-12)
    assert S.traffic(n, 0.0, n / mn, s, a["t_si"], a["t_sd"], tc_lo, mn) == pytest.approx(
        S.traffic_upper(s, P["t_si"], P["t_ti"], P["t_net"], mn), rel=1e-12)
    assert S.throughput(n, n / mn * mu, n / mn, a["t_si"], a["t_sd"], tc_hi, mn) == pytest.approx(
        S.throughput_lower(P["t_si"], P["t_sd"], P["t_ti"], P["t_net"], mn, mu), rel=1e-12)
    assert S.throughput(n, 0.0, n / mx, a["t_si"], a["t_sd"], tc_lo, mn) == pytest.approx(
        S.throughput_upper(P["t_si"], P["t_ti"], P["t_net"], mn, mx), rel=1e-12)

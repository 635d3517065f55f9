"""Oracle for the scheduling arithmetic around the training step: key-frame striding
(Algorithm 2) and the analytic bounds of Section 4.4 (Eqs. 2-14).

TEST INFRASTRUCTURE, NOT THE PRODUCT: plain double-precision formulas written out from the
paper's statements, sharing no code with the library.  Pinned by the numbers the paper prints
for its own configuration (tests/golden/printed_bounds.txt).
"""
from __future__ import annotations


def next_stride(stride, metric, threshold, min_stride, max_stride):
    """Algorithm 2.  The ratio of the next stride to the current one is piecewise linear in the
    metric: through (0, 0) and (THRESHOLD, 1) below the threshold, through (THRESHOLD, 1) and
    (1, 2) from it on; the product is clamped to [MIN_STRIDE, MAX_STRIDE]."""
    if metric < threshold:
        ratio = metric / threshold
    else:
        ratio = (metric - 2.0 * threshold + 1.0) / (1.0 - threshold)
    s = ratio * stride
    return min(max(s, min_stride), max_stride)


def t_c_bounds(t_si, t_ti, t_net, min_stride):
    """Eq. 2: execution time of the MIN_STRIDE frames after a key frame, (lower, upper):
    full overlap of inference and network on the client, or none."""
    return max(min_stride * t_si, t_net + t_ti), min_stride * t_si + t_net + t_ti


def t_total(n, d, k, t_si, t_sd, t_c, min_stride):
    """Eq. 3: time to process n frames with k key frames and d distillation steps."""
    return (n - k * min_stride) * t_si + d * t_sd + k * t_c


def traffic(n, d, k, s_net, t_si, t_sd, t_c, min_stride):
    """Eq. 4: networked bytes per second."""
    return k * s_net / t_total(n, d, k, t_si, t_sd, t_c, min_stride)


def throughput(n, d, k, t_si, t_sd, t_c, min_stride):
    """Eq. 9: frames per second."""
    return n / t_total(n, d, k, t_si, t_sd, t_c, min_stride)


def traffic_lower(s_net, t_si, t_sd, t_ti, t_net, max_stride, max_updates):
    """Eq. 8 (key frames every MAX_STRIDE, MAX_UPDATES steps each, no concurrency)."""
    return s_net / (max_stride * t_si + max_updates * t_sd + t_ti + t_net)


def traffic_upper(s_net, t_si, t_ti, t_net, min_stride):
    """Eq. 12 (key frames every MIN_STRIDE, no distillation, full concurrency)."""
    return s_net / max(min_stride * t_si, t_net + t_ti)


def throughput_lower(t_si, t_sd, t_ti, t_net, min_stride, max_updates):
    """Eq. 13."""
    return min_stride / (min_stride * t_si + max_updates * t_sd + t_ti + t_net)


def throughput_upper(t_si, t_ti, t_net, min_stride, max_stride):
    """Eq. 14."""
    return max_stride / ((max_stride - min_stride) * t_si + max(min_stride * t_si, t_net + t_ti))

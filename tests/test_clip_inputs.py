"""Host-side checks of the clip input generator (no GPU)."""
import numpy as np

import workloads as WL


def test_clip_frames_shapes_and_motion():
    wl = WL.small_variant(WL.WORKLOADS["tiny"], c_in=4, h=4, w=6, n_classes=3, n_sites=4,
                          extra={"frames": 3, "drift": 0.05, "shift_px": 2, "threshold": 0.75})
    a = list(WL.clip_frames(wl))
    b = list(WL.clip_frames(wl))
    assert len(a) == 3
    for (fa, la), (fb, lb) in zip(a, b):
        assert fa.shape == (1, 4, 4, 6) and la.shape == (1, 32, 48) and la.dtype == np.int32
        np.testing.assert_array_equal(fa, fb)
        np.testing.assert_array_equal(la, lb)
    # the label pattern moves right by shift_px per frame
    np.testing.assert_array_equal(a[1][1][:, :, 2:], a[0][1][:, :, :-2])
    # the features drift by N(0, drift^2) per frame
    d = (a[1][0] - a[0][0]).astype(np.float64)
    assert 0.02 < d.std() < 0.1

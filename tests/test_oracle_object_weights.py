"""Pins of the loss-weight map oracle (Section 5.2: a factor on pixels near and within
non-background objects): brute force over every pixel pair, a library dilation, closed-form
counts, and the cases that reduce to the label map itself."""
import numpy as np
import pytest
from scipy import ndimage

import workloads as WL
from oracle import object_weights as OW


def brute_force(lab, n_classes, radius, factor, background, ignore_index):
    """Every pixel against every other pixel of its frame, by the sentence of the definition."""
    n, H, W = lab.shape
    out = np.ones((n, H, W), np.uint8)
    for f in range(n):
        for y in range(H):
            for x in range(W):
                for yy in range(H):
                    for xx in range(W):
                        v = int(lab[f, yy, xx])
                        if abs(yy - y) <= radius and abs(xx - x) <= radius and 0 <= v < n_classes \
                                and v != background and v != ignore_index:
                            out[f, y, x] = factor
    return out


def random_labels(rng, n, H, W, n_classes, p_object, ignore_index=-1, p_ignore=0.0):
    lab = np.zeros((n, H, W), np.int32)
    m = rng.random(lab.shape) < p_object
    lab[m] = rng.integers(1, n_classes, size=int(m.sum()))
    if p_ignore:
        lab[rng.random(lab.shape) < p_ignore] = ignore_index
    return lab


@pytest.mark.parametrize("seed,radius", [(1, 0), (2, 1), (3, 2), (4, 3), (5, 7)])
def test_against_brute_force(seed, radius):
    rng = np.random.default_rng(seed)
    lab = random_labels(rng, 2, 7, 11, 5, 0.06, ignore_index=255, p_ignore=0.1)
    lab[0, 0, 0] = 9            # outside [0, n_classes): no object
    lab[1, 6, 10] = -3
    lab[1, 0, 10] = 5           # the first value that is no class index
    got = OW.object_weights(lab, 5, radius, factor=5, background=0, ignore_index=255)
    np.testing.assert_array_equal(got, brute_force(lab, 5, radius, 5, 0, 255))


@pytest.mark.parametrize("radius", [0, 1, 4, 9, 32])
def test_against_a_library_dilation(radius):
    """The same set is the morphological dilation of the object mask by a (2r+1) x (2r+1) square."""
    rng = np.random.default_rng(40 + radius)
    lab = random_labels(rng, 3, 50, 83, 19, 0.004)
    obj = (lab != 0)
    near = ndimage.binary_dilation(obj, structure=np.ones((1, 2 * radius + 1, 2 * radius + 1), bool))
    got = OW.object_weights(lab, 19, radius, factor=7)
    np.testing.assert_array_equal(got, np.where(near, 7, 1).astype(np.uint8))


def test_single_object_pixel_gives_a_clipped_square():
    """One object pixel at (y, x): the marked set is the square of side 2r + 1 around it cut off
    at the frame, so its size is a product of two clipped lengths."""
    H, W, r = 13, 17, 4
    for (y, x) in [(6, 8), (0, 0), (12, 16), (2, 15), (11, 1)]:
        lab = np.zeros((1, H, W), np.int32)
        lab[0, y, x] = 2
        w = OW.object_weights(lab, 3, r)
        rows = min(H - 1, y + r) - max(0, y - r) + 1
        cols = min(W - 1, x + r) - max(0, x - r) + 1
        assert int((w == 5).sum()) == rows * cols
        assert int((w == 1).sum()) == H * W - rows * cols
        assert w[0, max(0, y - r), max(0, x - r)] == 5 and w[0, min(H - 1, y + r), min(W - 1, x + r)] == 5


def test_radius_zero_marks_exactly_the_objects():
    rng = np.random.default_rng(7)
    lab = random_labels(rng, 2, 20, 30, 9, 0.3, ignore_index=255, p_ignore=0.05)
    w = OW.object_weights(lab, 9, 0, factor=5, ignore_index=255)
    np.testing.assert_array_equal(w == 5, (lab > 0) & (lab < 9))


def test_no_object_and_all_objects():
    lab = np.zeros((1, 6, 9), np.int32)
    assert (OW.object_weights(lab, 4, 3) == 1).all()
    lab[:] = 255
    assert (OW.object_weights(lab, 4, 3, ignore_index=255) == 1).all()
    lab[:] = 1
    assert (OW.object_weights(lab, 4, 0) == 5).all()


def test_background_class_and_frames_are_separate():
    """Another background index changes which labels are objects; an object in one frame marks
    nothing in the next."""
    lab = np.zeros((2, 5, 5), np.int32)
    lab[0, 2, 2] = 1
    w = OW.object_weights(lab, 3, 1)
    assert (w[1] == 1).all() and int((w[0] == 5).sum()) == 9
    w = OW.object_weights(lab, 3, 1, background=1)          # now class 0 is the object, class 1 background
    assert (w[1] == 5).all()
    assert (w[0] == 5).all()                                 # every pixel has a class-0 neighbour within 1


def test_ignore_index_inside_the_class_range_is_no_object():
    """An ignore value that is itself a class index (here 2 of 0 .. 4) marks nothing, alone or
    among objects; the same map with no ignore value marks around those pixels as well."""
    lab = np.zeros((1, 9, 12), np.int32)
    lab[0, 4, 3] = 2
    assert (OW.object_weights(lab, 5, 1, ignore_index=2) == 1).all()
    assert int((OW.object_weights(lab, 5, 1, ignore_index=-1) == 5).sum()) == 9
    lab[0, 4, 9] = 3
    w = OW.object_weights(lab, 5, 1, ignore_index=2)
    assert int((w == 5).sum()) == 9 and w[0, 4, 9] == 5 and w[0, 4, 3] == 1
    np.testing.assert_array_equal(w, brute_force(lab, 5, 1, 5, 0, 2))


def test_monotone_in_the_radius_and_asymmetric_extent():
    """A larger radius never clears a mark; a horizontal bar grows by r on every side."""
    lab = np.zeros((1, 21, 31), np.int32)
    lab[0, 10, 12:19] = 4
    prev = None
    for r in range(0, 6):
        w = OW.object_weights(lab, 6, r)[0] == 5
        ys, xs = np.nonzero(w)
        assert (ys.min(), ys.max(), xs.min(), xs.max()) == (10 - r, 10 + r, 12 - r, 18 + r)
        assert w.sum() == (2 * r + 1) * (7 + 2 * r)
        if prev is not None:
            assert (w | prev).sum() == w.sum()
        prev = w


def test_agrees_with_the_seeded_input_recipe():
    """The synthetic weight maps the workloads feed to the weighted-loss tests are this map with
    class 0 as background (the recipe builds it by repeated one-pixel dilations)."""
    wl = WL.small_variant(WL.WORKLOADS["720p"], h=12, w=20, n_sites=9)
    lab = WL.make_labels(wl)
    np.testing.assert_array_equal(OW.object_weights(lab, wl.n_classes, 4), WL.object_weight_map(lab, radius=4))

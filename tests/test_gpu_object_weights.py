"""GPU parity of st_object_weights (the loss-weight map of Section 5.2 from a label map) against
the CPU oracle: byte for byte, on shapes from a single pixel to the 1080p frame, widths that are
no multiple of the tile, of a 64-pixel word or of four, every radius class (0, small, the
maximum), ignored and out-of-range labels, several frames, another background class."""
import numpy as np
import pytest
import torch

import paper_2003_10735_amd as st
import workloads as WL
from oracle import object_weights as OW

pytestmark = pytest.mark.gpu


def sparse_labels(seed, n, H, W, n_classes, p_object, ignore_index=-1, p_ignore=0.0):
    rng = np.random.default_rng(seed)
    lab = np.zeros((n, H, W), np.int32)
    m = rng.random(lab.shape) < p_object
    lab[m] = rng.integers(1, n_classes, size=int(m.sum()))
    if p_ignore:
        lab[rng.random(lab.shape) < p_ignore] = ignore_index
    return lab


def run(lab, n_classes, radius, factor=5, background=0, ignore_index=-1):
    got = st.st_object_weights(torch.from_numpy(lab).cuda(), n_classes, radius, factor=factor, background=background,
                               ignore_index=ignore_index)
    torch.cuda.synchronize()
    want = OW.object_weights(lab, n_classes, radius, factor=factor, background=background, ignore_index=ignore_index)
    return got.cpu().numpy(), want


@pytest.mark.parametrize("n,H,W,radius", [
    (1, 1, 1, 4), (1, 1, 1, 0), (1, 3, 5, 32), (2, 16, 256, 3), (1, 17, 257, 3), (3, 37, 301, 1), (1, 37, 301, 0),
    (1, 20, 530, 7), (1, 50, 70, 32), (2, 33, 63, 9), (1, 64, 64, 16), (1, 15, 1023, 2), (1, 130, 258, 31)])
def test_shapes_and_radii(n, H, W, radius):
    lab = sparse_labels(1000 + H * W + radius, n, H, W, 9, 0.004, ignore_index=255, p_ignore=0.02)
    lab[0, 0, 0] = 3            # objects in the corners: their neighbourhoods are cut off at the edges
    lab[-1, -1, -1] = 2
    lab[0, H // 2, W // 2] = 11  # outside [0, n_classes): no object
    lab[0, H // 2, 0] = -7
    got, want = run(lab, 9, radius, ignore_index=255)
    np.testing.assert_array_equal(got, want)
    assert set(np.unique(got)) <= {1, 5}


def test_dense_objects_and_no_objects():
    lab = sparse_labels(5, 1, 40, 300, 5, 0.5)
    got, want = run(lab, 5, 2, factor=255)
    np.testing.assert_array_equal(got, want)
    got, want = run(np.zeros((2, 40, 300), np.int32), 5, 6)
    np.testing.assert_array_equal(got, want)
    assert (got == 1).all()


def test_background_class_and_factor():
    lab = sparse_labels(6, 2, 45, 130, 7, 0.01)
    lab[1] = 3
    lab[1, 20:24, 60:70] = 0
    got, want = run(lab, 7, 4, factor=9, background=3)
    np.testing.assert_array_equal(got, want)
    assert (got[1] == 9).sum() == (4 + 8) * (10 + 8)


def test_ignore_value_inside_the_class_range_and_first_non_class():
    lab = sparse_labels(9, 2, 30, 200, 6, 0.01)
    lab[0, 10, 50:60] = 2       # the ignore value, itself a class index: no object
    lab[1, 5, 5] = 6            # == n_classes: no class index, no object
    got, want = run(lab, 6, 3, ignore_index=2)
    np.testing.assert_array_equal(got, want)
    got2, want2 = run(lab, 6, 3, ignore_index=-1)
    np.testing.assert_array_equal(got2, want2)
    assert (got != got2).any()


def test_frames_do_not_leak_into_each_other():
    lab = np.zeros((3, 24, 280), np.int32)
    lab[1, 0, :] = 1            # top row of the middle frame
    lab[1, -1, :] = 1           # and its bottom row
    got, want = run(lab, 2, 5)
    np.testing.assert_array_equal(got, want)
    assert (got[0] == 1).all() and (got[2] == 1).all()


@pytest.mark.parametrize("name", ["720p", "1080p", "batch4"])
def test_the_workloads_label_maps(name):
    """The measured configurations' own label maps (Voronoi regions; 1080p with ignored pixels)."""
    wl = WL.WORKLOADS[name]
    lab = WL.make_labels(wl)
    got, want = run(lab, wl.n_classes, 4, ignore_index=wl.ignore_index)
    np.testing.assert_array_equal(got, want)


def test_unaligned_output_and_caller_buffer():
    """A result buffer that starts at an odd address takes the byte-wise stores; pixels outside
    the result are not written."""
    lab = sparse_labels(8, 2, 19, 100, 4, 0.01)
    buf = torch.full((2 * 19 * 100 + 9,), 77, dtype=torch.uint8, device="cuda")
    out = buf[3:3 + 2 * 19 * 100].view(2, 19, 100)
    st.st_object_weights(torch.from_numpy(lab).cuda(), 4, 3, weights=out)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(out.cpu().numpy(), OW.object_weights(lab, 4, 3))
    assert (buf[:3] == 77).all() and (buf[3 + 2 * 19 * 100:] == 77).all()


def test_weights_feed_the_training_call():
    """The map made on the device gives the training call the losses a host-made copy of the
    oracle's map gives it, bit for bit."""
    wl = WL.small_variant(WL.WORKLOADS["720p"], h=12, w=20, steps=2, n_sites=9)
    f, lab, p = WL.make_features(wl), WL.make_labels(wl), WL.make_head_params(wl)
    from gpu_util import to_dev_features
    desc = st.HeadDesc.of(wl)
    lab_d = torch.from_numpy(lab).cuda()
    outs = []
    for wts in (st.st_object_weights(lab_d, wl.n_classes, 4),
                torch.from_numpy(OW.object_weights(lab, wl.n_classes, 4)).cuda()):
        pt = torch.from_numpy(p).cuda()
        losses = torch.zeros(wl.steps + 1, dtype=torch.float32, device="cuda")
        st.st_partial_distill(desc, to_dev_features(wl, f), lab_d, pt, wl.steps, wl.lr, losses=losses, pixel_weights=wts)
        torch.cuda.synchronize()
        outs.append((losses.cpu().numpy(), pt.cpu().numpy()))
    np.testing.assert_array_equal(outs[0][0], outs[1][0])
    np.testing.assert_array_equal(outs[0][1], outs[1][1])

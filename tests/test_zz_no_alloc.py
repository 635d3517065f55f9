"""st_head_forward_noalloc -- the forward entry point for callers that cannot allocate -- against
st_head_forward on a caller's workspace: same kernels, so the low-resolution logits and the class
map must agree bit for bit.  Two calls in a row share the library's built-in scratch, the second
with a smaller input (it meets whatever the first one left there), then a float32 shape on the
plain kernels; a shape beyond the built-in scratch is refused before any GPU work."""
import ctypes as C

import numpy as np
import pytest
import torch

import paper_2003_10735_amd as st
import workloads as WL
from gpu_util import to_dev_features

pytestmark = pytest.mark.gpu


def both_ways(wl, seed):
    desc = st.HeadDesc.of(wl)
    f = to_dev_features(wl, WL.make_features(wl, seed=seed))
    p = torch.from_numpy(WL.make_head_params(wl, seed=seed + 1)).cuda()
    shape_z, shape_p = (wl.n, wl.n_classes, wl.h, wl.w), (wl.n, wl.H, wl.W)
    z_ref = torch.full(shape_z, float("nan"), dtype=torch.float32, device="cuda")
    q_ref = torch.full(shape_p, 255, dtype=torch.uint8, device="cuda")
    st.st_head_forward(desc, f, p, logits_lowres=z_ref, pred=q_ref, workspace=st.new_workspace(desc))
    z = torch.full(shape_z, float("nan"), dtype=torch.float32, device="cuda")
    q = torch.full(shape_p, 255, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    st.st_head_forward_noalloc(desc, f, p, logits_lowres=z, pred=q)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    np.testing.assert_array_equal(z.cpu().numpy(), z_ref.cpu().numpy())
    np.testing.assert_array_equal(q.cpu().numpy(), q_ref.cpu().numpy())
    assert np.isfinite(z_ref.cpu().numpy()).all() and int(q_ref.max()) < wl.n_classes
    assert len(np.unique(q_ref.cpu().numpy())) > 1            # a class map worth comparing
    # the class map alone (logits not asked for)
    q2 = torch.full(shape_p, 255, dtype=torch.uint8, device="cuda")
    st.st_head_forward_noalloc(desc, f, p, pred=q2)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(q2.cpu().numpy(), q_ref.cpu().numpy())


def test_two_calls_in_a_row_the_second_smaller():
    big = WL.WORKLOADS["720p"]
    assert st.st_workspace_bytes(st.HeadDesc.of(big)) <= st.ST_NOALLOC_MAX_WORKSPACE_MIB << 20
    both_ways(big, seed=41)
    small = WL.small_variant(big, h=12, w=40, c_in=64, c1=64, c2=64, n_classes=7)
    both_ways(small, seed=43)
    ragged = WL.small_variant(big, n=2, h=9, w=21, c_in=128, c1=64, c2=128, n_classes=21)
    both_ways(ragged, seed=45)
    both_ways(WL.WORKLOADS["tiny"], seed=47)                  # float32, the plain kernels
    both_ways(big, seed=49)                                   # and a large one again


def test_shapes_beyond_the_built_in_scratch_are_refused():
    wl = WL.WORKLOADS["1080p"]
    desc = st.HeadDesc.of(wl)
    assert st.st_workspace_bytes(desc) > st.ST_NOALLOC_MAX_WORKSPACE_MIB << 20
    d = desc.c()
    dummy = C.c_void_p(256)       # never dereferenced: the size check comes first
    assert st.lib().st_head_forward_noalloc(C.byref(d), dummy, dummy, None, None, None) == st.ST_ERR_TOO_LARGE
    assert b"scratch" in st.lib().st_strerror(st.ST_ERR_TOO_LARGE)

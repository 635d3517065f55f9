"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before any GPU work."""
import ctypes as C
import os
import re

import pytest

import paper_2003_10735_amd as st

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "shadowtutor_head.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(st_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = st.lib()
    names = declared_functions()
    assert set(st.EXPORTS) <= set(names)
    for n in names:
        assert hasattr(L, n), n


def good():
    return st.HeadDesc(1, 64, 16, 16, 64, 64, 9, st.ST_F32, st.ST_COMPUTE_F32)


def test_sizes():
    d = good()
    assert st.st_num_params(d) == 74441
    assert st.st_workspace_bytes(d) > 0
    d720 = st.HeadDesc(1, 256, 90, 160, 128, 128, 19)
    assert st.st_num_params(d720) == 445075
    lay = st.st_get_workspace_layout(d720)
    assert lay["total"] == st.st_workspace_bytes(d720) and lay["elem_size"] == 2
    assert st.st_version()


@pytest.mark.parametrize("field,value,status", [
    ("n", 0, st.ST_ERR_SHAPE), ("h", -1, st.ST_ERR_SHAPE), ("upscale", 4, st.ST_ERR_SHAPE),
    ("n_classes", 1, st.ST_ERR_SHAPE), ("n_classes", 33, st.ST_ERR_SHAPE),
    ("feat_dtype", 7, st.ST_ERR_ARG), ("compute", 2, st.ST_ERR_ARG), ("feat_layout", 2, st.ST_ERR_ARG),
    ("ignore_index", -2, st.ST_ERR_ARG), ("w", 1 << 24, st.ST_ERR_SHAPE),
])
def test_bad_descriptors_are_rejected_on_the_host(field, value, status):
    d = good()
    setattr(d, field, value)
    assert st.st_num_params(d) == 0 and st.st_workspace_bytes(d) == 0
    cd = d.c()
    dummy = C.c_void_p(256)       # never dereferenced: validation comes first
    L = st.lib()
    assert L.st_head_forward(C.byref(cd), dummy, dummy, None, None, dummy, None) == status
    assert L.st_partial_distill(C.byref(cd), dummy, dummy, dummy, 1, 0.1, None, None, dummy, None) == status


def test_grouped_descriptor_sizes_and_limits():
    """One head per frame: the per-head parameter count stays, the workspace holds n heads, and
    shapes off the matrix-core kernels are refused."""
    one = st.HeadDesc(4, 256, 90, 160, 128, 128, 19)
    grp = st.HeadDesc(4, 256, 90, 160, 128, 128, 19, grouped=1)
    assert st.st_num_params(grp) == st.st_num_params(one) == 445075
    extra = st.st_workspace_bytes(grp) - st.st_workspace_bytes(one)
    assert extra >= 3 * 445075 * 4 * 4            # theta, two state vectors, gradient copies of 3 more heads
    assert st.st_workspace_bytes(st.HeadDesc(1, 256, 90, 160, 128, 128, 19, grouped=1)) > 0
    # float32 compute, or channel counts the matrix-core kernels do not take
    assert st.st_workspace_bytes(st.HeadDesc(2, 64, 16, 16, 64, 64, 9, st.ST_F32, st.ST_COMPUTE_F32, grouped=1)) == 0
    assert st.st_workspace_bytes(st.HeadDesc(2, 20, 16, 16, 24, 16, 9, grouped=1)) == 0
    assert st.st_workspace_bytes(st.HeadDesc(2, 64, 16, 16, 64, 64, 9, grouped=2)) == 0


def test_null_and_argument_errors():
    L = st.lib()
    cd = good().c()
    dummy = C.c_void_p(256)
    assert L.st_head_forward(None, dummy, dummy, None, None, dummy, None) == st.ST_ERR_NULL
    assert L.st_head_forward(C.byref(cd), None, dummy, None, None, dummy, None) == st.ST_ERR_NULL
    assert L.st_head_forward(C.byref(cd), dummy, dummy, None, None, None, None) == st.ST_ERR_WORKSPACE
    assert L.st_head_forward(C.byref(cd), dummy, dummy, None, None, C.c_void_p(264), None) == st.ST_ERR_WORKSPACE
    pd = L.st_partial_distill
    assert pd(C.byref(cd), dummy, None, dummy, 1, 0.1, None, None, dummy, None) == st.ST_ERR_NULL
    assert pd(C.byref(cd), dummy, dummy, dummy, -1, 0.1, None, None, dummy, None) == st.ST_ERR_ARG
    assert pd(C.byref(cd), dummy, dummy, dummy, 1, float("nan"), None, None, dummy, None) == st.ST_ERR_ARG
    assert pd(C.byref(cd), dummy, dummy, dummy, 1, float("inf"), None, None, dummy, None) == st.ST_ERR_ARG
    opts = st.StDistillOpts(0.9, None, 0.0, 1, 0)
    assert pd(C.byref(cd), dummy, dummy, dummy, 1, 0.1, C.byref(opts), None, dummy, None) == st.ST_ERR_NULL
    opts = st.StDistillOpts(float("nan"), dummy, 0.0, 1, 0)
    assert pd(C.byref(cd), dummy, dummy, dummy, 1, 0.1, C.byref(opts), None, dummy, None) == st.ST_ERR_ARG
    # Adam: state arrays required, no momentum, constants in range
    def adam_opts(**kw):
        o = st.StDistillOpts(0.0, None, 0.0, 1, 0, st.ST_OPTIM_ADAM, 0.9, 0.999, 1e-8, dummy, dummy, 0)
        for k, v in kw.items():
            setattr(o, k, v)
        return o
    for kw, status in (({"adam_m": None}, st.ST_ERR_NULL), ({"adam_v": None}, st.ST_ERR_NULL),
                       ({"momentum": 0.5, "velocity": dummy}, st.ST_ERR_ARG), ({"beta1": 1.0}, st.ST_ERR_ARG),
                       ({"beta2": -0.1}, st.ST_ERR_ARG), ({"eps": 0.0}, st.ST_ERR_ARG),
                       ({"adam_t0": -1}, st.ST_ERR_ARG), ({"optimizer": 2}, st.ST_ERR_ARG)):
        o = adam_opts(**kw)
        assert pd(C.byref(cd), dummy, dummy, dummy, 1, 0.1, C.byref(o), None, dummy, None) == status, kw
    assert L.st_miou(None, dummy, 10, 3, -1, dummy, dummy, None) == st.ST_ERR_NULL
    assert L.st_miou(dummy, dummy, -1, 3, -1, dummy, dummy, None) == st.ST_ERR_SHAPE
    assert L.st_miou(None, None, 0, 3, -1, None, dummy, None) == st.ST_ERR_NULL
    assert L.st_miou(dummy, dummy, 10, 0, -1, dummy, dummy, None) == st.ST_ERR_SHAPE
    assert L.st_get_workspace_layout(C.byref(cd), None) == st.ST_ERR_NULL
    # the forward entry point on the built-in scratch validates in the same order, then the size
    na = L.st_head_forward_noalloc
    assert na(None, dummy, dummy, None, None, None) == st.ST_ERR_NULL
    assert na(C.byref(cd), None, dummy, None, None, None) == st.ST_ERR_NULL
    big = st.HeadDesc(1, 256, 135, 240, 128, 128, 19).c()
    assert na(C.byref(big), dummy, dummy, None, None, None) == st.ST_ERR_TOO_LARGE
    # the loss-weight map: shape, then value arguments, then pointers
    ow = L.st_object_weights
    assert ow(dummy, 0, 8, 8, 19, 0, -1, 4, 5, dummy, None) == st.ST_ERR_SHAPE
    assert ow(dummy, 1, 8, 0, 19, 0, -1, 4, 5, dummy, None) == st.ST_ERR_SHAPE
    assert ow(dummy, 70000, 8, 8, 19, 0, -1, 4, 5, dummy, None) == st.ST_ERR_SHAPE
    assert ow(dummy, 1, 8, 8, 0, 0, -1, 4, 5, dummy, None) == st.ST_ERR_SHAPE
    assert ow(dummy, 1, 8, 8, 19, 0, -1, -1, 5, dummy, None) == st.ST_ERR_ARG
    assert ow(dummy, 1, 8, 8, 19, 0, -1, st.ST_OBJECT_WEIGHTS_MAX_RADIUS + 1, 5, dummy, None) == st.ST_ERR_ARG
    assert ow(dummy, 1, 8, 8, 19, 0, -1, 4, 0, dummy, None) == st.ST_ERR_ARG
    assert ow(dummy, 1, 8, 8, 19, 0, -1, 4, 256, dummy, None) == st.ST_ERR_ARG
    assert ow(None, 1, 8, 8, 19, 0, -1, 4, 5, dummy, None) == st.ST_ERR_NULL
    assert ow(dummy, 1, 8, 8, 19, 0, -1, 4, 5, None, None) == st.ST_ERR_NULL
    for s in (0, -1, -2, -3, -4, -5, -6, -7, -99):
        assert L.st_strerror(s)


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2003_10735_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".hpp", ".h", ".cpp")):
                text = open(os.path.join(dirpath, fn)).read()
                assert "oracle" not in text.replace("no CPU fallback", ""), os.path.join(dirpath, fn)


def test_bench_refuses_more_than_one_gpu():
    """The library runs on one GPU: asked for more, the benchmark says so and stops before it
    touches a device."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stdout + r.stderr)

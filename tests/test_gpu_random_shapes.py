"""GPU parity on seeded random shapes of the matrix-core path: channel counts, grid sizes from a
single cell to several position tiles, 1 to 4 frames, one shared head or one head per frame,
2 to 32 classes, with and without ignored pixels and momentum -- each against the oracle's
bf16-operand mode (same rounding points: what is left is the order of additions)."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2003_10735_amd as st
import workloads as WL
from gpu_util import progress, rel_err, to_dev_features

pytestmark = pytest.mark.gpu


def random_case(seed):
    rng = np.random.default_rng(seed)
    cfg = dict(n=int(rng.integers(1, 5)), c_in=int(rng.choice([64, 128, 192, 256])), c1=int(rng.choice([64, 128])),
               c2=int(rng.choice([64, 128, 256])), h=int(rng.integers(1, 25)), w=int(rng.integers(1, 46)),
               n_classes=int(rng.integers(2, 33)))
    ignore = bool(rng.integers(0, 2))
    wl = WL.small_variant(WL.WORKLOADS["720p"], steps=int(rng.integers(1, 4)), lr=0.02, n_sites=int(rng.integers(2, 12)),
                          feat_seed=int(rng.integers(1, 10 ** 6)), label_seed=int(rng.integers(1, 10 ** 6)),
                          init_seed=int(rng.integers(1, 10 ** 6)), momentum=0.9 if rng.integers(0, 2) else 0.0,
                          ignore_index=255 if ignore else -1, ignore_fraction=0.1 if ignore else 0.0, **cfg)
    return wl, int(rng.integers(0, 2))


def check_updates(p0, pt, vel, o, wl):
    """The weights are dominated by their initial values, so the update itself (and the velocity)
    is compared as well: a wrong weight or bias gradient on an odd shape shows up here, block by
    block (W1, b1, W2, b2, W3, b3 of every head), each relative to its own largest entry."""
    got = pt.cpu().numpy().astype(np.float64).reshape(-1, wl.n_params)
    want = np.asarray(o["params"]).reshape(-1, wl.n_params)
    start = np.asarray(p0, dtype=np.float64).reshape(-1, wl.n_params)
    worst = 0.0
    for name, sl in WL.param_slices(wl).items():
        for hd in range(got.shape[0]):
            du = want[hd, sl] - start[hd, sl]
            if np.abs(du).max() < 1e-9:
                continue
            e = rel_err(got[hd, sl] - start[hd, sl], du)
            worst = max(worst, e)
            assert e < 3e-2, (name, hd)
    progress(f"update error random shape {wl.c_in}->{wl.c1}->{wl.c2}->{wl.n_classes} {wl.n}x{wl.h}x{wl.w}: {worst:.3g}")
    if vel is not None:
        v, vo = vel.cpu().numpy().reshape(-1, wl.n_params), np.asarray(o["s1"]).reshape(-1, wl.n_params)
        for name, sl in WL.param_slices(wl).items():
            for hd in range(v.shape[0]):
                if np.abs(vo[hd, sl]).max() < 1e-9:
                    continue
                assert rel_err(v[hd, sl], vo[hd, sl]) < 3e-2, (name, hd)


@pytest.mark.parametrize("seed", range(100, 116))
def test_random_shape(seed):
    wl, grouped = random_case(seed)
    heads = wl.n if grouped else 1
    f, lab = WL.make_features(wl), WL.make_labels(wl)
    p = np.stack([WL.make_head_params(wl, seed=wl.init_seed + 17 * i) for i in range(heads)]).astype(np.float32)
    desc = st.HeadDesc.of(wl)
    desc.grouped = grouped
    print(wl, "grouped", grouped)
    pt = torch.from_numpy(p if grouped else p[0]).cuda()
    vel = torch.zeros_like(pt) if wl.momentum else None
    losses = torch.zeros((wl.steps + 1, heads) if grouped else (wl.steps + 1,), dtype=torch.float32, device="cuda")
    mious = torch.zeros((wl.steps + 1, wl.n), dtype=torch.float64, device="cuda")
    conf = torch.zeros((wl.n, wl.n_classes, wl.n_classes), dtype=torch.int64, device="cuda")
    st.st_partial_distill(desc, to_dev_features(wl, f), torch.from_numpy(lab).cuda(), pt, wl.steps, wl.lr,
                          momentum=wl.momentum, velocity=vel, losses=losses, mious=mious, confusion=conf)
    torch.cuda.synchronize()
    d = O.desc_of(wl, True)
    opt = O.Optim(0, wl.lr, wl.momentum, 0, 0, 0, 0)
    f64 = WL.features_as_f64(wl, f)
    if grouped:
        o = O.partial_distill_grouped(d, f64, lab, p.astype(np.float64), wl.steps, opt)
    else:
        o = O.partial_distill_opt(d, f64, lab, p[0].astype(np.float64), wl.steps, opt)
    assert rel_err(losses.cpu().numpy(), o["losses"]) < 5e-4
    assert rel_err(pt.cpu().numpy(), o["params"]) < 5e-4
    check_updates(p if grouped else p[0], pt, vel, o, wl)
    np.testing.assert_allclose(mious.cpu().numpy(), o["mious"], atol=2e-2)
    # every valid pixel is counted exactly once
    valid = (lab != wl.ignore_index).reshape(wl.n, -1).sum(axis=1)
    np.testing.assert_array_equal(conf.cpu().numpy().sum(axis=(1, 2)), valid)


@pytest.mark.parametrize("seed", range(200, 208))
def test_random_shape_with_pixel_weights(seed):
    """The same random shapes with a random per-pixel weight map (0 .. 5, zeros included: such
    pixels count for nothing, like ignored ones, but stay in the confusion counts)."""
    wl, grouped = random_case(seed)
    heads = wl.n if grouped else 1
    rng = np.random.default_rng(seed + 5000)
    f, lab = WL.make_features(wl), WL.make_labels(wl)
    wts = rng.integers(0, 6, size=lab.shape).astype(np.uint8)
    p = np.stack([WL.make_head_params(wl, seed=wl.init_seed + 17 * i) for i in range(heads)]).astype(np.float32)
    desc = st.HeadDesc.of(wl)
    desc.grouped = grouped
    print(wl, "grouped", grouped)
    pt = torch.from_numpy(p if grouped else p[0]).cuda()
    vel = torch.zeros_like(pt) if wl.momentum else None
    losses = torch.zeros((wl.steps + 1, heads) if grouped else (wl.steps + 1,), dtype=torch.float32, device="cuda")
    conf = torch.zeros((wl.n, wl.n_classes, wl.n_classes), dtype=torch.int64, device="cuda")
    st.st_partial_distill(desc, to_dev_features(wl, f), torch.from_numpy(lab).cuda(), pt, wl.steps, wl.lr,
                          momentum=wl.momentum, velocity=vel, losses=losses, confusion=conf,
                          pixel_weights=torch.from_numpy(wts).cuda())
    torch.cuda.synchronize()
    d = O.desc_of(wl, True)
    opt = O.Optim(0, wl.lr, wl.momentum, 0, 0, 0, 0)
    f64 = WL.features_as_f64(wl, f)
    if grouped:
        o = O.partial_distill_grouped(d, f64, lab, p.astype(np.float64), wl.steps, opt, pixel_weights=wts)
    else:
        o = O.partial_distill_opt(O.with_pixel_weights(d, wts), f64, lab, p[0].astype(np.float64), wl.steps, opt)
    assert rel_err(losses.cpu().numpy(), o["losses"]) < 5e-4
    assert rel_err(pt.cpu().numpy(), o["params"]) < 5e-4
    check_updates(p if grouped else p[0], pt, vel, o, wl)
    valid = (lab != wl.ignore_index).reshape(wl.n, -1).sum(axis=1)
    np.testing.assert_array_equal(conf.cpu().numpy().sum(axis=(1, 2)), valid)

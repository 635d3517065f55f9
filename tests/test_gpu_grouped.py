"""GPU parity of the grouped mode: n clients, each with a head of its own and one key frame, trained
in one call (the server of Algorithm 3 keeps one student per client).  By definition head f's
result is that of a single-frame run on frame f alone; the oracle side is exactly that loop."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2003_10735_amd as st
import workloads as WL
from gpu_util import rel_err, to_dev_features

pytestmark = pytest.mark.gpu

SGD = lambda wl: O.Optim(0, wl.lr, wl.momentum, 0, 0, 0, 0)


def inputs(wl):
    """Per-frame features and labels, and a different initial head per client."""
    f, lab = WL.make_features(wl), WL.make_labels(wl)
    p = np.stack([WL.make_head_params(wl, seed=wl.init_seed + 17 * i) for i in range(wl.n)])
    return f, lab, p


def run_grouped(wl, feats, labels, params, steps, adam=False, weights=None, s1=None, s2=None, t0=0):
    desc = st.HeadDesc.of(wl)
    desc.grouped = 1
    n, P = params.shape
    assert P == st.st_num_params(desc)
    p = torch.from_numpy(params.astype(np.float32)).cuda()
    z32 = lambda a: torch.from_numpy((a if a is not None else np.zeros_like(params)).astype(np.float32)).cuda()
    vel = z32(s1) if (wl.momentum != 0.0 and not adam) else None
    am = dict(m=z32(s1), v=z32(s2), t0=t0) if adam else None
    losses = torch.full((steps + 1, n), float("nan"), dtype=torch.float32, device="cuda")
    mious = torch.full((steps + 1, n), float("nan"), dtype=torch.float64, device="cuda")
    conf = torch.zeros((n, wl.n_classes, wl.n_classes), dtype=torch.int64, device="cuda")
    pred = torch.zeros((n, wl.H, wl.W), dtype=torch.uint8, device="cuda")
    taken, _ = st.st_partial_distill(desc, to_dev_features(wl, feats), torch.from_numpy(labels).cuda(), p, steps,
                                     wl.lr, momentum=0.0 if adam else wl.momentum, velocity=vel, losses=losses,
                                     mious=mious, confusion=conf, pred=pred, adam=am,
                                     pixel_weights=None if weights is None else torch.from_numpy(weights).cuda())
    torch.cuda.synchronize()
    assert taken == steps
    out = dict(params=p.cpu().numpy(), losses=losses.cpu().numpy(), mious=mious.cpu().numpy(),
               conf=conf.cpu().numpy(), pred=pred.cpu().numpy())
    if vel is not None:
        out["s1"] = vel.cpu().numpy()
    if adam:
        out["s1"], out["s2"] = am["m"].cpu().numpy(), am["v"].cpu().numpy()
    return out


def run_single(wl, feats, labels, params, steps, f):
    """Head f alone, through the one-head form of the same entry point."""
    wl1 = WL.small_variant(wl, n=1)
    desc = st.HeadDesc.of(wl1)
    p = torch.from_numpy(params[f].astype(np.float32)).cuda()
    vel = torch.zeros_like(p) if wl.momentum != 0.0 else None
    losses = torch.full((steps + 1,), float("nan"), dtype=torch.float32, device="cuda")
    mious = torch.full((steps + 1, 1), float("nan"), dtype=torch.float64, device="cuda")
    conf = torch.zeros((1, wl.n_classes, wl.n_classes), dtype=torch.int64, device="cuda")
    pred = torch.zeros((1, wl.H, wl.W), dtype=torch.uint8, device="cuda")
    st.st_partial_distill(desc, to_dev_features(wl1, feats[f:f + 1]), torch.from_numpy(labels[f:f + 1]).cuda(), p,
                          steps, wl.lr, momentum=wl.momentum, velocity=vel, losses=losses, mious=mious,
                          confusion=conf, pred=pred)
    torch.cuda.synchronize()
    return dict(params=p.cpu().numpy(), losses=losses.cpu().numpy(), mious=mious.cpu().numpy()[:, 0],
                conf=conf.cpu().numpy()[0], pred=pred.cpu().numpy()[0])


def check_against_oracle(wl, g, o, p, tol_q=5e-4):
    for f in range(wl.n):
        assert rel_err(g["losses"][:, f], o["losses"][:, f]) < tol_q, f
        assert rel_err(g["params"][f], o["params"][f]) < tol_q, f
        assert rel_err(g["params"][f] - p[f], o["params"][f] - p[f]) < 3e-2, f
    np.testing.assert_allclose(g["mious"], o["mious"], atol=5e-3)


# frame sizes (h + 2) * pitch: 11 * 40 = 440 = 8 * 55 (an odd number of 8-position groups: a head's
# last 16-position unit reaches into the next frame), 19 * 16 = 304, 5 * 8 = 40 (less than one tile)
GROUPED_CASES = [
    dict(n=3, c_in=64, h=9, w=35, c1=64, c2=64, n_classes=6),
    dict(n=2, c_in=64, h=17, w=9, c1=64, c2=128, n_classes=21, ignore_index=255, ignore_fraction=0.05,
         momentum=0.9),
    dict(n=5, c_in=64, h=3, w=5, c1=128, c2=64, n_classes=4),
    dict(n=4, c_in=128, h=20, w=28, c1=64, c2=64, n_classes=19),
]


@pytest.mark.parametrize("case", range(len(GROUPED_CASES)))
def test_grouped_heads_match_the_oracle_head_by_head(case):
    wl = WL.small_variant(WL.WORKLOADS["720p"], steps=3, lr=0.02, n_sites=9, **GROUPED_CASES[case])
    f, lab, p = inputs(wl)
    g = run_grouped(wl, f, lab, p, 3)
    f64 = WL.features_as_f64(wl, f)
    orq = O.partial_distill_grouped(O.desc_of(wl, True), f64, lab, p.astype(np.float64), 3, SGD(wl))
    ora = O.partial_distill_grouped(O.desc_of(wl, False), f64, lab, p.astype(np.float64), 3, SGD(wl))
    check_against_oracle(wl, g, orq, p)
    for fi in range(wl.n):
        assert rel_err(g["losses"][:, fi], ora["losses"][:, fi]) < 2e-2
        assert rel_err(g["params"][fi], ora["params"][fi]) < 2e-2
    if wl.momentum:
        assert rel_err(g["s1"], orq["s1"]) < 3e-2
    # the heads do differ (different frames, different initial weights)
    assert not np.array_equal(g["params"][0], g["params"][1])
    # run twice: bit-identical
    again = run_grouped(wl, f, lab, p, 3)
    for k in ("params", "losses", "mious", "conf", "pred"):
        np.testing.assert_array_equal(g[k], again[k])


def test_grouped_equals_single_head_calls():
    """Head f of a grouped call against the one-head call on frame f alone: the same kernels on the
    same tiles; only the number of position splits of the weight gradient may differ."""
    wl = WL.small_variant(WL.WORKLOADS["720p"], steps=2, lr=0.02, n_sites=9, n=3, c_in=64, h=9, w=35, c1=64,
                          c2=64, n_classes=6, momentum=0.9)
    f, lab, p = inputs(wl)
    g = run_grouped(wl, f, lab, p, 2)
    for fi in range(wl.n):
        s = run_single(wl, f, lab, p, 2, fi)
        # the first forward pass involves no reduction whose order could differ
        assert g["losses"][0, fi] == s["losses"][0]
        assert g["mious"][0, fi] == s["mious"][0]
        assert rel_err(g["params"][fi], s["params"]) < 1e-5
        assert rel_err(g["params"][fi] - p[fi], s["params"] - p[fi]) < 1e-3
        assert rel_err(g["losses"][:, fi], s["losses"]) < 1e-5


def test_grouped_confusion_and_class_maps_bit_exact_from_own_logits():
    wl = WL.small_variant(WL.WORKLOADS["720p"], steps=1, lr=0.02, n_sites=9, n=3, c_in=64, h=9, w=35, c1=64,
                          c2=64, n_classes=6, ignore_index=255, ignore_fraction=0.1)
    f, lab, p = inputs(wl)
    desc = st.HeadDesc.of(wl)
    desc.grouped = 1
    pt = torch.from_numpy(p.astype(np.float32)).cuda()
    mious = torch.zeros((2, wl.n), dtype=torch.float64, device="cuda")
    conf = torch.zeros((wl.n, wl.n_classes, wl.n_classes), dtype=torch.int64, device="cuda")
    pred = torch.zeros((wl.n, wl.H, wl.W), dtype=torch.uint8, device="cuda")
    st.st_partial_distill(desc, to_dev_features(wl, f), torch.from_numpy(lab).cuda(), pt, 1, wl.lr, mious=mious,
                          confusion=conf, pred=pred)
    # the logits of the updated heads, through the grouped forward
    z = torch.zeros((wl.n, wl.n_classes, wl.h, wl.w), dtype=torch.float32, device="cuda")
    pred2 = torch.zeros_like(pred)
    st.st_head_forward(desc, to_dev_features(wl, f), pt, z, pred2)
    torch.cuda.synchronize()
    assert torch.equal(pred, pred2)
    pred_o = O.predict_from_logits(z.cpu().numpy())
    np.testing.assert_array_equal(pred.cpu().numpy(), pred_o)
    for i in range(wl.n):
        conf_o = O.confusion(pred_o[i], lab[i], wl.n_classes, wl.ignore_index)
        np.testing.assert_array_equal(conf[i].cpu().numpy(), conf_o)
        assert mious[1, i].item() == O.miou(conf_o)[0]


def test_grouped_adam_and_weighted_loss():
    wl = WL.small_variant(WL.WORKLOADS["720p"], steps=3, lr=0.01, n_sites=6, n=3, c_in=64, h=12, w=20, c1=64,
                          c2=64, n_classes=7)
    f, lab, p = inputs(wl)
    wts = WL.object_weight_map(lab, radius=4)
    f64 = WL.features_as_f64(wl, f)
    d = O.desc_of(wl, True)
    # weighted cross-entropy, plain descent
    g = run_grouped(wl, f, lab, p, 3, weights=wts)
    o = O.partial_distill_grouped(d, f64, lab, p.astype(np.float64), 3, SGD(wl), pixel_weights=wts)
    check_against_oracle(wl, g, o, p)
    plain = run_grouped(wl, f, lab, p, 3)
    assert np.all(np.abs(g["losses"][0] - plain["losses"][0]) > 1e-4)
    # Adam: parity where the first gradient is not tiny (the update is close to a sign function
    # of the gradient elsewhere), the second moments everywhere
    g = run_grouped(wl, f, lab, p, 3, adam=True)
    o = O.partial_distill_grouped(d, f64, lab, p.astype(np.float64), 3, O.adam_optim(wl.lr))
    for fi in range(wl.n):
        d1 = O.desc(1, wl.c_in, wl.h, wl.w, wl.c1, wl.c2, wl.n_classes, wl.ignore_index, True)
        _, g0, *_ = O.loss_and_grad(d1, f64[fi:fi + 1], lab[fi:fi + 1], p[fi].astype(np.float64))
        solid = np.abs(g0) > 1e-3 * np.abs(g0).max()
        scale = np.abs(o["params"][fi]).max()
        assert np.max(np.abs(g["params"][fi] - o["params"][fi])[solid]) <= 2e-2 * scale
        assert rel_err(g["s2"][fi], o["s2"][fi]) <= 2e-2
        np.testing.assert_allclose(g["losses"][:, fi], o["losses"][:, fi], rtol=2e-3, atol=2e-3)


def test_grouped_rejects_what_it_does_not_do():
    wl = WL.small_variant(WL.WORKLOADS["720p"], steps=1, n=2, c_in=64, h=4, w=4, c1=64, c2=64, n_classes=3)
    f, lab, p = inputs(wl)
    desc = st.HeadDesc.of(wl)
    desc.grouped = 1
    pt = torch.from_numpy(p.astype(np.float32)).cuda()
    args = (to_dev_features(wl, f), torch.from_numpy(lab).cuda(), pt, 1, 0.01)
    with pytest.raises(st.StError) as e:
        st.st_partial_distill(desc, *args, threshold=0.5)
    assert e.value.status == st.ST_ERR_ARG
    with pytest.raises(st.StError) as e:
        st.st_partial_distill(desc, *args, feature_grad=torch.zeros((2, 64, 4, 4), device="cuda"))
    assert e.value.status == st.ST_ERR_ARG
    torch.cuda.synchronize()
    np.testing.assert_array_equal(pt.cpu().numpy(), p.astype(np.float32))

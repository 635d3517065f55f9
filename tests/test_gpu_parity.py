"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Bars: bit-exact for class maps, confusion counts and mean IoU (from the same
low-resolution logits); 1e-4 relative for the float32 path; 2e-2 relative against the plain
oracle for the bfloat16 path (and a tighter bar against the oracle's bf16-operand mode, where
only the accumulation order differs)."""
import numpy as np
import pytest
import torch

import oracle as O
import paper_2003_10735_amd as st
import workloads as WL
from gpu_util import (check_pred_against_oracle, check_staged_bit_exact, rel_err, run_gpu, run_oracle,
                      progress, to_dev_features, update_err)

pytestmark = pytest.mark.gpu


def inputs(wl):
    return WL.make_features(wl), WL.make_labels(wl), WL.make_head_params(wl)


def test_tiny_f32_end_to_end():
    wl = WL.WORKLOADS["tiny"]
    f, lab, p = inputs(wl)
    gpu = run_gpu(wl, f, lab, p)
    ora = run_oracle(wl, f, lab, p)
    print("losses gpu", gpu["losses"], "oracle", ora["losses"], "miou", gpu["mious"].ravel())
    assert gpu["steps_taken"] == wl.steps
    assert rel_err(gpu["losses"], ora["losses"]) < 1e-4
    assert rel_err(gpu["params"], ora["params"]) < 1e-4
    assert rel_err(gpu["params"] - p, ora["params"] - p) < 1e-3      # the update itself
    check_staged_bit_exact(wl, gpu, lab)
    np.testing.assert_allclose(gpu["mious"], ora["mious"], atol=2e-3)
    check_pred_against_oracle(wl, gpu, ora, f, logit_tol=1e-4)


RAGGED = [
    dict(n=1, c_in=8, h=5, w=7, c1=8, c2=8, n_classes=3),
    dict(n=2, c_in=20, h=9, w=37, c1=24, c2=16, n_classes=5, ignore_index=255, ignore_fraction=0.1),
    dict(n=1, c_in=16, h=3, w=70, c1=16, c2=40, n_classes=21, momentum=0.9),
    dict(n=3, c_in=4, h=1, w=1, c1=4, c2=4, n_classes=2),
    # enough positions (2 x 33 x 37 = 2442) for the plain path's largest number of partial gradient
    # copies (16), with a ragged last share
    dict(n=2, c_in=12, h=33, w=37, c1=16, c2=12, n_classes=4, momentum=0.5),
]


@pytest.mark.parametrize("compute", ["f32", "bf16"])
@pytest.mark.parametrize("case", range(len(RAGGED)))
def test_ragged_shapes(case, compute):
    wl = WL.small_variant(WL.WORKLOADS["tiny"], steps=3, lr=0.05, compute=compute,
                          feat_dtype="bf16" if compute == "bf16" else "f32", n_sites=7, **RAGGED[case])
    f, lab, p = inputs(wl)
    gpu = run_gpu(wl, f, lab, p)
    check_staged_bit_exact(wl, gpu, lab)
    if compute == "f32":
        ora = run_oracle(wl, f, lab, p)
        assert rel_err(gpu["losses"], ora["losses"]) < 1e-4
        assert rel_err(gpu["params"], ora["params"]) < 1e-4
        assert rel_err(gpu["params"] - p, ora["params"] - p) < 2e-3
        if wl.momentum:
            assert rel_err(gpu["velocity"], ora["velocity"]) < 2e-3
    else:
        ora = run_oracle(wl, f, lab, p, bf16_operands=False)
        orq = run_oracle(wl, f, lab, p, bf16_operands=True)
        assert rel_err(gpu["losses"], ora["losses"]) < 2e-2
        assert rel_err(gpu["params"], ora["params"]) < 2e-2
        # against the oracle that rounds the same operands: accumulation order only
        assert rel_err(gpu["losses"], orq["losses"]) < 2e-4
        assert rel_err(gpu["params"], orq["params"]) < 2e-4
        assert update_err(f"ragged {case} bf16", gpu["params"] - p, orq["params"] - p) < 2e-2


def test_intermediate_gradient_buffers_f32():
    """d loss / d z and the parameter gradient of one step, read back from the workspace."""
    wl = WL.small_variant(WL.WORKLOADS["tiny"], steps=1, c_in=8, h=16, w=40, c1=8, c2=8, n_classes=4,
                          n_sites=6, lr=0.0)
    f, lab, p = inputs(wl)
    gpu = run_gpu(wl, f, lab, p)
    assert max(gpu["layout"]["splits"]) > 1          # the weight gradients arrive as partial copies
    d = O.desc_of(wl)
    f64 = WL.features_as_f64(wl, f)
    loss, grad, *_ = O.loss_and_grad(d, f64, lab, p.astype(np.float64))
    z, _ = O.head_forward(d, f64, p.astype(np.float64), want_pred=False)
    _, G, _ = O.softmax_ce(O.upsample8(z), lab)
    g = O.upsample8_adjoint(G)
    lay, ws = gpu["layout"], gpu["workspace"]
    gz = ws[lay["g"]:lay["g"] + 4 * g.size].view(torch.float32).cpu().numpy().reshape(g.shape)
    assert rel_err(gz, g) < 1e-5
    # gradient in the internal order: 3x3 weights as [o][kh][kw][i]
    n = p.size
    copies = ws[lay["grad"]:lay["grad"] + 4 * lay["grad_copies"] * lay["grad_stride"]].view(torch.float32).cpu().numpy()
    copies = copies.reshape(lay["grad_copies"], lay["grad_stride"])[:, :n].astype(np.float64)
    sl = WL.param_slices(wl)
    gi = np.zeros(n)
    for name in sl:                              # each block of parameters: the sum of its layer's copies
        layer = {"W1": 0, "b1": 0, "W2": 1, "b2": 1, "W3": 2, "b3": 2}[name]
        gi[sl[name]] = copies[:lay["splits"][layer], sl[name]].sum(axis=0)
    ref = grad.copy()
    for name, (co, ci) in (("W1", (wl.c1, wl.c_in)), ("W2", (wl.c2, wl.c1))):
        ref[sl[name]] = grad[sl[name]].reshape(co, ci, 3, 3).transpose(0, 2, 3, 1).ravel()
    for name in sl:
        assert rel_err(gi[sl[name]], ref[sl[name]]) < 1e-4, name
    assert abs(gpu["losses"][0] - loss) < 1e-5 * loss
    np.testing.assert_array_equal(gpu["params"], p)      # lr = 0 leaves the parameters alone


def test_intermediate_tensors_of_the_bf16_path_element_by_element():
    """The matrix-core path's own tensors after one step with a zero learning rate, read back from
    the workspace: both activations and both back-propagated gradients (stored as bfloat16),
    against a replay with the oracle's primitives that rounds where the
    bf16 path is defined to round (weights, a1, a2, the logit gradient, da2, da1).  Both sides
    round the same sums, added in different orders, so nearly every element must agree to the
    bit, the rest by one bfloat16 step (a sum that falls on the other side of a rounding
    boundary), and an element may be zero on one side only where a ReLU input is within rounding
    of zero.  A truncating conversion, a missing ReLU mask or a shifted layout would fail this by
    orders of magnitude."""
    wl = WL.small_variant(WL.WORKLOADS["720p"], n=2, c_in=64, h=9, w=21, c1=64, c2=128, n_classes=7, steps=1, lr=0.0,
                          n_sites=9, ignore_index=255, ignore_fraction=0.05)
    f, lab, p = inputs(wl)
    desc = st.HeadDesc.of(wl)
    ws = st.new_workspace(desc)
    # (with the feature gradient asked for, the gradient behind layer 1 is also left position-major)
    dfeat = torch.zeros((wl.n, wl.c_in, wl.h, wl.w), dtype=torch.float32, device="cuda")
    st.st_partial_distill(desc, to_dev_features(wl, f), torch.from_numpy(lab).cuda(), torch.from_numpy(p).cuda(), 1, 0.0,
                          workspace=ws, feature_grad=dfeat)
    torch.cuda.synchronize()
    lay = st.st_get_workspace_layout(desc)
    assert lay["elem_size"] == 2

    def grid(off, C):          # [n, h+2, row_pitch, C] bfloat16 -> [n, C, h, w] float64 (inside the zero border)
        Hp, Wp = wl.h + 2, lay["row_pitch"]
        t = ws[off:off + 2 * wl.n * Hp * Wp * C].view(torch.bfloat16).reshape(wl.n, Hp, Wp, C)
        inner = t[:, 1:wl.h + 1, 1:wl.w + 1, :].float().cpu().numpy().astype(np.float64)
        border = t.float().clone()
        border[:, 1:wl.h + 1, 1:wl.w + 1, :] = 0
        assert float(border.abs().max()) == 0.0          # the padding stays zero
        return inner.transpose(0, 3, 1, 2)

    sl = WL.param_slices(wl)
    p64 = p.astype(np.float64)
    W1 = O.round_bf16(p64[sl["W1"]].reshape(wl.c1, wl.c_in, 3, 3))
    W2 = O.round_bf16(p64[sl["W2"]].reshape(wl.c2, wl.c1, 3, 3))
    W3 = O.round_bf16(p64[sl["W3"]].reshape(wl.n_classes, wl.c2, 1, 1))
    x = WL.features_as_f64(wl, f)
    pre1 = O.conv_fwd(x, W1, p64[sl["b1"]])
    a1 = O.round_bf16(np.maximum(pre1, 0.0))
    pre2 = O.conv_fwd(a1, W2, p64[sl["b2"]])
    a2 = O.round_bf16(np.maximum(pre2, 0.0))
    z = O.conv_fwd(a2, W3, p64[sl["b3"]])
    _, G, _ = O.softmax_ce(O.upsample8(z), lab, wl.ignore_index)
    g = O.upsample8_adjoint(G)
    da2 = O.round_bf16(O.conv_dgrad(O.round_bf16(g), W3) * (a2 > 0))
    da1 = O.round_bf16(O.conv_dgrad(da2, W2) * (a1 > 0))

    def compare(name, got, want, exact_share, first_layer=False):
        ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(want), 1e-300))) - 7)      # one bfloat16 step at `want`
        diff = np.abs(got - want)
        one_sided_zero = (got == 0) != (want == 0)
        same = diff == 0
        print(name, "identical", same.mean(), "one-sided zeros", int(one_sided_zero.sum()), "of", want.size,
              "largest difference / largest value", diff.max() / np.abs(want).max())
        assert same.mean() > exact_share, name
        assert (want != 0).mean() > 0.05, name            # (not an empty comparison)
        ok = ~one_sided_zero
        if first_layer:     # identical inputs on both sides: never more than the one step
            assert np.all(diff[ok] <= 1.0001 * ulp[ok]), name
        else:               # inputs that differ by a step here and there move small results by more than their own step
            assert np.all(diff[ok] <= 1.0001 * ulp[ok] + 2e-3 * np.abs(want).max()), name
        return one_sided_zero

    z1 = compare("a1", grid(lay["a1"], wl.c1), a1, 0.999, first_layer=True)
    assert np.all(np.abs(pre1[z1]) < 1e-4)                 # ... only where the sum itself is next to zero
    z2 = compare("a2", grid(lay["a2"], wl.c2), a2, 0.999)
    assert np.all(np.abs(pre2[z2]) < 1e-2)
    # (d loss / d z itself is never assembled on this path: the classifier's backward kernel forms
    #  it from the loss kernel's per-tile shares and rounds it in registers; da2 is its first image)
    # a gradient element is zero on one side only through such a mask element (or by falling below bfloat16's range)
    zd2 = compare("da2", grid(lay["da2"], wl.c2), da2, 0.99)
    assert zd2.sum() <= z2.sum() + 0.001 * da2.size
    zd1 = compare("da1", grid(lay["da1"], wl.c1), da1, 0.98)
    assert zd1.sum() <= z1.sum() + 0.002 * da1.size


@pytest.mark.parametrize("compute", ["f32", "bf16"])
def test_equal_logits_go_to_the_lowest_class(compute):
    """With a zero classifier every pixel's logits are the biases, exactly: the predicted class
    is the lowest index among the largest biases (ties are decided the same way everywhere)."""
    shape = dict(c_in=64, h=9, w=21, c1=64, c2=64, n_classes=7) if compute == "bf16" else \
        dict(c_in=12, h=9, w=21, c1=16, c2=8, n_classes=7)
    wl = WL.small_variant(WL.WORKLOADS["720p" if compute == "bf16" else "tiny"], **shape)
    f, lab, p = inputs(wl)
    sl = WL.param_slices(wl)
    desc = st.HeadDesc.of(wl)
    pred = torch.empty((wl.n, wl.H, wl.W), dtype=torch.uint8, device="cuda")
    for b3, want in ((np.zeros(7), 0), (np.array([0, 1, 1, 0, 1, 0, 0.5]), 1), (np.array([-1, -1, -2, -1, -3, -1, -1]), 0),
                     (np.array([0, 0, 0, 0, 0, 0, 1e-30]), 6)):
        q = p.copy()
        q[sl["W3"]] = 0.0
        q[sl["b3"]] = b3.astype(np.float32)
        st.st_head_forward(desc, to_dev_features(wl, f), torch.from_numpy(q).cuda(), None, pred)
        torch.cuda.synchronize()
        got = pred.cpu().numpy()
        assert (got == want).all(), (b3, np.unique(got))
        # and the oracle takes the same decision from the same logits
        z = np.broadcast_to(b3.astype(np.float32)[None, :, None, None], (wl.n, 7, wl.h, wl.w)).copy()
        assert (O.predict_from_logits(z) == want).all()


@pytest.mark.parametrize("case", ["f32", "mfma", "mfma_grouped"])
def test_channels_last_features_give_the_same_call(case):
    """feat_layout = ST_NHWC: the same features handed over as [n, h, w, c_in] must give, bit for
    bit, what the [n, c_in, h, w] call gives (only the packing role differs)."""
    if case == "f32":
        wl = WL.small_variant(WL.WORKLOADS["tiny"], n=2, c_in=20, h=9, w=37, c1=24, c2=16, n_classes=5, steps=2)
    else:
        wl = WL.small_variant(WL.WORKLOADS["720p"], n=2, c_in=64, h=11, w=40, c1=64, c2=64, n_classes=7, steps=2,
                              n_sites=9)
    grouped = 1 if case == "mfma_grouped" else 0
    heads = wl.n if grouped else 1
    f, lab, _ = inputs(wl)
    p = np.stack([WL.make_head_params(wl, seed=wl.init_seed + 17 * i) for i in range(heads)]).astype(np.float32)
    fd = to_dev_features(wl, f)
    results = []
    for layout in (st.ST_NCHW, st.ST_NHWC):
        desc = st.HeadDesc.of(wl)
        desc.grouped, desc.feat_layout = grouped, layout
        feats = fd if layout == st.ST_NCHW else fd.permute(0, 2, 3, 1).contiguous()
        pt = torch.from_numpy(p if grouped else p[0]).cuda()
        losses = torch.zeros((wl.steps + 1, heads) if grouped else (wl.steps + 1,), dtype=torch.float32, device="cuda")
        pred = torch.zeros((wl.n, wl.H, wl.W), dtype=torch.uint8, device="cuda")
        dfeat = None if (grouped or case == "f32") else torch.zeros((wl.n, wl.c_in, wl.h, wl.w), dtype=torch.float32,
                                                                    device="cuda")
        st.st_partial_distill(desc, feats, torch.from_numpy(lab).cuda(), pt, wl.steps, wl.lr, losses=losses, pred=pred,
                              feature_grad=dfeat)
        z = torch.empty((wl.n, wl.n_classes, wl.h, wl.w), dtype=torch.float32, device="cuda")
        if not grouped:
            st.st_head_forward(desc, feats, pt, z, None)
        torch.cuda.synchronize()
        results.append([t.cpu().numpy() for t in (pt, losses, pred, z)] + ([dfeat.cpu().numpy()] if dfeat is not None else []))
    for a, b in zip(*results):
        np.testing.assert_array_equal(a, b)
    assert np.abs(results[0][0] - (p if grouped else p[0])).max() > 0


def test_head_forward_matches_oracle():
    wl = WL.small_variant(WL.WORKLOADS["tiny"], c_in=12, h=10, w=33, c1=16, c2=8, n_classes=6)
    f, lab, p = inputs(wl)
    desc = st.HeadDesc.of(wl)
    z = torch.empty((wl.n, wl.n_classes, wl.h, wl.w), dtype=torch.float32, device="cuda")
    pred = torch.empty((wl.n, wl.H, wl.W), dtype=torch.uint8, device="cuda")
    st.st_head_forward(desc, to_dev_features(wl, f), torch.from_numpy(p).cuda(), z, pred)
    torch.cuda.synchronize()
    zo, _ = O.head_forward(O.desc_of(wl), WL.features_as_f64(wl, f), p.astype(np.float64), want_pred=False)
    assert rel_err(z.cpu().numpy(), zo) < 1e-5
    np.testing.assert_array_equal(pred.cpu().numpy(), O.predict_from_logits(z.cpu().numpy()))
    # pred only / logits only
    pred2 = torch.empty_like(pred)
    st.st_head_forward(desc, to_dev_features(wl, f), torch.from_numpy(p).cuda(), None, pred2)
    torch.cuda.synchronize()
    assert torch.equal(pred, pred2)


@pytest.mark.parametrize("P,C,ignore", [(0, 3, -1), (1, 2, -1), (1000, 19, 255), (65537, 21, 255),
                                        (300001, 9, -1), (4097, 200, 7)])
def test_miou_matches_oracle_bit_exact(P, C, ignore):
    rng = np.random.default_rng(P + C)
    pred = rng.integers(0, min(C, 256), size=P).astype(np.uint8)
    lab = rng.integers(0, C, size=P).astype(np.int32)
    # long constant runs, like real label maps
    if P > 100:
        lab[: P // 2] = lab[0]
        pred[: P // 3] = pred[0]
    if ignore >= 0 and P:
        lab[rng.random(P) < 0.07] = ignore
    conf, m = st.st_miou(torch.from_numpy(pred).cuda(), torch.from_numpy(lab).cuda(), C, ignore)
    torch.cuda.synchronize()
    conf_o = O.confusion(pred, lab, C, ignore)
    np.testing.assert_array_equal(conf.cpu().numpy(), conf_o)
    assert m.item() == O.miou(conf_o)[0]


@pytest.mark.parametrize("P,C", [(1920 * 1080, 19), (4 * 720 * 1280, 21), (600001, 200)])
def test_miou_many_blocks_and_reused_result_buffers(P, C):
    """Frame-sized maps (the histogram runs on up to 256 blocks, spread over all XCDs) with calls
    in a row into the same result buffers, on maps that change between the calls: every call
    exact."""
    rng = np.random.default_rng(P % 1000 + C)
    pred = rng.integers(0, min(C, 256), size=P).astype(np.uint8)
    lab = rng.integers(0, C, size=P).astype(np.int32)
    lab[: P // 2] = lab[0]
    pred[: P // 3] = pred[0]
    dp, dl = torch.from_numpy(pred).cuda(), torch.from_numpy(lab).cuda()
    conf = torch.full((C, C), -7, dtype=torch.int64, device="cuda")
    m = torch.full((1,), float("nan"), dtype=torch.float64, device="cuda")
    for rep in range(6):
        if rep:
            lo, hi = rep * (P // 8), rep * (P // 8) + P // 16
            lab[lo:hi] = (rep * 3) % C
            pred[lo + 100:hi + 100] = (rep * 5) % min(C, 256)
            dp.copy_(torch.from_numpy(pred)); dl.copy_(torch.from_numpy(lab))
        st.st_miou(dp, dl, C, -1, confusion=conf, miou=m)
        torch.cuda.synchronize()
        conf_o = O.confusion(pred, lab, C, -1)
        np.testing.assert_array_equal(conf.cpu().numpy(), conf_o)
        assert m.item() == O.miou(conf_o)[0], rep
    # calls queued back to back without a synchronisation in between
    for _ in range(20):
        st.st_miou(dp, dl, C, -1, confusion=conf, miou=m)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(conf.cpu().numpy(), conf_o)
    assert m.item() == O.miou(conf_o)[0]


def test_miou_unaligned_maps_and_out_of_range_entries():
    # maps that start off a 16-byte boundary, labels outside [0, C) and predictions >= C: the
    # vector path must not be taken and such pixels must not be counted
    P, C = 70001, 11
    rng = np.random.default_rng(77)
    pred = rng.integers(0, 14, size=P + 3).astype(np.uint8)
    lab = rng.integers(-2, 13, size=P + 3).astype(np.int32)
    lab[1000:40000] = 4
    pred[500:30000] = 4
    dp, dl = torch.from_numpy(pred).cuda(), torch.from_numpy(lab).cuda()
    for off_p, off_l in ((3, 3), (0, 1), (1, 0)):
        conf, m = st.st_miou(dp[off_p:off_p + P], dl[off_l:off_l + P], C, -1)
        torch.cuda.synchronize()
        conf_o = O.confusion(pred[off_p:off_p + P], lab[off_l:off_l + P], C, -1)
        np.testing.assert_array_equal(conf.cpu().numpy(), conf_o)
        assert m.item() == O.miou(conf_o)[0]


def test_steps_zero_and_determinism():
    wl = WL.small_variant(WL.WORKLOADS["tiny"], c_in=8, h=9, w=35, c1=8, c2=8, n_classes=5, steps=2)
    f, lab, p = inputs(wl)
    g0 = run_gpu(wl, f, lab, p, steps=0)
    np.testing.assert_array_equal(g0["params"], p)
    assert g0["steps_taken"] == 0
    a = run_gpu(wl, f, lab, p)
    b = run_gpu(wl, f, lab, p)
    for k in ("params", "losses", "mious", "conf", "pred"):
        np.testing.assert_array_equal(a[k], b[k])
    assert a["losses"][0] == g0["losses"][0]


def test_training_loop_exits():
    wl = WL.small_variant(WL.WORKLOADS["tiny"], c_in=8, h=6, w=6, c1=8, c2=8, n_classes=3, n_sites=5,
                          label_seed=5, steps=8, lr=0.05)
    lab = WL.make_labels(wl)
    f = WL.make_learnable_features(wl, lab)
    p = WL.make_head_params(wl)
    trace = run_gpu(wl, f, lab, p)
    m = trace["mious"][:, 0]
    assert m.max() > m[0] + 0.05
    # already at THRESHOLD: nothing happens
    r = run_gpu(wl, f, lab, p, threshold=float(m[0]), return_best=True)
    assert r["steps_taken"] == 0 and r["first_metric"] == m[0] and r["best_metric"] == m[0]
    np.testing.assert_array_equal(r["params"], p)
    # unreachable THRESHOLD: every update taken, the first strict maximum returned
    r = run_gpu(wl, f, lab, p, threshold=1.5, return_best=True)
    assert r["steps_taken"] == 8 and r["best_metric"] == m.max() and r["first_metric"] == m[0]
    assert trace["first_metric"] is None          # fixed-step form: no metric is read back
    best_i = int(np.argmax(m))
    ref = run_gpu(wl, f, lab, p, steps=best_i)
    np.testing.assert_array_equal(r["params"], ref["params"])
    # the best parameters into a buffer of their own, the last ones in place
    desc = st.HeadDesc.of(wl)
    pt, bt = torch.from_numpy(p.copy()).cuda(), torch.zeros(p.size, dtype=torch.float32, device="cuda")
    taken, best = st.st_partial_distill(desc, to_dev_features(wl, f), torch.from_numpy(lab).cuda(), pt, 8, wl.lr,
                                        threshold=1.5, return_best=False, best_params=bt)
    torch.cuda.synchronize()
    assert taken == 8 and best == m.max()
    np.testing.assert_array_equal(bt.cpu().numpy(), ref["params"])
    np.testing.assert_array_equal(pt.cpu().numpy(), trace["params"])
    # reachable THRESHOLD: leave at the first metric strictly above it ('>'), or at it ('>=')
    j = next(i for i in range(1, 9) if m[i] > m[0])
    r_ge = run_gpu(wl, f, lab, p, threshold=float(m[j]), strict_break=False)
    assert r_ge["steps_taken"] == j
    r_gt = run_gpu(wl, f, lab, p, threshold=float(m[j]), strict_break=True)
    assert r_gt["steps_taken"] > j or not (m[j + 1:] > m[j]).any()
    # and the whole trace agrees with the oracle's run of Algorithm 1
    ora = O.train(O.desc_of(wl), WL.features_as_f64(wl, f), lab, p.astype(np.float64), 8, wl.lr, 1.5)
    np.testing.assert_allclose(m, ora["metrics"], atol=5e-3)


def test_training_loop_comparisons_on_exact_ties():
    """Algorithm 1's comparisons where the metrics tie exactly.  A step too small to change any
    predicted class leaves every iteration's metric equal while the parameters move: the
    strictly-better rule keeps the initial parameters as best_student (a '>=' would return the
    last ones); a first metric equal to THRESHOLD takes no update; one ulp above it trains."""
    wl = WL.small_variant(WL.WORKLOADS["tiny"], c_in=8, h=6, w=6, c1=8, c2=8, n_classes=3, n_sites=5,
                          label_seed=5, steps=3, lr=1e-5)
    lab = WL.make_labels(wl)
    f = WL.make_learnable_features(wl, lab)
    p = WL.make_head_params(wl)
    trace = run_gpu(wl, f, lab, p)
    m = trace["mious"][:, 0]
    assert (m == m[0]).all() and not np.array_equal(trace["params"], p)
    r = run_gpu(wl, f, lab, p, threshold=1.5, return_best=True)
    assert r["steps_taken"] == 3 and r["best_metric"] == m[0] and r["first_metric"] == m[0]
    np.testing.assert_array_equal(r["params"], p)
    r = run_gpu(wl, f, lab, p, threshold=1.5, return_best=False)
    np.testing.assert_array_equal(r["params"], trace["params"])
    r = run_gpu(wl, f, lab, p, threshold=float(m[0]), return_best=True)
    assert r["steps_taken"] == 0
    np.testing.assert_array_equal(r["params"], p)
    r = run_gpu(wl, f, lab, p, threshold=float(np.nextafter(m[0], 2.0)), return_best=True)
    assert r["steps_taken"] == 3
    # the oracle scores this problem the same
    ora = O.train(O.desc_of(wl), WL.features_as_f64(wl, f), lab, p.astype(np.float64), 3, wl.lr, 1.5)
    assert ora["updates"] == 3 and (ora["metrics"] == ora["metrics"][0]).all()
    np.testing.assert_allclose(m, ora["metrics"], atol=5e-3)


def test_frame_that_needs_no_training_leaves_everything_untouched():
    """Algorithm 1's skip branch (the common case in a video: most frames are not key frames): a
    head that already scores at the threshold takes no update, and the call leaves the caller's
    parameters, velocity and best-parameter buffer's source bit for bit as they were -- on the
    float32 path and on the matrix-core path."""
    for kw in (dict(c_in=8, h=6, w=6, c1=8, c2=8, n_classes=3, compute="f32", feat_dtype="f32"),
               dict(c_in=64, h=6, w=12, c1=64, c2=64, n_classes=3, compute="bf16", feat_dtype="bf16")):
        wl = WL.small_variant(WL.WORKLOADS["tiny"], n_sites=5, label_seed=5, steps=8, lr=0.05, momentum=0.9, **kw)
        lab = WL.make_labels(wl)
        f = WL.make_learnable_features(wl, lab)
        p = WL.make_head_params(wl)
        trained = run_gpu(wl, f, lab, p)                      # eight steps: a head that scores well
        m_end = float(trained["mious"][-1, 0])
        assert m_end > trained["mious"][0, 0] + 0.05
        desc = st.HeadDesc.of(wl)
        pt = torch.from_numpy(trained["params"].copy()).cuda()
        vel = torch.from_numpy(trained["velocity"].copy()).cuda()
        best = torch.full((p.size,), 7.0, dtype=torch.float32, device="cuda")
        r = st.st_partial_distill(desc, to_dev_features(wl, f), torch.from_numpy(lab).cuda(), pt, 8, wl.lr,
                                  momentum=0.9, velocity=vel, threshold=m_end, return_best=True, best_params=best)
        torch.cuda.synchronize()
        assert r[0] == 0 and r[1] == m_end and r.first_metric == m_end
        np.testing.assert_array_equal(pt.cpu().numpy(), trained["params"])
        np.testing.assert_array_equal(vel.cpu().numpy(), trained["velocity"])
        np.testing.assert_array_equal(best.cpu().numpy(), trained["params"])     # best_student = the head as given


def test_best_is_not_last_with_momentum():
    """A run whose metric rises and falls again (large step, momentum 0.9).  head_params receives
    the best iteration's parameters; the velocity, the class map, the confusion counts and the
    last losses / mious entries are those of the last pass (the header says so)."""
    wl = WL.small_variant(WL.WORKLOADS["tiny"], c_in=8, h=6, w=6, c1=8, c2=8, n_classes=3, n_sites=5,
                          label_seed=5, steps=8, lr=0.2, momentum=0.9)
    lab = WL.make_labels(wl)
    f = WL.make_learnable_features(wl, lab)
    p = WL.make_head_params(wl)
    ora = O.train(O.desc_of(wl), WL.features_as_f64(wl, f), lab, p.astype(np.float64), 8, wl.lr, 1.5, momentum=0.9)
    mo = ora["metrics"]
    best_i = int(np.argmax(mo))
    assert 0 < best_i < 8 and mo[8] < mo[best_i] - 0.1
    r = run_gpu(wl, f, lab, p, threshold=1.5, return_best=True)
    m = r["mious"][:, 0]
    np.testing.assert_allclose(m, mo, atol=2e-2)
    assert r["steps_taken"] == 8 and int(np.argmax(m)) == best_i and r["best_metric"] == m[best_i]
    assert rel_err(r["params"], ora["params"]) < 1e-3
    fixed_best = run_gpu(wl, f, lab, p, steps=best_i)
    fixed_last = run_gpu(wl, f, lab, p, steps=8)
    np.testing.assert_array_equal(r["params"], fixed_best["params"])
    np.testing.assert_array_equal(r["velocity"], fixed_last["velocity"])
    np.testing.assert_array_equal(r["pred"], fixed_last["pred"])
    np.testing.assert_array_equal(r["conf"], fixed_last["conf"])
    assert rel_err(r["velocity"], ora["velocity"]) < 2e-2


def test_early_exit_polling_and_event_wait_agree():
    """The early-exit loop reads each iteration's metric either by polling the host buffer the
    bookkeeping kernel writes or by waiting on an event behind it (the fallback of a platform
    whose host memory is not coherent while a kernel runs): both give the same run, bit for bit
    -- steps taken, metrics, best parameters, last parameters, velocity."""
    wl = WL.small_variant(WL.WORKLOADS["tiny"], c_in=8, h=6, w=6, c1=8, c2=8, n_classes=3, n_sites=5,
                          label_seed=5, steps=8, lr=0.2, momentum=0.9)
    lab = WL.make_labels(wl)
    f = WL.make_learnable_features(wl, lab)
    p = WL.make_head_params(wl)
    wm = WL.small_variant(WL.WORKLOADS["720p"], h=20, w=28, c_in=64, c1=64, c2=64, n_classes=7, steps=4, lr=0.05)
    fm, labm, pm = inputs(wm)
    runs = []
    try:
        for polling in (True, False, True):
            st.st_metric_polling(polling)
            a = run_gpu(wl, f, lab, p, threshold=1.5, return_best=True)
            b = run_gpu(wl, f, lab, p, threshold=float(a["mious"][2, 0]), strict_break=False)
            c = run_gpu(wm, fm, labm, pm, threshold=1.5, return_best=False)
            runs.append((a, b, c))
    finally:
        st.st_metric_polling(True)
    for other in runs[1:]:
        for x, y in zip(runs[0], other):
            assert x["steps_taken"] == y["steps_taken"] and x["best_metric"] == y["best_metric"]
            assert x["first_metric"] == y["first_metric"]
            for k in ("params", "mious", "losses", "pred", "conf"):
                np.testing.assert_array_equal(x[k], y[k], err_msg=k)
    np.testing.assert_array_equal(runs[0][0]["velocity"], runs[1][0]["velocity"])
    assert 0 < runs[0][1]["steps_taken"] < 8


def test_key_frame_hint_changes_the_order_of_work_not_the_result():
    """expect_key_frame makes the first pass compute its gradients and queue the backward pass
    before the host has seen the metric.  Every outcome of Algorithm 1 -- no update at all, an
    exit on the way, all updates, best parameters that are not the last -- is the same with and
    without it, bit for bit; a frame that needs no training leaves the caller's vectors alone."""
    wl = WL.small_variant(WL.WORKLOADS["tiny"], c_in=8, h=6, w=6, c1=8, c2=8, n_classes=3, n_sites=5,
                          label_seed=5, steps=8, lr=0.2, momentum=0.9)
    lab = WL.make_labels(wl)
    f = WL.make_learnable_features(wl, lab)
    p = WL.make_head_params(wl)
    wm = WL.small_variant(WL.WORKLOADS["720p"], h=20, w=28, c_in=64, c1=64, c2=64, n_classes=7, steps=4, lr=0.05)
    fm, labm, pm = inputs(wm)

    def call(w, feats, labels, params, threshold, hint, **kw):
        desc = st.HeadDesc.of(w)
        pt = torch.from_numpy(params.copy()).cuda()
        vel = torch.zeros_like(pt) if w.momentum else None
        bt = torch.full_like(pt, 7.0)
        mious = torch.full((w.steps + 1, w.n), float("nan"), dtype=torch.float64, device="cuda")
        losses = torch.full((w.steps + 1,), float("nan"), dtype=torch.float32, device="cuda")
        r = st.st_partial_distill(desc, to_dev_features(w, feats), torch.from_numpy(labels).cuda(), pt, w.steps, w.lr,
                                  momentum=w.momentum, velocity=vel, threshold=threshold, mious=mious, losses=losses,
                                  best_params=bt, expect_key_frame=hint, **kw)
        torch.cuda.synchronize()
        return dict(ret=tuple(r), first=r.first_metric, params=pt.cpu().numpy(), best=bt.cpu().numpy(),
                    vel=None if vel is None else vel.cpu().numpy(), mious=mious.cpu().numpy(), losses=losses.cpu().numpy())

    trace = call(wl, f, lab, p, 1.5, False)
    m = trace["mious"][:, 0]
    cases = [(wl, f, lab, p, 1.5, dict(return_best=True)), (wl, f, lab, p, 1.5, dict(return_best=False)),
             (wl, f, lab, p, float(m[0]), dict(return_best=True)),                        # no key frame
             (wl, f, lab, p, float(m[2]), dict(strict_break=False)),                      # leaves on the way
             (wm, fm, labm, pm, 1.5, dict(return_best=True))]                              # matrix-core path
    for w, feats, labels, params, thr, kw in cases:
        a, b = call(w, feats, labels, params, thr, False, **kw), call(w, feats, labels, params, thr, True, **kw)
        assert a["ret"] == b["ret"] and a["first"] == b["first"], (thr, kw)
        taken = a["ret"][0]
        for k in ("params", "best", "vel"):
            if a[k] is not None:
                np.testing.assert_array_equal(a[k], b[k], err_msg=k)
        np.testing.assert_array_equal(a["mious"][:taken + 1], b["mious"][:taken + 1])
        np.testing.assert_array_equal(a["losses"][:taken + 1], b["losses"][:taken + 1])
    nokey = call(wl, f, lab, p, float(m[0]), True, return_best=True)
    assert nokey["ret"][0] == 0
    np.testing.assert_array_equal(nokey["params"], p)
    assert (nokey["vel"] == 0).all()


def test_non_finite_parameters_stay_in_range():
    """A diverged head (every parameter NaN): the class map stays inside [0, C) -- class 0, the
    oracle's answer as well -- the confusion counts still hold every valid pixel exactly once,
    and the loss reports the condition by being non-finite.  Both the float32 and the
    matrix-core path, with a class count that needs padding."""
    for kw in (dict(c_in=8, h=6, w=9, c1=8, c2=8, n_classes=5, compute="f32", feat_dtype="f32"),
               dict(c_in=64, h=6, w=9, c1=64, c2=64, n_classes=19, compute="bf16", feat_dtype="bf16")):
        wl = WL.small_variant(WL.WORKLOADS["tiny"], n_sites=7, steps=0, **kw)
        f, lab, p = inputs(wl)
        g = run_gpu(wl, f, lab, np.full_like(p, np.nan), steps=0)
        assert not np.isfinite(g["losses"][0])
        assert (g["pred"] == 0).all()
        assert g["conf"].sum() == lab.size and (g["conf"][0][:, 1:] == 0).all()
        np.testing.assert_array_equal(g["pred"], O.predict_from_logits(g["z"]))


MFMA_CASES = [
    dict(n=1, c_in=64, h=12, w=40, c1=64, c2=64, n_classes=19),
    dict(n=2, c_in=128, h=9, w=21, c1=64, c2=128, n_classes=21, ignore_index=255, ignore_fraction=0.05,
         momentum=0.9),
    dict(n=1, c_in=64, h=3, w=5, c1=96, c2=256, n_classes=5),
    dict(n=3, c_in=64, h=17, w=9, c1=32, c2=64, n_classes=32),
]


@pytest.mark.parametrize("case", range(len(MFMA_CASES)))
def test_matrix_core_path_small_shapes(case):
    """Shapes that take the MFMA kernels (channels in multiples of 64 / 32) with ragged grids:
    several position tiles, a ragged last tile, more than one frame."""
    wl = WL.small_variant(WL.WORKLOADS["720p"], steps=3, lr=0.02, n_sites=9, **MFMA_CASES[case])
    f, lab, p = inputs(wl)
    gpu = run_gpu(wl, f, lab, p)
    check_staged_bit_exact(wl, gpu, lab)
    ora = run_oracle(wl, f, lab, p, bf16_operands=False)
    orq = run_oracle(wl, f, lab, p, bf16_operands=True)
    assert rel_err(gpu["losses"], ora["losses"]) < 2e-2
    assert rel_err(gpu["params"], ora["params"]) < 2e-2
    assert rel_err(gpu["losses"], orq["losses"]) < 5e-4
    assert rel_err(gpu["params"], orq["params"]) < 5e-4
    assert update_err(f"mfma case {case}", gpu["params"] - p, orq["params"] - p) < 3e-2
    if wl.momentum:
        assert rel_err(gpu["velocity"], orq["velocity"]) < 3e-2
    # run twice: bit-identical (fixed-order reductions, no floating-point atomics)
    again = run_gpu(wl, f, lab, p)
    for k in ("params", "losses", "mious", "conf", "pred"):
        np.testing.assert_array_equal(gpu[k], again[k])


@pytest.mark.parametrize("path", ["f32", "mfma"])
def test_every_class_count(path):
    """2 .. 32 classes, each on both paths: the fused loss kernel is compiled once per class count
    (its arithmetic runs over exactly the classes that exist, its buffers over the count rounded
    up to a multiple of four), so every count is a kernel of its own.  Small grids with a ragged
    tile edge, ignored pixels, two steps: losses and parameters against the oracle; predictions,
    confusion counts and mean IoU bit for bit from the call's own final logits."""
    for C in range(2, 33):
        if path == "f32":
            wl = WL.small_variant(WL.WORKLOADS["tiny"], steps=2, lr=0.05, n_sites=11, n=1, c_in=6, h=4, w=35, c1=8,
                                  c2=8, n_classes=C, ignore_index=255, ignore_fraction=0.05)
        else:
            wl = WL.small_variant(WL.WORKLOADS["720p"], steps=2, lr=0.02, n_sites=11, n=1, c_in=64, h=4, w=35, c1=32,
                                  c2=64, n_classes=C, ignore_index=255, ignore_fraction=0.05)
        f, lab, p = inputs(wl)
        gpu = run_gpu(wl, f, lab, p)
        check_staged_bit_exact(wl, gpu, lab)
        ora = run_oracle(wl, f, lab, p, bf16_operands=(path == "mfma"))
        tol = 1e-4 if path == "f32" else 5e-4
        assert rel_err(gpu["losses"], ora["losses"]) < tol, C
        assert rel_err(gpu["params"], ora["params"]) < tol, C
        assert update_err(f"{C} classes {path}", gpu["params"] - p, ora["params"] - p) < (2e-3 if path == "f32" else 3e-2), C
        progress(f"every class count: {path} C={C} ok")


# ------------------------------------------------------------------ Adam (the paper's optimiser, Section 5.2)
def run_gpu_adam(wl, feats, labels, params, steps, t0=0, m=None, v=None, object_radius=None):
    import torch
    import paper_2003_10735_amd as st
    from gpu_util import to_dev_features
    desc = st.HeadDesc.of(wl)
    p = torch.from_numpy(params.astype(np.float32)).cuda()
    mt = torch.from_numpy((m if m is not None else np.zeros_like(params)).astype(np.float32)).cuda()
    vt = torch.from_numpy((v if v is not None else np.zeros_like(params)).astype(np.float32)).cuda()
    losses = torch.full((steps + 1,), float("nan"), dtype=torch.float32, device="cuda")
    lab = torch.from_numpy(labels).cuda()
    # the loss weights of Section 5.2, made by the library from the labels
    wts = None if object_radius is None else st.st_object_weights(lab, wl.n_classes, object_radius, factor=5,
                                                                 ignore_index=wl.ignore_index)
    taken, _ = st.st_partial_distill(desc, to_dev_features(wl, feats), lab, p, steps,
                                     wl.lr, losses=losses, adam=dict(m=mt, v=vt, t0=t0), pixel_weights=wts)
    torch.cuda.synchronize()
    assert taken == steps
    return dict(params=p.cpu().numpy(), m=mt.cpu().numpy(), v=vt.cpu().numpy(), losses=losses.cpu().numpy())


def check_adam(wl, feats, labels, params, steps, bf16_operands, loss_tol, tol, object_radius=None):
    """Adam's update m / (sqrt(v) + eps) is (nearly) the sign of the gradient where the
    gradient is tiny, so two correct implementations whose gradients differ in the last bits
    may move such a parameter in opposite directions.  Elementwise parity of the weights is
    therefore required only where the oracle's own first gradient is not tiny; the losses, the
    second moments (continuous in g) and the share of excused elements are checked as well."""
    d = O.desc_of(wl, bf16_operands)
    if object_radius is not None:       # with the x5 weighting near objects: the oracle's own map
        from oracle import object_weights as OW
        d = O.with_pixel_weights(d, OW.object_weights(labels, wl.n_classes, object_radius, factor=5,
                                                      ignore_index=wl.ignore_index))
    f64 = WL.features_as_f64(wl, feats)
    o = O.partial_distill_opt(d, f64, labels, params.astype(np.float64), steps, O.adam_optim(wl.lr))
    g = run_gpu_adam(wl, feats, labels, params, steps, object_radius=object_radius)
    np.testing.assert_allclose(g["losses"], o["losses"], rtol=loss_tol, atol=loss_tol)
    _, g0, _, _, _ = O.loss_and_grad(d, f64, labels, params.astype(np.float64))
    solid = np.abs(g0) > 1e-3 * np.abs(g0).max()
    assert solid.mean() > 0.5
    scale = np.abs(o["params"]).max()
    assert np.max(np.abs(g["params"] - o["params"])[solid]) <= tol * scale
    # everywhere: never further apart than the walk of `steps` full-size steps in opposite directions
    assert np.max(np.abs(g["params"] - o["params"])) <= 2.0 * steps * wl.lr * 1.01
    assert rel_err(g["v"], o["s2"]) <= max(tol, 1e-3)
    return g, o


def test_adam_tiny_f32():
    wl = WL.WORKLOADS["tiny"]
    f, lab, p = WL.make_features(wl), WL.make_labels(wl), WL.make_head_params(wl)
    g, o = check_adam(wl, f, lab, p, 4, None, 1e-4, 1e-3)
    # the step counter continues: two calls of two steps equal one call of four
    a = run_gpu_adam(wl, f, lab, p, 2)
    b = run_gpu_adam(wl, f, lab, a["params"], 2, t0=2, m=a["m"], v=a["v"])
    np.testing.assert_array_equal(b["params"], g["params"])
    np.testing.assert_array_equal(b["v"], g["v"])


def test_adam_matrix_core_path():
    wl = WL.small_variant(WL.WORKLOADS["720p"], h=20, w=28, c_in=64, c1=64, c2=64, n_classes=7, steps=3, lr=0.01)
    f, lab, p = WL.make_features(wl), WL.make_labels(wl), WL.make_head_params(wl)
    check_adam(wl, f, lab, p, 3, True, 2e-3, 2e-2)


def test_adam_with_object_weights_matrix_core_path():
    """The training recipe of the paper's experiments (Section 5.2): Adam at learning rate 0.01
    on the cross-entropy weighted x5 near and within objects."""
    wl = WL.small_variant(WL.WORKLOADS["720p"], h=20, w=28, c_in=64, c1=64, c2=64, n_classes=7, steps=3, lr=0.01)
    f, lab, p = WL.make_features(wl), WL.make_labels(wl), WL.make_head_params(wl)
    g, _ = check_adam(wl, f, lab, p, 3, True, 2e-3, 2e-2, object_radius=3)
    plain = run_gpu_adam(wl, f, lab, p, 3)
    assert abs(g["losses"][0] - plain["losses"][0]) > 1e-3        # the weights do change the loss


# ------------------------------------------------------------------ weighted cross-entropy (Section 5.2)
def run_gpu_weighted(wl, feats, labels, params, wts, steps):
    import torch
    import paper_2003_10735_amd as st
    from gpu_util import to_dev_features
    desc = st.HeadDesc.of(wl)
    p = torch.from_numpy(params.astype(np.float32)).cuda()
    losses = torch.full((steps + 1,), float("nan"), dtype=torch.float32, device="cuda")
    mious = torch.full((steps + 1, wl.n), float("nan"), dtype=torch.float64, device="cuda")
    st.st_partial_distill(desc, to_dev_features(wl, feats), torch.from_numpy(labels).cuda(), p, steps, wl.lr,
                          losses=losses, mious=mious, pixel_weights=torch.from_numpy(wts).cuda())
    torch.cuda.synchronize()
    return dict(params=p.cpu().numpy(), losses=losses.cpu().numpy(), mious=mious.cpu().numpy())


def check_weighted(wl, steps, bf16_operands, tol):
    f, lab, p = WL.make_features(wl), WL.make_labels(wl), WL.make_head_params(wl)
    wts = WL.object_weight_map(lab, radius=4)
    assert (wts == 5).any() and (wts == 1).any()
    d = O.with_pixel_weights(O.desc_of(wl, bf16_operands), wts)
    o = O.partial_distill_opt(d, WL.features_as_f64(wl, f), lab, p.astype(np.float64), steps,
                              O.Optim(0, wl.lr, 0.0, 0, 0, 0, 0))
    g = run_gpu_weighted(wl, f, lab, p, wts, steps)
    plain = run_gpu(wl, f, lab, p, steps=steps)
    assert abs(g["losses"][0] - plain["losses"][0]) > 1e-3        # the weights do change the loss
    assert rel_err(g["losses"], o["losses"]) < tol
    assert rel_err(g["params"], o["params"]) < tol
    assert rel_err(g["params"] - p, o["params"] - p) < max(30 * tol, 1e-3)
    np.testing.assert_allclose(g["mious"], o["mious"], atol=5e-3)


def test_weighted_loss_tiny_f32():
    # class 0 plays the background
    check_weighted(WL.small_variant(WL.WORKLOADS["tiny"], n_sites=6), 4, None, 1e-4)


def test_weighted_loss_ragged_with_ignore_f32():
    wl = WL.small_variant(WL.WORKLOADS["tiny"], c_in=8, h=7, w=37, c1=8, c2=8, n_classes=5, n_sites=9,
                          ignore_index=255, ignore_fraction=0.1, steps=2)
    check_weighted(wl, 2, None, 1e-4)


def test_weighted_loss_matrix_core_path():
    wl = WL.small_variant(WL.WORKLOADS["720p"], h=20, w=28, c_in=64, c1=64, c2=64, n_classes=7, steps=3)
    check_weighted(wl, 3, True, 5e-4)


# ------------------------------------------------------------------ degenerate inputs
@pytest.mark.parametrize("mfma", [False, True])
def test_all_labels_ignored(mfma):
    """No valid pixel: loss 0, gradient 0 (the parameters do not move), mean IoU 0, empty counts."""
    if mfma:
        wl = WL.small_variant(WL.WORKLOADS["720p"], h=9, w=20, c_in=64, c1=32, c2=64, n_classes=6, steps=2,
                              ignore_index=255)
    else:
        wl = WL.small_variant(WL.WORKLOADS["tiny"], c_in=8, h=5, w=7, c1=8, c2=8, n_classes=3, steps=2,
                              ignore_index=255)
    f, _, p = inputs(wl)
    lab = np.full((wl.n, wl.H, wl.W), 255, dtype=np.int32)
    g = run_gpu(wl, f, lab, p)
    assert np.all(g["losses"] == 0.0) and np.all(g["mious"] == 0.0) and not g["conf"].any()
    np.testing.assert_array_equal(g["params"], p.astype(np.float32))
    o = run_oracle(wl, f, lab, p)
    assert np.all(o["losses"] == 0.0)
    np.testing.assert_array_equal(o["params"], p.astype(np.float64))
    check_staged_bit_exact(wl, g, lab)


def test_single_class_labels_and_maximum_class_count():
    """Every pixel of one class (one row of the confusion matrix, mean IoU over one class), with
    the largest class count the library takes (32)."""
    wl = WL.small_variant(WL.WORKLOADS["tiny"], c_in=8, h=6, w=9, c1=8, c2=16, n_classes=32, steps=2, lr=0.05)
    f, _, p = inputs(wl)
    lab = np.full((wl.n, wl.H, wl.W), 31, dtype=np.int32)
    g = run_gpu(wl, f, lab, p)
    o = run_oracle(wl, f, lab, p)
    check_staged_bit_exact(wl, g, lab)
    assert g["conf"][0, :31].sum() == 0 and g["conf"][0, 31].sum() == wl.H * wl.W
    assert rel_err(g["losses"], o["losses"]) < 1e-4
    assert rel_err(g["params"], o["params"]) < 1e-4
    np.testing.assert_allclose(g["mious"], o["mious"], atol=2e-3)
    assert g["losses"][-1] < g["losses"][0]       # a constant target is learnt quickly


def test_workspace_reuse_across_calls_leaves_no_trace():
    """A workspace that served another call (other data, other optimiser state) gives the same
    result bit for bit as a fresh one: everything a call relies on is re-established by the call."""
    import torch
    import paper_2003_10735_amd as st
    wl = WL.small_variant(WL.WORKLOADS["720p"], h=12, w=25, c_in=64, c1=64, c2=64, n_classes=5, steps=2)
    f, lab, p = inputs(wl)
    ws = st.new_workspace(st.HeadDesc.of(wl))
    ws.fill_(0xFF)                                  # NaN patterns everywhere
    a = run_gpu(wl, f, lab, p, workspace=ws)
    f2, lab2 = WL.make_features(wl, seed=77), WL.make_labels(wl, frame_shift=13)
    run_gpu(wl, f2, lab2, p, workspace=ws)          # dirty it with another problem
    b = run_gpu(wl, f, lab, p, workspace=ws)
    fresh = run_gpu(wl, f, lab, p)
    for k in ("params", "losses", "mious", "conf", "pred"):
        np.testing.assert_array_equal(a[k], fresh[k])
        np.testing.assert_array_equal(b[k], fresh[k])
    assert np.all(np.isfinite(a["losses"]))


# ------------------------------------------------------------------ full backward pass (feature gradient)
def run_gpu_feature_grad(wl, feats, labels, params, steps):
    import torch
    import paper_2003_10735_amd as st
    from gpu_util import to_dev_features
    desc = st.HeadDesc.of(wl)
    p = torch.from_numpy(params.astype(np.float32)).cuda()
    df = torch.full((wl.n, wl.c_in, wl.h, wl.w), float("nan"), dtype=torch.float32, device="cuda")
    st.st_partial_distill(desc, to_dev_features(wl, feats), torch.from_numpy(labels).cuda(), p, steps, wl.lr,
                          feature_grad=df)
    torch.cuda.synchronize()
    return p.cpu().numpy(), df.cpu().numpy()


def check_feature_grad(wl, bf16_operands, tol):
    """One step: the feature gradient belongs to the initial parameters, and asking for it must
    not change the step itself.  On the bfloat16 path the tolerance against the oracle with the
    same rounding points is wider than for the weights: the operands da2 and da1 are themselves
    rounded sums, the two sides add in different orders, so a few operand elements round the other
    way (2^-8 relative each), and an element of d features sums only 9 * c1 products -- it does
    not average such flips over all positions the way a weight gradient does."""
    f, lab, p = inputs(wl)
    params, df = run_gpu_feature_grad(wl, f, lab, p, 1)
    plain = run_gpu(wl, f, lab, p, steps=1)
    np.testing.assert_array_equal(params, plain["params"])
    d = O.desc_of(wl, bf16_operands)
    _, _, df_o = O.feature_grad(d, WL.features_as_f64(wl, f), lab, p.astype(np.float64))
    assert np.all(np.isfinite(df))
    assert rel_err(df, df_o) < tol, rel_err(df, df_o)
    if bf16_operands:
        # Against the oracle that rounds nothing only a loose bound holds, by the nature of the
        # bfloat16 semantics and not of the implementation: where an activation is within rounding
        # noise of zero its ReLU mask differs between the two, which switches whole elements of
        # da2 / da1 on or off (the oracle's own two modes differ by 10 % in the maximum norm here,
        # while the weight gradients, sums over all positions, agree to 1-2 %).
        _, _, df_p = O.feature_grad(O.desc_of(wl, False), WL.features_as_f64(wl, f), lab, p.astype(np.float64))
        assert rel_err(df, df_p) < 0.3, rel_err(df, df_p)
        assert np.median(np.abs(df - df_p)) < 1e-2 * np.abs(df_p).max()


def test_feature_grad_tiny_f32():
    check_feature_grad(WL.WORKLOADS["tiny"], None, 1e-4)


def test_feature_grad_ragged_generic_bf16():
    wl = WL.small_variant(WL.WORKLOADS["tiny"], n=2, c_in=20, h=9, w=37, c1=24, c2=16, n_classes=5, compute="bf16",
                          feat_dtype="bf16", steps=1)
    check_feature_grad(wl, True, 5e-3)


def test_feature_grad_matrix_core_path():
    wl = WL.small_variant(WL.WORKLOADS["720p"], n=2, h=20, w=28, c_in=128, c1=64, c2=64, n_classes=7, steps=1)
    check_feature_grad(wl, True, 5e-3)

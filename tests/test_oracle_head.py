"""Pins of the oracle's composed path: head forward, loss, hand-derived backward, the k-step
loop and the training loop's exits.  Independent checks: CPU PyTorch float64 autograd, central
finite differences, closed forms, and the loop's own definition replayed from its trace."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle as O
import workloads as WL

torch.set_num_threads(4)
RNG = np.random.default_rng(777)


def T(a):
    return torch.from_numpy(np.ascontiguousarray(a))


def tiny(n=1, c_in=3, h=4, w=5, c1=4, c2=4, C=3, ignore=-1, bf16=False):
    return O.desc(n, c_in, h, w, c1, c2, C, ignore, bf16)


def split(d, p):
    o = 0
    out = []
    for shape in [(d.c1, d.c_in, 3, 3), (d.c1,), (d.c2, d.c1, 3, 3), (d.c2,),
                  (d.n_classes, d.c2, 1, 1), (d.n_classes,)]:
        sz = int(np.prod(shape))
        out.append(p[o:o + sz].reshape(shape))
        o += sz
    assert o == (p.numel() if hasattr(p, "numel") else p.size)
    return out


def torch_loss(d, f, lab, p):
    W1, b1, W2, b2, W3, b3 = split(d, p)
    a1 = F.relu(F.conv2d(f, W1, b1, padding=1))
    a2 = F.relu(F.conv2d(a1, W2, b2, padding=1))
    z = F.conv2d(a2, W3, b3)
    Z = F.interpolate(z, scale_factor=8, mode="bilinear", align_corners=False)
    ign = d.ignore_index if d.ignore_index >= 0 else -100
    return F.cross_entropy(Z, lab.long(), ignore_index=ign), z, Z


def random_problem(d, seed=0, ignore_frac=0.0):
    rng = np.random.default_rng(seed)
    f = rng.standard_normal((d.n, d.c_in, d.h, d.w))
    p = 0.5 * rng.standard_normal(O.num_params(d))
    lab = rng.integers(0, d.n_classes, size=(d.n, 8 * d.h, 8 * d.w)).astype(np.int32)
    if ignore_frac:
        lab[rng.random(lab.shape) < ignore_frac] = d.ignore_index
    return f, lab, p


def test_num_params_formula():
    d = tiny()
    assert O.num_params(d) == 4 * 3 * 9 + 4 + 4 * 4 * 9 + 4 + 3 * 4 + 3
    wl = WL.WORKLOADS["720p"]
    assert O.num_params(O.desc_of(wl)) == 445075 == wl.n_params
    assert WL.WORKLOADS["tiny"].n_params == 74441
    assert WL.WORKLOADS["batch4"].n_params == 1333013


@pytest.mark.parametrize("n,ignore", [(1, -1), (2, 255)])
def test_loss_and_grad_match_library_autograd(n, ignore):
    d = tiny(n=n, ignore=ignore)
    f, lab, p = random_problem(d, seed=n, ignore_frac=0.1 if ignore >= 0 else 0.0)
    pt = T(p).requires_grad_()
    ft = T(f).requires_grad_()
    loss_t, z_t, Z_t = torch_loss(d, ft, T(lab), pt)
    loss_t.backward()
    loss, grad, pred, conf, mi = O.loss_and_grad(d, f, lab, p)
    assert abs(loss - loss_t.item()) < 1e-12
    np.testing.assert_allclose(grad, pt.grad.numpy(), rtol=1e-9, atol=1e-13)
    z, pred2 = O.head_forward(d, f, p)
    np.testing.assert_allclose(z, z_t.detach().numpy(), rtol=1e-12, atol=1e-13)
    np.testing.assert_array_equal(pred, pred2)
    # prediction = argmax of the up-sampled logits (float32 decision; the float64 library
    # result may differ only where the top two are closer than float32 resolves)
    ref_pred = Z_t.detach().argmax(dim=1).numpy()
    top2 = np.sort(Z_t.detach().numpy(), axis=1)[:, -2:]
    margin = top2[:, 1] - top2[:, 0]
    bad = pred != ref_pred
    assert bad.mean() < 1e-3 and np.all(margin[bad] < 1e-5)
    # metric consistency
    for i in range(n):
        np.testing.assert_array_equal(conf[i], O.confusion(pred[i], lab[i], d.n_classes, ignore))
        assert mi[i] == O.miou(conf[i])[0]


def test_gradient_by_central_finite_differences():
    d = tiny()
    f, lab, p = random_problem(d, seed=5)
    _, grad, *_ = O.loss_and_grad(d, f, lab, p)
    # skip parameters whose perturbation could cross a ReLU kink: probe a1/a2 pre-activations
    eps = 1e-6
    idx = np.random.default_rng(1).choice(p.size, size=60, replace=False)
    checked = 0
    for i in idx:
        pp, pm = p.copy(), p.copy()
        pp[i] += eps
        pm[i] -= eps
        lp = O.loss_and_grad(d, f, lab, pp, want_grad=False, want_metric=False)[0]
        lm = O.loss_and_grad(d, f, lab, pm, want_grad=False, want_metric=False)[0]
        fd = (lp - lm) / (2 * eps)
        # second difference tells whether a kink was crossed
        l0 = O.loss_and_grad(d, f, lab, p, want_grad=False, want_metric=False)[0]
        if abs(lp - 2 * l0 + lm) > 1e-9:
            continue
        assert abs(fd - grad[i]) < 1e-6 * max(1.0, abs(grad[i])) + 2e-9, (i, fd, grad[i])
        checked += 1
    assert checked >= 40


def test_last_bias_gradient_sums_to_zero_and_zero_last_layer_gives_log_C():
    d = tiny(c_in=5, C=4)
    f, lab, p = random_problem(d, seed=9)
    _, grad, *_ = O.loss_and_grad(d, f, lab, p)
    assert abs(grad[-d.n_classes:].sum()) < 1e-14
    p0 = p.copy()
    p0[-(d.n_classes * d.c2 + d.n_classes):] = 0.0
    loss, *_ = O.loss_and_grad(d, f, lab, p0)
    assert abs(loss - np.log(d.n_classes)) < 1e-12


def test_k_steps_match_library_loop_sgd_and_momentum():
    for mu in (0.0, 0.9):
        d = tiny(n=2, ignore=255)
        f, lab, p = random_problem(d, seed=11, ignore_frac=0.05)
        res = O.partial_distill(d, f, lab, p, steps=5, lr=0.05, momentum=mu)
        pt = T(p.copy()).requires_grad_()
        opt = torch.optim.SGD([pt], lr=0.05, momentum=mu)
        losses = []
        for it in range(6):
            opt.zero_grad()
            loss_t, _, _ = torch_loss(d, T(f), T(lab), pt)
            losses.append(loss_t.item())
            if it == 5:
                break
            loss_t.backward()
            opt.step()
        np.testing.assert_allclose(res["losses"], losses, rtol=1e-10)
        np.testing.assert_allclose(res["params"], pt.detach().numpy(), rtol=1e-9, atol=1e-12)
        # entry i of the traces describes the parameters before update i+1
        l0, _, _, conf0, mi0 = O.loss_and_grad(d, f, lab, p, want_grad=False)
        assert res["losses"][0] == l0 and np.array_equal(res["mious"][0], mi0)
        lk, _, predk, confk, mik = O.loss_and_grad(d, f, lab, res["params"], want_grad=False)
        assert res["losses"][-1] == lk
        np.testing.assert_array_equal(res["conf"], confk)
        np.testing.assert_array_equal(res["pred"], predk)
        np.testing.assert_array_equal(res["mious"][-1], mik)


@pytest.mark.parametrize("mu", [0.0, 0.9])
def test_stepwise_loop_is_the_c_loop(mu):
    """The step-by-step front-end (used where a long run has to report progress) gives bit for bit
    what the C loop gives."""
    d = tiny()
    f, lab, p = random_problem(d, seed=21)
    a = O.partial_distill(d, f, lab, p, steps=3, lr=0.1, momentum=mu)
    seen = []
    b = O.partial_distill_stepwise(d, f, lab, p, steps=3, lr=0.1, momentum=mu, on_step=lambda it, loss: seen.append(it))
    assert seen == [0, 1, 2, 3]
    for k in ("params", "velocity", "losses", "mious", "conf", "pred"):
        np.testing.assert_array_equal(a[k], b[k])


def test_partial_means_features_untouched_and_steps0_is_forward_only():
    d = tiny()
    f, lab, p = random_problem(d, seed=13)
    f0, p0 = f.copy(), p.copy()
    res = O.partial_distill(d, f, lab, p, steps=0, lr=0.1)
    np.testing.assert_array_equal(f, f0)
    np.testing.assert_array_equal(res["params"], p0)
    assert res["losses"].shape == (1,)
    res = O.partial_distill(d, f, lab, p, steps=2, lr=0.1)
    np.testing.assert_array_equal(f, f0)
    np.testing.assert_array_equal(p, p0)          # caller's array is not modified either


def test_bf16_operand_mode_against_library_replay():
    """Rounding points of the 'bf16 in, fp32 accumulate' variant: features, weights, a1, a2,
    the low-resolution loss gradient g, da2, da1.  Replayed with library convolutions."""
    d = tiny(n=1, c_in=4, h=5, w=6, c1=6, c2=5, C=4, bf16=True)
    f, lab, p = random_problem(d, seed=17)
    f = O.round_bf16(f)
    loss, grad, *_ = O.loss_and_grad(d, f, lab, p)

    def q(t):
        return t.to(torch.float32).to(torch.bfloat16).to(torch.float64)

    W1, b1, W2, b2, W3, b3 = [T(a.copy()) for a in split(d, p)]
    ft = T(f)
    a1 = q(F.relu(F.conv2d(ft, q(W1), b1, padding=1)))
    a2 = q(F.relu(F.conv2d(a1, q(W2), b2, padding=1)))
    z = F.conv2d(a2, q(W3), b3).requires_grad_()
    Z = F.interpolate(z, scale_factor=8, mode="bilinear", align_corners=False)
    L = F.cross_entropy(Z, T(lab).long())
    L.backward()
    g = q(z.grad)
    from torch.nn.grad import conv2d_input, conv2d_weight
    dW3 = conv2d_weight(a2, W3.shape, g)
    da2 = q(conv2d_input(a2.shape, q(W3), g) * (a2 > 0))
    dW2 = conv2d_weight(a1, W2.shape, da2, padding=1)
    da1 = q(conv2d_input(a1.shape, q(W2), da2, padding=1) * (a1 > 0))
    dW1 = conv2d_weight(ft, W1.shape, da1, padding=1)
    ref = torch.cat([dW1.ravel(), da1.sum((0, 2, 3)), dW2.ravel(), da2.sum((0, 2, 3)),
                     dW3.ravel(), g.sum((0, 2, 3))]).numpy()
    assert abs(loss - L.item()) < 1e-12
    np.testing.assert_allclose(grad, ref, rtol=1e-9, atol=1e-14)
    # and it stays close to the unrounded gradient (bf16 has 8 significant bits)
    d64 = tiny(n=1, c_in=4, h=5, w=6, c1=6, c2=5, C=4, bf16=False)
    _, g64, *_ = O.loss_and_grad(d64, f, lab, p)
    assert np.max(np.abs(grad - g64)) < 2e-2 * np.max(np.abs(g64))


def learnable_problem():
    wl = WL.small_variant(WL.WORKLOADS["tiny"], c_in=8, h=6, w=6, c1=8, c2=8, n_classes=3,
                          n_sites=5, label_seed=5, feat_dtype="f32", compute="f32")
    lab = WL.make_labels(wl)
    f = WL.make_learnable_features(wl, lab).astype(np.float64)
    p = WL.make_head_params(wl).astype(np.float64)
    return O.desc_of(wl), f, lab, p


def test_training_loop_exits_follow_algorithm_1():
    d, f, lab, p = learnable_problem()
    trace = O.partial_distill(d, f, lab, p, steps=8, lr=0.05)
    m = trace["mious"][:, 0]
    assert m.max() > m[0] + 0.05, "the test problem must be learnable"
    # (a) first metric already at THRESHOLD or above: no update, parameters returned unchanged
    r = O.train(d, f, lab, p, max_updates=8, lr=0.05, threshold=m[0])
    assert r["updates"] == 0 and r["best_metric"] == m[0]
    np.testing.assert_array_equal(r["params"], p)
    # (b) unreachable THRESHOLD: all updates taken, the best (first strict maximum) returned
    r = O.train(d, f, lab, p, max_updates=8, lr=0.05, threshold=1.5)
    assert r["updates"] == 8
    np.testing.assert_array_equal(r["metrics"], m)
    best_i = int(np.argmax(m))           # argmax returns the first maximum = strict '>' rule
    assert r["best_metric"] == m[best_i]
    ref = O.partial_distill(d, f, lab, p, steps=best_i, lr=0.05)["params"]
    np.testing.assert_array_equal(r["params"], ref)
    # (c) reachable THRESHOLD: leave at the first metric strictly above it
    thr = float(np.sort(m)[len(m) // 2])
    first = next(i for i in range(1, 9) if m[i] > thr) if m[0] < thr else 0
    r = O.train(d, f, lab, p, max_updates=8, lr=0.05, threshold=thr)
    assert r["updates"] == first
    # (d) '>=' variant stops when the metric equals THRESHOLD exactly; '>' does not
    j = next(i for i in range(1, 9) if m[i] > m[0])
    r_ge = O.train(d, f, lab, p, max_updates=8, lr=0.05, threshold=m[j], strict_break=False)
    r_gt = O.train(d, f, lab, p, max_updates=8, lr=0.05, threshold=m[j], strict_break=True)
    assert r_ge["updates"] == j and r_gt["updates"] > j


def test_training_loop_comparisons_on_exact_ties():
    """The three comparisons of Algorithm 1 on metrics that tie exactly.  With a step so small that
    no pixel changes its class, every iteration scores the same while the parameters do move:
      * best update is strictly-better ('>'): best_student stays the initial one ('>=' would
        return the last parameters);
      * the entry test is 'best_metric < THRESHOLD': a first metric equal to THRESHOLD skips the
        loop ('<=' would train);
      * the exit is 'metric > THRESHOLD' as printed: a metric equal to THRESHOLD does not leave
        the loop, the '>=' variant does at the first update."""
    d, f, lab, p = learnable_problem()
    lr = 1e-12
    trace = O.partial_distill(d, f, lab, p, steps=3, lr=lr)
    m = trace["mious"][:, 0]
    assert (m == m[0]).all(), "the step must be too small to change any predicted class"
    assert not np.array_equal(trace["params"], p)
    r = O.train(d, f, lab, p, max_updates=3, lr=lr, threshold=1.5)
    assert r["updates"] == 3 and r["best_metric"] == m[0]
    np.testing.assert_array_equal(r["metrics"], m)
    np.testing.assert_array_equal(r["params"], p)
    r = O.train(d, f, lab, p, max_updates=3, lr=lr, threshold=m[0])
    assert r["updates"] == 0
    np.testing.assert_array_equal(r["params"], p)
    above = np.nextafter(m[0], 2.0)
    r = O.train(d, f, lab, p, max_updates=3, lr=lr, threshold=above)
    assert r["updates"] == 3                       # below THRESHOLD by one ulp: trains, never exceeds it
    # exit comparison: learnable run, THRESHOLD exactly at the first metric that beats the start
    full = O.partial_distill(d, f, lab, p, steps=8, lr=0.05)["mious"][:, 0]
    j = next(i for i in range(1, 9) if full[i] > full[0])
    later = next(i for i in range(j + 1, 9) if full[i] > full[j])
    assert O.train(d, f, lab, p, 8, 0.05, threshold=full[j], strict_break=True)["updates"] == later
    assert O.train(d, f, lab, p, 8, 0.05, threshold=full[j], strict_break=False)["updates"] == j


def test_best_is_not_last_with_momentum():
    """A run whose metric rises and then falls (large step, momentum): Algorithm 1 returns the
    parameters of the best iteration, which are those of a fixed-step run of that length."""
    d, f, lab, p = learnable_problem()
    r = O.train(d, f, lab, p, max_updates=8, lr=0.2, threshold=1.5, momentum=0.9)
    m = r["metrics"]
    best_i = int(np.argmax(m))
    assert 0 < best_i < 8 and m[8] < m[best_i] - 0.1, m
    assert r["best_metric"] == m[best_i]
    ref = O.partial_distill(d, f, lab, p, steps=best_i, lr=0.2, momentum=0.9)
    np.testing.assert_array_equal(r["params"], ref["params"])


# ------------------------------------------------------------------ gradient with respect to the features
def test_feature_gradient_against_autograd_and_finite_differences():
    """d loss / d features (what an unfrozen front part would receive) against CPU PyTorch
    autograd through the same head, and against central differences on a few entries."""
    import torch
    import torch.nn.functional as F
    wl = WL.small_variant(WL.WORKLOADS["tiny"], n=2, c_in=3, h=4, w=5, c1=4, c2=3, n_classes=3, n_sites=5,
                          ignore_index=255, ignore_fraction=0.1)
    d = O.desc_of(wl)
    f = WL.features_as_f64(wl, WL.make_features(wl))
    lab = WL.make_labels(wl)
    p = WL.make_head_params(wl).astype(np.float64)
    p += np.random.default_rng(3).standard_normal(p.size) * 0.05
    loss, grad, df = O.feature_grad(d, f, lab, p)
    loss2, grad2, _, _, _ = O.loss_and_grad(d, f, lab, p)
    assert loss == loss2
    np.testing.assert_array_equal(grad, grad2)
    sl = WL.param_slices(wl)
    ft = torch.tensor(f, requires_grad=True)
    W1 = torch.tensor(p[sl["W1"]].reshape(wl.c1, wl.c_in, 3, 3)); b1 = torch.tensor(p[sl["b1"]])
    W2 = torch.tensor(p[sl["W2"]].reshape(wl.c2, wl.c1, 3, 3)); b2 = torch.tensor(p[sl["b2"]])
    W3 = torch.tensor(p[sl["W3"]].reshape(wl.n_classes, wl.c2, 1, 1)); b3 = torch.tensor(p[sl["b3"]])
    z = F.conv2d(F.relu(F.conv2d(F.relu(F.conv2d(ft, W1, b1, padding=1)), W2, b2, padding=1)), W3, b3)
    Z = F.interpolate(z, scale_factor=8, mode="bilinear", align_corners=False)
    lt = torch.tensor(np.where(lab == 255, -100, lab).astype(np.int64))
    ref = F.cross_entropy(Z, lt, ignore_index=-100)
    ref.backward()
    assert abs(loss - ref.item()) < 1e-12
    np.testing.assert_allclose(df, ft.grad.numpy(), rtol=0, atol=1e-13)
    rng = np.random.default_rng(4)
    for _ in range(10):
        idx = tuple(rng.integers(0, s) for s in f.shape)
        e = np.zeros_like(f); e[idx] = 1e-6
        lp = O.loss_and_grad(d, f + e, lab, p, want_grad=False)[0]
        lm = O.loss_and_grad(d, f - e, lab, p, want_grad=False)[0]
        assert abs((lp - lm) / 2e-6 - df[idx]) < 1e-7 + 1e-5 * abs(df[idx])


def test_grouped_heads_are_independent_runs():
    """The grouped form (one head and one frame per client, Algorithm 3) is n separate runs: head
    f's trace is that of a single-frame run on frame f, whatever the other frames hold, and the
    per-head columns of the result come in the frames' order."""
    wl = WL.small_variant(WL.WORKLOADS["tiny"], n=3, c_in=4, h=3, w=4, c1=5, c2=4, n_classes=3, n_sites=5, steps=2)
    f = WL.features_as_f64(wl, WL.make_features(wl))
    lab = WL.make_labels(wl)
    p = np.stack([WL.make_head_params(wl, seed=11 + i) for i in range(3)]).astype(np.float64)
    d = O.desc_of(wl)
    opt = O.Optim(0, 0.05, 0.9, 0, 0, 0, 0)
    g = O.partial_distill_grouped(d, f, lab, p, 2, opt)
    assert g["params"].shape == p.shape and g["losses"].shape == (3, 3) and g["mious"].shape == (3, 3)
    d1 = O.desc(1, wl.c_in, wl.h, wl.w, wl.c1, wl.c2, wl.n_classes)
    for i in range(3):
        s = O.partial_distill(d1, f[i:i + 1], lab[i:i + 1], p[i], 2, 0.05, momentum=0.9)
        np.testing.assert_array_equal(g["params"][i], s["params"])
        np.testing.assert_array_equal(g["losses"][:, i], s["losses"])
        np.testing.assert_array_equal(g["mious"][:, i], s["mious"][:, 0])
        np.testing.assert_array_equal(g["s1"][i], s["velocity"])
    # other clients' frames do not matter, and it is not the shared-head mini-batch
    f2, lab2 = f.copy(), lab.copy()
    f2[1:] *= -0.5
    lab2[1:] = (lab2[1:] + 1) % wl.n_classes
    g2 = O.partial_distill_grouped(d, f2, lab2, p, 2, opt)
    np.testing.assert_array_equal(g2["params"][0], g["params"][0])
    assert not np.array_equal(g2["params"][1], g["params"][1])
    shared = O.partial_distill(d, f, lab, p[0], 2, 0.05, momentum=0.9)
    assert not np.allclose(shared["params"], g["params"][0])


@pytest.mark.parametrize("name,steps", [("720p", 8), ("1080p", 2), ("batch4", 1)])
def test_full_size_key_frame_matches_library_loop(name, steps):
    """The measured workloads themselves (1280x720: all eight steps; 1920x1080 with ignored pixels
    and momentum: two; the batch of four frames with the wider head: one), float64, against the
    same loop written with CPU PyTorch autograd and torch.optim.SGD: losses of every pass and the
    trained parameters."""
    torch.set_num_threads(8)
    wl = WL.WORKLOADS[name]
    d = O.desc_of(wl, False)
    f = WL.features_as_f64(wl, WL.make_features(wl))
    lab = WL.make_labels(wl)
    p = WL.make_head_params(wl).astype(np.float64)
    res = O.partial_distill(d, f, lab, p, steps, wl.lr, momentum=wl.momentum)
    pt = T(p.copy()).requires_grad_()
    opt = torch.optim.SGD([pt], lr=wl.lr, momentum=wl.momentum)
    ft, labt = T(f), T(lab)
    losses = []
    for it in range(steps + 1):
        opt.zero_grad()
        loss_t, _, _ = torch_loss(d, ft, labt, pt)
        losses.append(loss_t.item())
        if it == steps:
            break
        loss_t.backward()
        opt.step()
    torch.set_num_threads(4)
    np.testing.assert_allclose(res["losses"], losses, rtol=1e-11)
    np.testing.assert_allclose(res["params"], pt.detach().numpy(), rtol=0, atol=1e-12)
    assert np.abs(res["params"] - p).max() > 1e-4        # the steps did move the head


def test_identity_convolutions_reduce_the_head_to_logistic_regression():
    """With centre-delta 3x3 kernels and positive features both hidden layers are the identity,
    and since a 1x1 convolution commutes with the (linear, per-channel) up-sampling the head is
    multinomial logistic regression on the up-sampled features: loss and the textbook gradient
    X^T (softmax - onehot) / N for the classifier, written out here in numpy."""
    C_IN, NC = 4, 3
    d = tiny(n=2, c_in=C_IN, h=4, w=5, c1=C_IN, c2=C_IN, C=NC)
    rng = np.random.default_rng(5)
    f = rng.random((d.n, C_IN, d.h, d.w)) + 0.1
    lab = rng.integers(0, NC, size=(d.n, 8 * d.h, 8 * d.w)).astype(np.int32)
    eye = np.zeros((C_IN, C_IN, 3, 3))
    eye[np.arange(C_IN), np.arange(C_IN), 1, 1] = 1.0
    W3 = rng.standard_normal((NC, C_IN))
    b3 = rng.standard_normal(NC)
    p = np.concatenate([eye.ravel(), np.zeros(C_IN), eye.ravel(), np.zeros(C_IN), W3.ravel(), b3])
    loss, grad, *_ = O.loss_and_grad(d, f, lab, p)
    # the design matrix: every frame pixel's up-sampled feature vector (an independent library's
    # interpolation), one row per pixel
    X = F.interpolate(T(f), scale_factor=8, mode="bilinear", align_corners=False).numpy()
    X = X.transpose(0, 2, 3, 1).reshape(-1, C_IN)
    y = lab.reshape(-1)
    logits = X @ W3.T + b3
    logits -= logits.max(axis=1, keepdims=True)
    P = np.exp(logits)
    P /= P.sum(axis=1, keepdims=True)
    N = y.size
    assert abs(loss - (-np.log(P[np.arange(N), y]).mean())) < 1e-12
    R = P.copy()
    R[np.arange(N), y] -= 1.0
    n3 = NC * C_IN + NC
    np.testing.assert_allclose(grad[-n3:-NC].reshape(NC, C_IN), R.T @ X / N, atol=1e-13)
    np.testing.assert_allclose(grad[-NC:], R.sum(axis=0) / N, atol=1e-13)

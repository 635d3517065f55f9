"""Pins of the CPU oracle against things other than itself.

Each test names what it pins and with what: an independent library routine (CPU PyTorch in
float64), a closed form, an invariant of the mathematics, brute force, or central finite
differences.  None of these tests touches a GPU.
"""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle as O
import workloads as WL

torch.set_num_threads(4)
RNG = np.random.default_rng(12345)


def T(a):
    return torch.from_numpy(np.ascontiguousarray(a))


# ------------------------------------------------------------------ convolution
@pytest.mark.parametrize("k", [1, 3])
@pytest.mark.parametrize("shape", [(1, 3, 4, 5, 4), (2, 5, 7, 6, 3)])
def test_conv_fwd_matches_library(k, shape):
    n, ci, h, w, co = shape
    x = RNG.standard_normal((n, ci, h, w))
    W = RNG.standard_normal((co, ci, k, k))
    b = RNG.standard_normal(co)
    ref = F.conv2d(T(x), T(W), T(b), padding=k // 2).numpy()
    np.testing.assert_allclose(O.conv_fwd(x, W, b), ref, rtol=1e-12, atol=1e-12)


def test_conv1x1_is_matmul():
    x = RNG.standard_normal((2, 6, 3, 4))
    W = RNG.standard_normal((5, 6, 1, 1))
    y = O.conv_fwd(x, W, None)
    ref = np.einsum("oi,nihw->nohw", W[:, :, 0, 0], x)
    np.testing.assert_allclose(y, ref, rtol=1e-12, atol=1e-12)


def test_conv3x3_centre_delta_is_identity_and_shifts():
    x = RNG.standard_normal((1, 3, 5, 6))
    W = np.zeros((3, 3, 3, 3))
    for c in range(3):
        W[c, c, 1, 1] = 1.0
    np.testing.assert_array_equal(O.conv_fwd(x, W, None), x)
    # a tap at (kh, kw) = (0, 2) reads the input one row up and one column right
    W = np.zeros((1, 1, 3, 3))
    W[0, 0, 0, 2] = 1.0
    x1 = RNG.standard_normal((1, 1, 4, 4))
    y = O.conv_fwd(x1, W, None)
    ref = np.zeros_like(x1)
    ref[0, 0, 1:, :-1] = x1[0, 0, :-1, 1:]
    np.testing.assert_array_equal(y, ref)


@pytest.mark.parametrize("k", [1, 3])
def test_conv_adjoint_identities(k):
    n, ci, co, h, w = 2, 4, 3, 5, 7
    x = RNG.standard_normal((n, ci, h, w))
    W = RNG.standard_normal((co, ci, k, k))
    y = RNG.standard_normal((n, co, h, w))
    lhs = float((O.conv_fwd(x, W, None) * y).sum())
    assert abs(lhs - float((x * O.conv_dgrad(y, W)).sum())) < 1e-9 * max(1, abs(lhs))
    dW, db = O.conv_wgrad(x, y, k)
    assert abs(lhs - float((W * dW).sum())) < 1e-9 * max(1, abs(lhs))
    np.testing.assert_allclose(db, y.sum(axis=(0, 2, 3)), rtol=1e-12)


@pytest.mark.parametrize("k", [1, 3])
def test_conv_grads_match_library_autograd(k):
    n, ci, co, h, w = 2, 3, 4, 6, 5
    x = T(RNG.standard_normal((n, ci, h, w))).requires_grad_()
    W = T(RNG.standard_normal((co, ci, k, k))).requires_grad_()
    b = T(RNG.standard_normal(co)).requires_grad_()
    dy = RNG.standard_normal((n, co, h, w))
    F.conv2d(x, W, b, padding=k // 2).backward(T(dy))
    np.testing.assert_allclose(O.conv_dgrad(dy, W.detach().numpy()), x.grad.numpy(), atol=1e-11)
    dW, db = O.conv_wgrad(x.detach().numpy(), dy, k)
    np.testing.assert_allclose(dW, W.grad.numpy(), atol=1e-11)
    np.testing.assert_allclose(db, b.grad.numpy(), atol=1e-11)


# ------------------------------------------------------------------ up-sampling
def test_upsample_matches_library_half_pixel_convention():
    z = RNG.standard_normal((2, 3, 5, 7))
    ref = F.interpolate(T(z), scale_factor=8, mode="bilinear", align_corners=False).numpy()
    np.testing.assert_allclose(O.upsample8(z), ref, rtol=1e-12, atol=1e-12)


def test_upsample_constant_ramp_and_weights():
    c = np.full((1, 1, 3, 4), 0.7310585786300049)
    assert np.all(O.upsample8(c) == c[0, 0, 0, 0])
    assert np.all(O.upsample8_f32(c) == np.float32(c[0, 0, 0, 0]))
    # impulse response = interpolation weights: multiples of 1/16 per axis, summing to 1
    for (iy, ix) in [(0, 0), (1, 2), (2, 3)]:
        d = np.zeros((1, 1, 3, 4))
        d[0, 0, iy, ix] = 1.0
        Z = O.upsample8(d)[0, 0]
        assert np.all(Z * 256 == np.round(Z * 256))
    ones = sum(O.upsample8(np.eye(12)[i].reshape(1, 1, 3, 4)) for i in range(12))
    np.testing.assert_array_equal(ones, np.ones((1, 1, 24, 32)))
    # a linear ramp is reproduced exactly between the first and last cell centres
    h, w = 4, 6
    ramp = (2.0 * np.arange(h)[:, None] + 3.0 * np.arange(w)[None, :]).reshape(1, 1, h, w)
    Z = O.upsample8(ramp)[0, 0]
    Y, X = np.meshgrid(np.arange(8 * h), np.arange(8 * w), indexing="ij")
    sy, sx = (Y + 0.5) / 8 - 0.5, (X + 0.5) / 8 - 0.5
    inside = (sy >= 0) & (sy <= h - 1) & (sx >= 0) & (sx <= w - 1)
    np.testing.assert_allclose(Z[inside], (2.0 * sy + 3.0 * sx)[inside], rtol=0, atol=1e-12)
    # phase weights for destination index 8q + j: {9,11,13,15,1,3,5,7}/16
    line = np.zeros((1, 1, 1, 3))
    line[0, 0, 0, 1] = 1.0
    row = O.upsample8(line)[0, 0, 0]
    np.testing.assert_array_equal(row[8:16] * 16, [9, 11, 13, 15, 15, 13, 11, 9])


def test_upsample_adjoint():
    n, c, h, w = 2, 3, 4, 5
    x = RNG.standard_normal((n, c, h, w))
    y = RNG.standard_normal((n, c, 8 * h, 8 * w))
    lhs = float((O.upsample8(x) * y).sum())
    rhs = float((x * O.upsample8_adjoint(y)).sum())
    assert abs(lhs - rhs) < 1e-10 * abs(lhs)
    np.testing.assert_allclose(O.upsample8_adjoint(y).sum(axis=(2, 3)), y.sum(axis=(2, 3)),
                               rtol=1e-12)


def test_upsample_f32_close_to_f64_and_rounds_once_per_op():
    z = RNG.standard_normal((1, 2, 4, 5)).astype(np.float32)
    Zf = O.upsample8_f32(z)
    Zd = O.upsample8(z.astype(np.float64))
    assert np.max(np.abs(Zf - Zd)) < 4e-7 * np.max(np.abs(Zd))
    # replay the stated operation order with numpy float32 scalars and exact float64 fma
    def lerp(a, b, t):
        d = np.float32(b - a)
        return np.float32(np.float64(t) * np.float64(d) + np.float64(a))
    # (float64 holds the 24x24-bit product exactly and the sum to within its own rounding; a
    #  double rounding could differ from a true fma only in rare ties, so compare to 1 ulp and
    #  require most values identical)
    h, w = 4, 5
    exact = 0
    for Y in range(8 * h):
        sy = (Y + 0.5) / 8 - 0.5
        y0 = math.floor(sy); wy = np.float32(sy - y0)
        y1 = min(max(y0 + 1, 0), h - 1); y0 = min(max(y0, 0), h - 1)
        for X in range(8 * w):
            sx = (X + 0.5) / 8 - 0.5
            x0 = math.floor(sx); wx = np.float32(sx - x0)
            x1 = min(max(x0 + 1, 0), w - 1); x0 = min(max(x0, 0), w - 1)
            p = z[0, 1]
            r0 = lerp(p[y0, x0], p[y0, x1], wx)
            r1 = lerp(p[y1, x0], p[y1, x1], wx)
            v = lerp(r0, r1, wy)
            assert abs(float(v) - float(Zf[0, 1, Y, X])) <= np.spacing(abs(v))
            exact += int(v == Zf[0, 1, Y, X])
    assert exact >= 0.99 * 64 * h * w


# ------------------------------------------------------------------ loss
def test_softmax_ce_matches_library_with_ignore():
    n, c, H, W = 2, 5, 8, 16
    Z = 3.0 * RNG.standard_normal((n, c, H, W))
    lab = RNG.integers(0, c, size=(n, H, W)).astype(np.int32)
    lab[RNG.random(lab.shape) < 0.2] = 255
    Zt = T(Z).requires_grad_()
    ref = F.cross_entropy(Zt, T(lab).long(), ignore_index=255)
    ref.backward()
    loss, G, nv = O.softmax_ce(Z, lab, ignore_index=255)
    assert nv == int((lab != 255).sum())
    assert abs(loss - ref.item()) < 1e-12
    np.testing.assert_allclose(G, Zt.grad.numpy(), atol=1e-14)


@pytest.mark.parametrize("C", [9, 19, 21])
def test_softmax_ce_uniform_logits_is_log_C(C):
    golden = {}
    import os
    with open(os.path.join(os.path.dirname(__file__), "golden", "closed_forms.txt")) as fh:
        for line in fh:
            if line.strip() and not line.startswith("#"):
                k, v = line.split()[:2]
                golden[k] = float(v)
    Z = np.zeros((1, C, 8, 8))
    lab = RNG.integers(0, C, size=(1, 8, 8)).astype(np.int32)
    loss, G, nv = O.softmax_ce(Z, lab)
    assert abs(loss - golden[f"ln{C}"]) < 1e-5          # printed to 5 decimals
    assert abs(loss - math.log(C)) < 1e-14
    onehot = np.eye(C)[lab].transpose(0, 3, 1, 2)
    np.testing.assert_allclose(G, (1.0 / C - onehot) / nv, atol=1e-16)


def test_softmax_ce_invariants():
    n, c, H, W = 1, 4, 8, 8
    Z = 10.0 * RNG.standard_normal((n, c, H, W))
    lab = RNG.integers(0, c, size=(n, H, W)).astype(np.int32)
    loss, G, _ = O.softmax_ce(Z, lab)
    assert loss >= 0.0
    np.testing.assert_allclose(G.sum(axis=1), 0.0, atol=1e-15)
    # shifting all logits of a pixel leaves the loss unchanged; huge logits do not overflow
    loss2, _, _ = O.softmax_ce(Z + 1000.0, lab)
    assert abs(loss - loss2) < 1e-9
    # all pixels ignored: loss 0, gradient 0
    loss3, G3, nv3 = O.softmax_ce(Z, np.full_like(lab, 255), ignore_index=255)
    assert loss3 == 0.0 and nv3 == 0 and not G3.any()


# ------------------------------------------------------------------ metric
def brute_force_miou(pred, lab, C, ignore):
    valid = [(p, l) for p, l in zip(pred.ravel().tolist(), lab.ravel().tolist())
             if l != ignore and 0 <= l < C]
    ious = []
    for c in range(C):
        pred_c = {i for i, (p, l) in enumerate(valid) if p == c}
        label_c = {i for i, (p, l) in enumerate(valid) if l == c}
        if label_c:
            ious.append(len(pred_c & label_c) / len(pred_c | label_c))
    return sum(ious) / len(ious) if ious else 0.0


def test_confusion_and_miou_brute_force():
    C = 5
    pred = RNG.integers(0, C, size=(12, 9)).astype(np.uint8)
    lab = RNG.integers(0, C - 1, size=(12, 9)).astype(np.int32)   # class C-1 never in the label
    lab[RNG.random(lab.shape) < 0.1] = 255
    conf = O.confusion(pred, lab, C, ignore_index=255)
    assert conf.sum() == int((lab != 255).sum())
    for a in range(C):
        for b in range(C):
            assert conf[a, b] == int(((lab == a) & (pred == b)).sum())
    m, present = O.miou(conf)
    assert present == len(set(lab[lab != 255].tolist()))
    assert abs(m - brute_force_miou(pred, lab, C, 255)) < 1e-15


def test_miou_special_cases():
    C = 4
    lab = RNG.integers(0, C, size=(16, 16)).astype(np.int32)
    assert O.miou(O.confusion(lab.astype(np.uint8), lab, C))[0] == 1.0
    perm = ((lab + 1) % C).astype(np.uint8)
    assert O.miou(O.confusion(perm, lab, C))[0] == 0.0
    # a class that is predicted but absent from the label adds no term of its own
    lab2 = np.array([[0, 0, 1, 1]], dtype=np.int32)
    pred2 = np.array([[0, 2, 1, 1]], dtype=np.uint8)
    m, present = O.miou(O.confusion(pred2, lab2, 3))
    assert present == 2 and abs(m - (0.5 + 1.0) / 2) < 1e-15
    # nothing valid
    assert O.miou(np.zeros((3, 3), dtype=np.int64)) == (0.0, 0)
    # argmax ties go to the lowest class index
    Z = np.zeros((1, 3, 8, 8), dtype=np.float32)
    Z[0, 1] = 1.0
    Z[0, 2] = 1.0
    assert np.all(O.argmax_f32(Z) == 1)


# ------------------------------------------------------------------ optimiser
def test_sgd_hand_computed_and_library():
    theta = np.array([1.0, -2.0, 0.5])
    g1 = np.array([0.5, 0.25, -1.0])
    g2 = np.array([-1.0, 0.5, 2.0])
    t1, v1 = O.sgd(theta, g1, np.zeros(3), lr=0.1, mu=0.9)
    np.testing.assert_allclose(v1, g1)
    np.testing.assert_allclose(t1, [0.95, -2.025, 0.6])
    t2, v2 = O.sgd(t1, g2, v1, lr=0.1, mu=0.9)
    np.testing.assert_allclose(v2, [-0.55, 0.725, 1.1])
    np.testing.assert_allclose(t2, [1.005, -2.0975, 0.49])
    # mu = 0 equals plain descent bit for bit
    p0, _ = O.sgd(theta, g1, None, lr=0.1, mu=0.0)
    pm, _ = O.sgd(theta, g1, np.zeros(3), lr=0.1, mu=0.0)
    np.testing.assert_array_equal(p0, theta - 0.1 * g1)
    np.testing.assert_array_equal(p0, pm)
    # library optimiser, three steps
    p = torch.tensor(theta.copy(), requires_grad=True)
    opt = torch.optim.SGD([p], lr=0.1, momentum=0.9)
    th, v = theta.copy(), np.zeros(3)
    for g in (g1, g2, g1):
        p.grad = T(g.copy())
        opt.step()
        th, v = O.sgd(th, g, v, lr=0.1, mu=0.9)
    np.testing.assert_allclose(th, p.detach().numpy(), rtol=1e-14)


# ------------------------------------------------------------------ bfloat16 rounding
def test_bf16_rounding_matches_library_and_ties_to_even():
    x = np.concatenate([RNG.standard_normal(4096) * 10.0 ** RNG.integers(-6, 6, 4096),
                        [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895313892515355e38]])
    ref = T(x.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(O.round_bf16(x), ref)
    # 1 + 2^-8 lies halfway between 1 and 1 + 2^-7: even mantissa wins -> 1.0
    assert O.round_bf16(np.array([1.00390625]))[0] == 1.0
    # 1 + 3*2^-8 lies halfway between 1+2^-7 and 1+2^-6 -> 1 + 2^-6
    assert O.round_bf16(np.array([1.01171875]))[0] == 1.015625


# ------------------------------------------------------------------ Adam (Section 5.2: the paper's optimiser)
def test_adam_first_step_closed_form():
    """From zero state the bias-corrected moments of step 1 are g and g^2, so the step is
    -lr * g / (|g| + eps) whatever beta1, beta2 are."""
    rng = np.random.default_rng(11)
    theta, g = rng.standard_normal(257), rng.standard_normal(257) * 1e-3
    g[::17] = 0.0
    for b1, b2 in ((0.9, 0.999), (0.5, 0.8)):
        t1, m, v = O.adam(theta, g, np.zeros(257), np.zeros(257), 0.01, b1, b2, 1e-8, 1)
        np.testing.assert_allclose(t1, theta - 0.01 * g / (np.abs(g) + 1e-8), rtol=0, atol=1e-15)
        np.testing.assert_allclose(m, (1 - b1) * g, rtol=1e-15, atol=0)
        np.testing.assert_allclose(v, (1 - b2) * g * g, rtol=1e-15, atol=0)
    assert np.all(t1[::17] == theta[::17])   # zero gradient: no move


def test_adam_constant_gradient_walks_at_lr():
    """With the same gradient every step, mhat = g and vhat = g^2 for every t: each step moves
    every parameter by lr * g / (|g| + eps), i.e. by lr against the gradient's sign."""
    g = np.array([2.0, -0.5, 1e-3, -7.0])
    theta, m, v = np.zeros(4), np.zeros(4), np.zeros(4)
    for t in range(1, 21):
        theta, m, v = O.adam(theta, g, m, v, 0.01, 0.9, 0.999, 1e-8, t)
    np.testing.assert_allclose(theta, -20 * 0.01 * g / (np.abs(g) + 1e-8), rtol=1e-12)


def test_adam_matches_independent_library():
    """Ten steps on a changing gradient against torch.optim.Adam (float64, CPU)."""
    rng = np.random.default_rng(12)
    x0 = rng.standard_normal(300)
    grads = [rng.standard_normal(300) * (0.1 + i) for i in range(10)]
    w = torch.tensor(x0.copy(), dtype=torch.float64, requires_grad=True)
    opt = torch.optim.Adam([w], lr=0.01, betas=(0.9, 0.999), eps=1e-8)
    theta, m, v = x0.copy(), np.zeros(300), np.zeros(300)
    for t, g in enumerate(grads, start=1):
        w.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        theta, m, v = O.adam(theta, g, m, v, 0.01, 0.9, 0.999, 1e-8, t)
        np.testing.assert_allclose(theta, w.detach().numpy(), rtol=0, atol=1e-13)


def test_adam_loop_equals_manual_steps():
    """The optimiser-generic loop with Adam is the manual sequence loss/gradient -> Adam step,
    with the step counter continuing from t0."""
    wl = WL.small_variant(WL.WORKLOADS["tiny"], c_in=4, h=4, w=5, c1=4, c2=4, n_classes=3, n_sites=4)
    d = O.desc_of(wl)
    f = WL.features_as_f64(wl, WL.make_features(wl))
    lab = WL.make_labels(wl)
    p0 = WL.make_head_params(wl).astype(np.float64)
    r = O.partial_distill_opt(d, f, lab, p0, 3, O.adam_optim(0.01, t0=5))
    theta, m, v = p0.copy(), np.zeros_like(p0), np.zeros_like(p0)
    for k in range(3):
        loss, grad, _ = O.loss_and_grad(d, f, lab, theta)[:3]
        assert loss == r["losses"][k]
        theta, m, v = O.adam(theta, grad, m, v, 0.01, 0.9, 0.999, 1e-8, 5 + k + 1)
    np.testing.assert_array_equal(theta, r["params"])
    np.testing.assert_array_equal(m, r["s1"])
    np.testing.assert_array_equal(v, r["s2"])
    # and the descent-with-momentum description reproduces the dedicated entry point
    a = O.partial_distill(d, f, lab, p0, 3, 0.01, momentum=0.9)
    b = O.partial_distill_opt(d, f, lab, p0, 3, O.Optim(0, 0.01, 0.9, 0, 0, 0, 0))
    np.testing.assert_array_equal(a["params"], b["params"])


# ------------------------------------------------------------------ weighted cross-entropy (Section 5.2)
def test_weighted_ce_matches_independent_library():
    """sum_p w_p CE_p / sum_p w_p and its gradient against CPU PyTorch (per-pixel losses from
    F.cross_entropy, weighting and autograd by torch), with ignored pixels."""
    rng = np.random.default_rng(21)
    n, Cn, H, W = 2, 5, 8, 16
    Z = rng.standard_normal((n, Cn, H, W)) * 3
    lab = rng.integers(0, Cn, size=(n, H, W)).astype(np.int32)
    lab[rng.random(lab.shape) < 0.1] = 255
    wts = rng.choice([1, 5], size=(n, H, W)).astype(np.uint8)
    loss, G, wsum = O.softmax_ce(Z, lab, ignore_index=255, weights=wts)
    zt = torch.tensor(Z, dtype=torch.float64, requires_grad=True)
    lt = torch.tensor(np.where(lab == 255, -100, lab).astype(np.int64))
    per = F.cross_entropy(zt, lt, ignore_index=-100, reduction="none")
    wt = torch.tensor(wts.astype(np.float64)) * (lt != -100)
    ref = (per * wt).sum() / wt.sum()
    ref.backward()
    assert wsum == int(wt.sum().item())
    assert abs(loss - ref.item()) < 1e-12
    np.testing.assert_allclose(G, zt.grad.numpy(), rtol=0, atol=1e-14)


def test_weighted_ce_special_cases():
    rng = np.random.default_rng(22)
    Z = rng.standard_normal((1, 4, 8, 8))
    lab = rng.integers(0, 4, size=(1, 8, 8)).astype(np.int32)
    base, G0, n0 = O.softmax_ce(Z, lab)
    # all weights 1: the unweighted mean; a constant weight changes nothing either
    l1, G1, s1 = O.softmax_ce(Z, lab, weights=np.ones((1, 8, 8), np.uint8))
    l5, G5, s5 = O.softmax_ce(Z, lab, weights=np.full((1, 8, 8), 5, np.uint8))
    assert l1 == base and s1 == n0 and s5 == 5 * n0
    np.testing.assert_array_equal(G1, G0)
    np.testing.assert_allclose(G5, G0, rtol=1e-15, atol=1e-18)
    assert abs(l5 - base) < 1e-15
    # weight 0 removes a pixel exactly like the ignore label does
    w0 = np.ones((1, 8, 8), np.uint8); w0[0, 3, 4] = 0
    lab_ign = lab.copy(); lab_ign[0, 3, 4] = 255
    la, Ga, _ = O.softmax_ce(Z, lab, weights=w0)
    lb, Gb, _ = O.softmax_ce(Z, lab_ign, ignore_index=255)
    assert abs(la - lb) < 1e-15
    np.testing.assert_allclose(Ga, Gb, rtol=0, atol=1e-17)
    # uniform logits: every pixel's loss is ln C, so is any weighted mean of them
    lu, _, _ = O.softmax_ce(np.zeros((1, 4, 8, 8)), lab, weights=rng.choice([1, 5], size=(1, 8, 8)).astype(np.uint8))
    assert abs(lu - math.log(4)) < 1e-12


def test_weighted_loss_gradient_by_finite_differences():
    """The whole head's loss with pixel weights: analytic parameter gradient against central
    differences (the weights enter the backward pass through d loss / d logits only)."""
    wl = WL.small_variant(WL.WORKLOADS["tiny"], c_in=3, h=3, w=4, c1=4, c2=3, n_classes=3, n_sites=4)
    lab = WL.make_labels(wl)
    wts = WL.object_weight_map(lab, radius=2)
    assert set(np.unique(wts)) <= {1, 5} and (wts == 5).any()
    d = O.with_pixel_weights(O.desc_of(wl), wts)
    f = WL.features_as_f64(wl, WL.make_features(wl))
    p = WL.make_head_params(wl).astype(np.float64)
    p += np.random.default_rng(5).standard_normal(p.size) * 0.05      # biases away from zero
    loss, grad, _, _, _ = O.loss_and_grad(d, f, lab, p)
    loss_plain, _, _, _, _ = O.loss_and_grad(O.desc_of(wl), f, lab, p)
    assert loss != loss_plain
    rng = np.random.default_rng(6)
    for j in rng.choice(p.size, size=40, replace=False):
        e = np.zeros_like(p); e[j] = 1e-6
        lp = O.loss_and_grad(d, f, lab, p + e, want_grad=False)[0]
        lm = O.loss_and_grad(d, f, lab, p - e, want_grad=False)[0]
        assert abs((lp - lm) / 2e-6 - grad[j]) < 1e-7 + 1e-5 * abs(grad[j]), j


def test_object_weight_map_is_a_square_dilation():
    lab = np.zeros((1, 9, 9), np.int32)
    lab[0, 4, 4] = 3
    w = WL.object_weight_map(lab, radius=2)
    ref = np.ones((9, 9), np.uint8); ref[2:7, 2:7] = 5
    np.testing.assert_array_equal(w[0], ref)

"""ctypes front-end of the CPU oracle (oracle/st_oracle.c).

TEST INFRASTRUCTURE.  Only tests/, the smoke check and the benchmark's cpu_baseline leg may
import this package; the product (paper_2003_10735_amd) never does.  All arrays are numpy,
float64 unless said otherwise, NCHW / OIHW, C-contiguous.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

_LIB = None


class Desc(C.Structure):
    _fields_ = [("n", C.c_int32), ("c_in", C.c_int32), ("h", C.c_int32), ("w", C.c_int32),
                ("c1", C.c_int32), ("c2", C.c_int32), ("n_classes", C.c_int32),
                ("ignore_index", C.c_int32), ("bf16_operands", C.c_int32),
                ("pixel_weights", C.c_void_p)]


def lib():
    global _LIB
    if _LIB is None:
        path = _build.LIB
        if not os.path.exists(path):
            _build.build(force=True)
        _LIB = C.CDLL(path)
        _LIB.sto_softmax_ce.restype = C.c_double
        _LIB.sto_softmax_ce_w.restype = C.c_double
        _LIB.sto_loss_and_grad.restype = C.c_double
        _LIB.sto_loss_and_grad_full.restype = C.c_double
        _LIB.sto_num_params.restype = C.c_int64
        _LIB.sto_miou.restype = C.c_int
        _LIB.sto_train.restype = C.c_int
        _LIB.sto_num_threads.restype = C.c_int
    return _LIB


def num_threads() -> int:
    return int(lib().sto_num_threads())


def _d(a):
    return a.ctypes.data_as(C.POINTER(C.c_double)) if a is not None else None


def _p(a, ty):
    return a.ctypes.data_as(C.POINTER(ty)) if a is not None else None


def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def desc(n, c_in, h, w, c1, c2, n_classes, ignore_index=-1, bf16_operands=False) -> Desc:
    return Desc(n, c_in, h, w, c1, c2, n_classes, ignore_index, 1 if bf16_operands else 0, None)


def with_pixel_weights(d: Desc, weights) -> Desc:
    """A copy of the descriptor whose loss scales pixel p by weights[p] (uint8 [n,8h,8w]).  The
    returned descriptor keeps the array alive."""
    w = np.ascontiguousarray(weights, dtype=np.uint8)
    assert w.shape == (d.n, 8 * d.h, 8 * d.w)
    out = Desc(d.n, d.c_in, d.h, d.w, d.c1, d.c2, d.n_classes, d.ignore_index, d.bf16_operands,
               w.ctypes.data_as(C.c_void_p))
    out._keep = w
    return out


def desc_of(wl, bf16_operands: bool | None = None) -> Desc:
    """Descriptor of a workloads.Workload; bf16-operand rounding follows its compute type."""
    q = (wl.compute == "bf16") if bf16_operands is None else bf16_operands
    return desc(wl.n, wl.c_in, wl.h, wl.w, wl.c1, wl.c2, wl.n_classes, wl.ignore_index, q)


# ------------------------------------------------------------------ single operations
def conv_fwd(x, W, b=None):
    x, W = _f64(x), _f64(W)
    n, ci, h, w = x.shape
    co, ci2, k, k2 = W.shape
    assert ci == ci2 and k == k2 and k in (1, 3)
    b = _f64(b) if b is not None else None
    y = np.empty((n, co, h, w))
    lib().sto_conv_fwd(_d(x), _d(W), _d(b), _d(y), n, ci, co, h, w, k)
    return y


def conv_dgrad(dy, W):
    dy, W = _f64(dy), _f64(W)
    n, co, h, w = dy.shape
    co2, ci, k, _ = W.shape
    assert co == co2
    dx = np.empty((n, ci, h, w))
    lib().sto_conv_dgrad(_d(dy), _d(W), _d(dx), n, ci, co, h, w, k)
    return dx


def conv_wgrad(x, dy, k):
    x, dy = _f64(x), _f64(dy)
    n, ci, h, w = x.shape
    co = dy.shape[1]
    dW = np.empty((co, ci, k, k))
    db = np.empty(co)
    lib().sto_conv_wgrad(_d(x), _d(dy), _d(dW), _d(db), n, ci, co, h, w, k)
    return dW, db


def round_bf16(x):
    y = _f64(x).copy()
    lib().sto_round_bf16(_d(y), C.c_int64(y.size))
    return y


def upsample8(z):
    z = _f64(z)
    n, c, h, w = z.shape
    Z = np.empty((n, c, 8 * h, 8 * w))
    lib().sto_upsample8(_d(z), _d(Z), n * c, h, w)
    return Z


def upsample8_f32(z):
    z = np.ascontiguousarray(z, dtype=np.float32)
    n, c, h, w = z.shape
    Z = np.empty((n, c, 8 * h, 8 * w), dtype=np.float32)
    lib().sto_upsample8_f32(_p(z, C.c_float), _p(Z, C.c_float), n * c, h, w)
    return Z


def upsample8_adjoint(G):
    G = _f64(G)
    n, c, H, W = G.shape
    g = np.empty((n, c, H // 8, W // 8))
    lib().sto_upsample8_adjoint(_d(G), _d(g), n * c, H // 8, W // 8)
    return g


def argmax_f32(Zf):
    Zf = np.ascontiguousarray(Zf, dtype=np.float32)
    n, c, H, W = Zf.shape
    pred = np.empty((n, H, W), dtype=np.uint8)
    lib().sto_argmax_f32(_p(Zf, C.c_float), _p(pred, C.c_uint8), n, c, C.c_int64(H * W))
    return pred


def predict_from_logits(z_f32):
    """pred [n,8h,8w] from float32 low-resolution logits: float32 interpolation, argmax."""
    return argmax_f32(upsample8_f32(z_f32))


def softmax_ce(Z, labels, ignore_index=-1, want_grad=True, weights=None):
    """Returns (loss, gradient, sum of the weights of the valid pixels)."""
    Z = _f64(Z)
    n, c, H, W = Z.shape
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    G = np.empty_like(Z) if want_grad else None
    nv = C.c_int64(0)
    wts = np.ascontiguousarray(weights, dtype=np.uint8) if weights is not None else None
    loss = lib().sto_softmax_ce_w(_d(Z), _p(labels, C.c_int32), _p(wts, C.c_uint8), _d(G), n, c,
                                  C.c_int64(H * W), ignore_index, C.byref(nv))
    return float(loss), G, int(nv.value)


def confusion(pred, labels, n_classes, ignore_index=-1):
    pred = np.ascontiguousarray(pred, dtype=np.uint8).ravel()
    labels = np.ascontiguousarray(labels, dtype=np.int32).ravel()
    conf = np.empty((n_classes, n_classes), dtype=np.int64)
    lib().sto_confusion(_p(pred, C.c_uint8), _p(labels, C.c_int32), C.c_int64(pred.size),
                        n_classes, ignore_index, _p(conf, C.c_int64))
    return conf


def miou(conf):
    conf = np.ascontiguousarray(conf, dtype=np.int64)
    out = C.c_double(0.0)
    present = lib().sto_miou(_p(conf, C.c_int64), conf.shape[0], C.byref(out))
    return float(out.value), int(present)


def sgd(theta, grad, vel, lr, mu):
    theta, grad = _f64(theta).copy(), _f64(grad)
    vel = _f64(vel).copy() if vel is not None else None
    lib().sto_sgd(_d(theta), _d(grad), _d(vel), C.c_int64(theta.size), C.c_double(lr),
                  C.c_double(mu))
    return theta, vel


class Optim(C.Structure):
    """kind 0: gradient descent with optional momentum; kind 1: Adam (t0 = steps taken before)."""
    _fields_ = [("kind", C.c_int32), ("lr", C.c_double), ("mu", C.c_double), ("beta1", C.c_double),
                ("beta2", C.c_double), ("eps", C.c_double), ("t0", C.c_int64)]


def adam_optim(lr, beta1=0.9, beta2=0.999, eps=1e-8, t0=0) -> Optim:
    return Optim(1, lr, 0.0, beta1, beta2, eps, t0)


def adam(theta, grad, m, v, lr, beta1, beta2, eps, t):
    """One Adam step number t (1-based) on copies; returns (theta, m, v)."""
    theta, grad, m, v = _f64(theta).copy(), _f64(grad), _f64(m).copy(), _f64(v).copy()
    lib().sto_adam(_d(theta), _d(grad), _d(m), _d(v), C.c_int64(theta.size), C.c_double(lr),
                   C.c_double(beta1), C.c_double(beta2), C.c_double(eps), C.c_int64(t))
    return theta, m, v


# ------------------------------------------------------------------ the head
def num_params(d: Desc) -> int:
    return int(lib().sto_num_params(C.byref(d)))


def head_forward(d: Desc, features, params, want_pred=True):
    features, params = _f64(features), _f64(params)
    z = np.empty((d.n, d.n_classes, d.h, d.w))
    pred = np.empty((d.n, 8 * d.h, 8 * d.w), dtype=np.uint8) if want_pred else None
    lib().sto_head_forward(C.byref(d), _d(features), _d(params), _d(z), _p(pred, C.c_uint8))
    return z, pred


def loss_and_grad(d: Desc, features, labels, params, want_grad=True, want_metric=True):
    features, params = _f64(features), _f64(params)
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    grad = np.empty_like(params) if want_grad else None
    Cn = d.n_classes
    pred = np.empty((d.n, 8 * d.h, 8 * d.w), dtype=np.uint8) if want_metric else None
    conf = np.empty((d.n, Cn, Cn), dtype=np.int64) if want_metric else None
    mi = np.empty(d.n) if want_metric else None
    loss = lib().sto_loss_and_grad(C.byref(d), _d(features), _p(labels, C.c_int32), _d(params),
                                   _d(grad), _p(pred, C.c_uint8), _p(conf, C.c_int64), _d(mi))
    return float(loss), grad, pred, conf, mi


def feature_grad(d: Desc, features, labels, params):
    """(loss, parameter gradient, d loss / d features [n,c_in,h,w]): the full backward pass, i.e.
    what partial distillation saves plus what it keeps."""
    features, params = _f64(features), _f64(params)
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    grad = np.empty_like(params)
    df = np.empty_like(features)
    loss = lib().sto_loss_and_grad_full(C.byref(d), _d(features), _p(labels, C.c_int32), _d(params),
                                        _d(grad), _d(df), None, None, None)
    return float(loss), grad, df


def partial_distill(d: Desc, features, labels, params, steps, lr, momentum=0.0, velocity=None):
    """k fixed steps.  Returns dict(params, velocity, losses[k+1], mious[k+1,n], conf[n,C,C],
    pred[n,8h,8w])."""
    features = _f64(features)
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    params = _f64(params).copy()
    vel = (_f64(velocity).copy() if velocity is not None else np.zeros_like(params))
    losses = np.empty(steps + 1)
    mious = np.empty((steps + 1, d.n))
    conf = np.empty((d.n, d.n_classes, d.n_classes), dtype=np.int64)
    pred = np.empty((d.n, 8 * d.h, 8 * d.w), dtype=np.uint8)
    lib().sto_partial_distill(C.byref(d), _d(features), _p(labels, C.c_int32), _d(params),
                              _d(vel), steps, C.c_double(lr), C.c_double(momentum), _d(losses),
                              _d(mious), _p(conf, C.c_int64), _p(pred, C.c_uint8))
    return dict(params=params, velocity=vel, losses=losses, mious=mious, conf=conf, pred=pred)


def partial_distill_stepwise(d: Desc, features, labels, params, steps, lr, momentum=0.0, velocity=None,
                             on_step=None):
    """The loop of partial_distill written out around loss_and_grad and sgd -- the very routines
    the C loop calls, in its order -- so that a long run can report between steps
    (on_step(it, loss) after every pass).  Same dict as partial_distill; a CPU test holds the two
    bit for bit equal."""
    features = _f64(features)
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    params = _f64(params).copy()
    vel = (_f64(velocity).copy() if velocity is not None else np.zeros_like(params))
    losses = np.empty(steps + 1)
    mious = np.empty((steps + 1, d.n))
    conf = pred = None
    for it in range(steps + 1):
        last = it == steps
        loss, grad, pred, conf, mi = loss_and_grad(d, features, labels, params, want_grad=not last)
        losses[it], mious[it] = loss, mi
        if on_step is not None:
            on_step(it, loss)
        if last:
            break
        params, v2 = sgd(params, grad, vel if momentum != 0.0 else None, lr, momentum)
        if v2 is not None:
            vel = v2
    return dict(params=params, velocity=vel, losses=losses, mious=mious, conf=conf, pred=pred)


def partial_distill_opt(d: Desc, features, labels, params, steps, optim: Optim, s1=None, s2=None):
    """k fixed steps with an explicit optimiser description; s1 / s2 are its state arrays
    (velocity, or Adam's m and v), zero when absent.  Returns the same dict as partial_distill
    plus s1, s2."""
    features = _f64(features)
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    params = _f64(params).copy()
    s1 = _f64(s1).copy() if s1 is not None else np.zeros_like(params)
    s2 = _f64(s2).copy() if s2 is not None else np.zeros_like(params)
    losses = np.empty(steps + 1)
    mious = np.empty((steps + 1, d.n))
    conf = np.empty((d.n, d.n_classes, d.n_classes), dtype=np.int64)
    pred = np.empty((d.n, 8 * d.h, 8 * d.w), dtype=np.uint8)
    lib().sto_partial_distill_opt(C.byref(d), _d(features), _p(labels, C.c_int32), _d(params),
                                  C.byref(optim), _d(s1), _d(s2), steps, _d(losses), _d(mious),
                                  _p(conf, C.c_int64), _p(pred, C.c_uint8))
    return dict(params=params, s1=s1, s2=s2, losses=losses, mious=mious, conf=conf, pred=pred)


def partial_distill_grouped(d: Desc, features, labels, params, steps, optim: Optim, s1=None,
                            s2=None, pixel_weights=None):
    """n clients, each with a student head of its own and one key frame (the server of Algorithm 3
    keeps one student per client and trains it on that client's frames only).  By definition this
    is n independent runs of partial_distill_opt on one frame each; nothing is shared.
    params, s1, s2: [n, num_params]; pixel_weights: uint8 [n,8h,8w] or None.
    Returns dict(params[n,P], s1, s2, losses[k+1,n], mious[k+1,n], conf[n,C,C], pred[n,8h,8w])."""
    features = _f64(features)
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    params = _f64(params)
    n = d.n
    assert params.shape[0] == n and features.shape[0] == n and labels.shape[0] == n
    runs = []
    for f in range(n):
        d1 = desc(1, d.c_in, d.h, d.w, d.c1, d.c2, d.n_classes, d.ignore_index, bool(d.bf16_operands))
        if pixel_weights is not None:
            d1 = with_pixel_weights(d1, pixel_weights[f:f + 1])
        runs.append(partial_distill_opt(d1, features[f:f + 1], labels[f:f + 1], params[f], steps, optim,
                                        None if s1 is None else s1[f], None if s2 is None else s2[f]))
    return dict(params=np.stack([r["params"] for r in runs]),
                s1=np.stack([r["s1"] for r in runs]), s2=np.stack([r["s2"] for r in runs]),
                losses=np.stack([r["losses"] for r in runs], axis=1),
                mious=np.concatenate([r["mious"] for r in runs], axis=1),
                conf=np.concatenate([r["conf"] for r in runs], axis=0),
                pred=np.concatenate([r["pred"] for r in runs], axis=0))


def train(d: Desc, features, labels, params, max_updates, lr, threshold, momentum=0.0,
          velocity=None, strict_break=True):
    """Student training with the skip / best-tracking / early-exit rules.
    Returns dict(params=best, best_metric, updates, metrics[0..updates])."""
    features = _f64(features)
    labels = np.ascontiguousarray(labels, dtype=np.int32)
    params = _f64(params).copy()
    vel = (_f64(velocity).copy() if velocity is not None else np.zeros_like(params))
    bm = C.c_double(0.0)
    metrics = np.full(max_updates + 1, np.nan)
    upd = lib().sto_train(C.byref(d), _d(features), _p(labels, C.c_int32), _d(params), _d(vel),
                          max_updates, C.c_double(lr), C.c_double(momentum),
                          C.c_double(threshold), 1 if strict_break else 0, C.byref(bm),
                          _d(metrics))
    return dict(params=params, velocity=vel, best_metric=float(bm.value), updates=int(upd),
                metrics=metrics[:upd + 1])

"""Helpers of the GPU parity tests: run one workload through the C ABI (via the Python binding)
and through the CPU oracle on identical seeded inputs."""
from __future__ import annotations

import os
import time

import numpy as np
import torch

import oracle as O
import paper_2003_10735_amd as st
import workloads as WL


_ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def progress(msg):
    """One line per finished piece of a long test (a frame, a step): printed, and appended to a
    log file in the run's output folder, so that a run whose output is captured still shows that
    it moves."""
    line = time.strftime("%H:%M:%S ") + str(msg)
    print(line, flush=True)
    try:
        os.makedirs(os.path.join(_ROOT, "gpurun_out"), exist_ok=True)
        with open(os.path.join(_ROOT, "gpurun_out", "test_progress.log"), "a") as fh:
            fh.write(line + "\n")
    except OSError:
        pass


def golden_source_digest():
    """SHA-256 over the oracle's sources and the input generators: what a stored oracle result
    depends on (the same recipe as tests/golden/make_full_length_expectations.py)."""
    import hashlib
    h = hashlib.sha256()
    for rel in ("oracle/st_oracle.c", "oracle/__init__.py", "workloads/__init__.py"):
        with open(os.path.join(_ROOT, rel), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def load_golden(name):
    """The oracle's stored full-length result `name` (written by the committed script
    tests/golden/make_full_length_expectations.py, which calls only the oracle).  Refuses a file
    made from other oracle sources or input generators than the tree holds."""
    g = np.load(os.path.join(_ROOT, "tests", "golden", f"full_length_{name}.npz"))
    assert str(g["digest"]) == golden_source_digest(), \
        "tests/golden/full_length_%s.npz is stale: run tests/golden/make_full_length_expectations.py" % name
    return g


def live_oracle():
    """ST_LIVE_ORACLE=1: the full-length tests run the oracle themselves (minutes of CPU time)
    instead of reading its stored results."""
    return os.environ.get("ST_LIVE_ORACLE", "0") not in ("", "0")


def to_dev_features(wl, feats):
    t = torch.from_numpy(feats.view(np.int16) if feats.dtype == np.uint16 else feats).cuda()
    return t.view(torch.bfloat16) if feats.dtype == np.uint16 else t


def run_gpu(wl, feats, labels, params, steps=None, velocity=None, threshold=0.0, strict_break=True,
            return_best=False, workspace=None):
    """Returns dict with params, velocity, losses, mious, conf, pred, z (final low-res logits),
    steps_taken, best_metric; everything as numpy."""
    desc = st.HeadDesc.of(wl)
    steps = wl.steps if steps is None else steps
    f = to_dev_features(wl, feats)
    lab = torch.from_numpy(labels).cuda()
    p = torch.from_numpy(params.astype(np.float32)).cuda()
    vel = None
    if wl.momentum != 0.0:
        vel = torch.from_numpy((velocity if velocity is not None else np.zeros_like(params)).astype(np.float32)).cuda()
    losses = torch.full((steps + 1,), float("nan"), dtype=torch.float32, device="cuda")
    mious = torch.full((steps + 1, wl.n), float("nan"), dtype=torch.float64, device="cuda")
    conf = torch.zeros((wl.n, wl.n_classes, wl.n_classes), dtype=torch.int64, device="cuda")
    pred = torch.zeros((wl.n, wl.H, wl.W), dtype=torch.uint8, device="cuda")
    ws = workspace if workspace is not None else st.new_workspace(desc)
    ret = st.st_partial_distill(desc, f, lab, p, steps, wl.lr, momentum=wl.momentum, velocity=vel,
                                threshold=threshold, strict_break=strict_break,
                                return_best=return_best, losses=losses, mious=mious,
                                confusion=conf, pred=pred, workspace=ws)
    taken, best = ret
    torch.cuda.synchronize()
    lay = st.st_get_workspace_layout(desc)
    nz = wl.n * wl.n_classes * wl.h * wl.w
    z = ws[lay["z"]:lay["z"] + 4 * nz].view(torch.float32).reshape(wl.n, wl.n_classes, wl.h, wl.w)
    return dict(params=p.cpu().numpy(), velocity=None if vel is None else vel.cpu().numpy(),
                losses=losses.cpu().numpy(), mious=mious.cpu().numpy(), conf=conf.cpu().numpy(),
                pred=pred.cpu().numpy(), z=z.cpu().numpy(), steps_taken=taken, best_metric=best,
                first_metric=ret.first_metric,
                workspace=ws, layout=lay)


def run_oracle(wl, feats, labels, params, steps=None, bf16_operands=None, velocity=None, report=None):
    """`report`: a tag; the run then goes step by step and leaves a progress line per pass."""
    d = O.desc_of(wl, bf16_operands)
    steps = wl.steps if steps is None else steps
    if report:
        return O.partial_distill_stepwise(d, WL.features_as_f64(wl, feats), labels, params.astype(np.float64), steps,
                                          wl.lr, momentum=wl.momentum, velocity=velocity,
                                          on_step=lambda it, loss: progress(f"{report}: oracle pass {it} loss {loss:.6f}"))
    return O.partial_distill(d, WL.features_as_f64(wl, feats), labels, params.astype(np.float64), steps,
                             wl.lr, momentum=wl.momentum, velocity=velocity)


def rel_err(a, b):
    """max |a - b| / max |b| over a tensor (per-tensor relative error)."""
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    den = np.max(np.abs(b))
    return float(np.max(np.abs(a - b)) / (den if den > 0 else 1.0))


def update_err(tag, got, want):
    """Relative error of an update (trained minus initial parameters), logged: the parameters
    themselves are dominated by their initial values, the update is what a wrong gradient moves."""
    e = rel_err(got, want)
    progress(f"update error {tag}: {e:.3g}")
    return e


def check_staged_bit_exact(wl, gpu, labels):
    """From the GPU's own final low-resolution logits the oracle must reproduce the GPU's class
    map, confusion counts and mean IoU bit for bit."""
    pred_o = O.predict_from_logits(gpu["z"])
    np.testing.assert_array_equal(gpu["pred"], pred_o)
    for i in range(wl.n):
        conf_o = O.confusion(pred_o[i], labels[i], wl.n_classes, wl.ignore_index)
        np.testing.assert_array_equal(gpu["conf"][i], conf_o)
        assert gpu["mious"][gpu["steps_taken"], i] == O.miou(conf_o)[0]


def check_pred_against_oracle(wl, gpu, oracle_res, feats, logit_tol):
    """End to end the two class maps may differ only where the oracle's two best up-sampled
    logits are closer than the logit tolerance."""
    bad = gpu["pred"] != oracle_res["pred"]
    if not bad.any():
        return 0
    d = O.desc_of(wl)
    z, _ = O.head_forward(d, WL.features_as_f64(wl, feats), oracle_res["params"], want_pred=False)
    Z = O.upsample8(z)
    top2 = np.sort(Z, axis=1)[:, -2:]
    margin = top2[:, 1] - top2[:, 0]
    assert np.all(margin[bad] <= logit_tol), (int(bad.sum()), float(margin[bad].max()))
    return int(bad.sum())

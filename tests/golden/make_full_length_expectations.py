#!/usr/bin/env python3
"""Writes the oracle's results for the two workloads whose full-length oracle run takes minutes
of CPU time -- the batch of four frames at its sixteen steps, and the 32-frame temporal clip --
into tests/golden/full_length_*.npz, so that the GPU parity tests can hold the HIP path to them
at the configurations' own lengths without re-running the oracle every time.

Calls only `oracle/` and the seeded input generators in `workloads/`: no value written here comes
from the HIP path.  Every file records the SHA-256 of the oracle's source, of its Python
front-end and of the input generators; the tests refuse a file whose digests do not match the
tree (then run this script again: `python tests/golden/make_full_length_expectations.py`,
about half an hour on 8 cores).

Stored per run: losses and per-frame mean IoU of every pass (or, for the clip, every frame's
score, key-frame flag and update count), and the trained parameters at every SAMPLE_STRIDE-th
index plus all biases (as float32: 6e-8 relative, far below the tests' tolerances), with the
largest |parameter| and |update| of the whole vector (the tests' relative errors are taken
against those).
"""
from __future__ import annotations

import hashlib
import os
import sys
import time

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
sys.path.insert(0, ROOT)

import oracle as O          # noqa: E402
import workloads as WL      # noqa: E402

SAMPLE_STRIDE = 13          # coprime with every tile, tap and channel count of the kernels under test


def source_digest() -> str:
    h = hashlib.sha256()
    for rel in ("oracle/st_oracle.c", "oracle/__init__.py", "workloads/__init__.py"):
        with open(os.path.join(ROOT, rel), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()


def sample_index(wl) -> np.ndarray:
    """Every SAMPLE_STRIDE-th parameter, and every bias."""
    idx = set(range(0, wl.n_params, SAMPLE_STRIDE))
    for name, sl in WL.param_slices(wl).items():
        if name.startswith("b"):
            idx.update(range(sl.start, sl.stop))
    return np.array(sorted(idx), dtype=np.int64)


def say(msg):
    print(time.strftime("%H:%M:%S"), msg, flush=True)


def batch4():
    wl = WL.WORKLOADS["batch4"]
    f, lab, p = WL.make_features(wl), WL.make_labels(wl), WL.make_head_params(wl)
    idx = sample_index(wl)
    out = {"digest": np.array(source_digest()), "index": idx.astype(np.int32), "steps": np.array(wl.steps)}
    for tag, mode in (("bf16", True), ("exact", False)):
        r = O.partial_distill_stepwise(O.desc_of(wl, mode), WL.features_as_f64(wl, f), lab, p.astype(np.float64),
                                       wl.steps, wl.lr, momentum=wl.momentum,
                                       on_step=lambda it, loss: say(f"batch4 {tag} pass {it} loss {loss:.6f}"))
        out[f"{tag}_losses"] = r["losses"]
        out[f"{tag}_mious"] = r["mious"]
        out[f"{tag}_params"] = r["params"][idx].astype(np.float32)
        out[f"{tag}_max_abs_param"] = np.array(np.abs(r["params"]).max())
        out[f"{tag}_max_abs_update"] = np.array(np.abs(r["params"] - p).max())
        out[f"{tag}_conf"] = r["conf"]
    np.savez_compressed(os.path.join(HERE, "full_length_batch4.npz"), **out)


def clip():
    wl = WL.WORKLOADS["clip"]
    thr = float(wl.extra["threshold"])
    frames = list(WL.clip_frames(wl))
    p0 = WL.make_head_params(wl)
    idx = sample_index(wl)
    out = {"digest": np.array(source_digest()), "index": idx.astype(np.int32), "frames": np.array(len(frames)),
           "threshold": np.array(thr)}
    for tag, mode in (("bf16", True), ("exact", False)):
        d = O.desc_of(wl, mode)
        params = p0.astype(np.float64).copy()
        scores, key, updates, trained = [], [], [], []
        for t, (f, lab) in enumerate(frames):
            # Algorithm 1 scores the head first and trains only under the threshold ('>=' leaves the
            # loop, as the clip configuration words it); its first metric is the frame's score
            r = O.train(d, WL.features_as_f64(wl, f), lab, params, wl.steps, wl.lr, thr, momentum=wl.momentum,
                        strict_break=False)
            scores.append(r["metrics"][0]); key.append(r["metrics"][0] < thr); updates.append(r["updates"])
            trained.append(r["best_metric"])
            params = r["params"]
            say(f"clip {tag} frame {t}: score {scores[-1]:.4f} updates {updates[-1]}")
        out[f"{tag}_scores"] = np.array(scores)
        out[f"{tag}_key"] = np.array(key)
        out[f"{tag}_updates"] = np.array(updates, dtype=np.int64)
        out[f"{tag}_trained_scores"] = np.array(trained)
        out[f"{tag}_params"] = params[idx].astype(np.float32)
        out[f"{tag}_max_abs_param"] = np.array(np.abs(params).max())
        out[f"{tag}_max_abs_update"] = np.array(np.abs(params - p0).max())
    np.savez_compressed(os.path.join(HERE, "full_length_clip.npz"), **out)


if __name__ == "__main__":
    which = sys.argv[1:] or ["batch4", "clip"]
    if "batch4" in which:
        batch4()
    if "clip" in which:
        clip()

"""Clip driver: the per-frame schedule of Algorithms 3 and 4 around the head's training step.

Every frame the head runs forward and is scored against the teacher's label map (mean IoU,
Eq. 1).  A frame whose score falls below THRESHOLD is a key frame: the head is trained on it
with Algorithm 1 (at most MAX_UPDATES optimiser steps, leaving as soon as the score reaches the
threshold) and the updated head serves the following frames.  `run_clip` does both with one
st_partial_distill call per frame (Algorithm 1 scores first and trains only under the
threshold); `run_clip_strided` keeps the client's head apart from the server's and scores it with
st_head_forward + st_miou.  Only argument marshalling and the
loop live here; every computation is a call into the HIP library.
"""
from __future__ import annotations

import time

from . import (HeadDesc, new_workspace, st_head_forward, st_miou, st_partial_distill)


def run_clip(desc: HeadDesc, frames, head_params, *, threshold: float, max_updates: int, lr: float,
             momentum: float = 0.0, strict_break: bool = False, return_best: bool = True,
             workspace=None, stream=None, expect_key_frames: bool = False) -> dict:
    """`frames` yields (features, teacher_labels) pairs of cuda tensors ([n,c_in,h,w] bfloat16 or
    float32; [n,8h,8w] int32).  `head_params` (float32 cuda tensor) is updated in place on key
    frames.  Returns per-frame scores before training, which frames were key frames, the
    optimiser steps each took, the score the training call reported, and the frame rate."""
    import torch

    ws = workspace if workspace is not None else new_workspace(desc, head_params.device)
    velocity = torch.zeros_like(head_params) if momentum != 0.0 else None
    scores, key, updates, trained, frame_ms = [], [], [], [], []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    n_frames = 0
    for features, labels in frames:
        # One call per frame is Algorithm 1 as printed: it scores the head on the frame first
        # (forward + mean IoU) and trains only if that score is under the threshold (the schedule
        # is decided on the host, inside the call, on the metric it reads back).  A frame that is
        # no key frame costs that forward pass and nothing else; the call has finished on return.
        tf = time.perf_counter()
        r = st_partial_distill(desc, features, labels, head_params, max_updates, lr,
                               momentum=momentum, velocity=velocity, threshold=threshold,
                               strict_break=strict_break, return_best=return_best,
                               workspace=ws, stream=stream, expect_key_frame=expect_key_frames)
        frame_ms.append((time.perf_counter() - tf) * 1e3)
        taken, best = r
        score = r.first_metric
        scores.append(score)
        is_key = score < threshold
        key.append(is_key)
        updates.append(taken if is_key else 0)
        trained.append(best if is_key else None)
        n_frames += 1
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    return dict(scores=scores, key_frames=key, updates=updates, trained_scores=trained, frame_ms=frame_ms,
                frames_per_s=n_frames / dt if dt > 0 else float("nan"), n_key_frames=sum(key))


def run_clip_strided(desc: HeadDesc, frames, head_params, *, threshold: float, max_updates: int, lr: float,
                     min_stride: float, max_stride: float, delay: int = 1, momentum: float = 0.0,
                     strict_break: bool = True, workspace=None, stream=None) -> dict:
    """The client / server schedule of Algorithms 3 and 4 in one process.

    The first frame is a key frame; afterwards a frame is a key frame once `stride` frames have
    passed since the last one (the stride can be fractional after Algorithm 2: the test
    "step = stride" is taken as step >= stride).  On a key frame the server's copy of the head is
    trained (Algorithm 1, best parameters returned) and the result reaches the client `delay`
    frames later (1 <= delay <= MIN_STRIDE: the client waits for it at the latest then); until
    then the client keeps predicting with the head it has.  When the update is applied the
    stride is recomputed from the metric the training reported (Algorithm 2).

    `head_params` is the client's head (updated in place when updates arrive).  Returns the
    client's per-frame scores, the key-frame flags, the steps taken on each key frame, the
    stride after each frame and the frame rate."""
    import torch

    from . import st_next_stride

    if not (1 <= delay <= min_stride):
        raise ValueError("delay must lie in [1, MIN_STRIDE]")
    ws = workspace if workspace is not None else new_workspace(desc, head_params.device)
    server = head_params.clone()
    velocity = torch.zeros_like(head_params) if momentum != 0.0 else None
    pred = None
    conf = torch.empty((desc.n_classes, desc.n_classes), dtype=torch.int64, device=head_params.device)
    miou = torch.empty(1, dtype=torch.float64, device=head_params.device)
    stride, step, updated = float(min_stride), float(min_stride), True
    pending_metric = None
    scores, key, updates, strides = [], [], [], []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    n_frames = 0
    for features, labels in frames:
        is_key = step >= stride
        if is_key:
            taken, best = st_partial_distill(desc, features, labels, server, max_updates, lr,
                                             momentum=momentum, velocity=velocity, threshold=threshold,
                                             strict_break=strict_break, return_best=True,
                                             workspace=ws, stream=stream)
            pending_metric = best
            step, updated = 0.0, False
            updates.append(taken)
        else:
            updates.append(0)
        key.append(is_key)
        if pred is None:
            pred = torch.empty(labels.shape, dtype=torch.uint8, device=labels.device)
        st_head_forward(desc, features, head_params, pred=pred, workspace=ws, stream=stream)
        st_miou(pred, labels, desc.n_classes, desc.ignore_index, confusion=conf, miou=miou, stream=stream)
        scores.append(float(miou.item()))
        step += 1.0
        if not updated and step >= delay:
            head_params.copy_(server)
            stride = st_next_stride(stride, pending_metric, threshold, min_stride, max_stride)
            updated = True
        strides.append(stride)
        n_frames += 1
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    return dict(scores=scores, key_frames=key, updates=updates, strides=strides,
                frames_per_s=n_frames / dt if dt > 0 else float("nan"), n_key_frames=sum(key))

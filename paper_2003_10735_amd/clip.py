"""Clip driver: the per-frame schedule of Algorithms 3 and 4 around the head's training step.

Every frame the head runs forward and is scored against the teacher's label map (mean IoU,
Eq. 1).  A frame whose score falls below THRESHOLD is a key frame: the head is trained on it
with Algorithm 1 (at most MAX_UPDATES optimiser steps, leaving as soon as the score reaches the
threshold) and the updated head serves the following frames.  Only argument marshalling and the
loop live here; every computation is a call into the HIP library.
"""
from __future__ import annotations

import time

from . import (HeadDesc, new_workspace, st_head_forward, st_miou, st_partial_distill)


def run_clip(desc: HeadDesc, frames, head_params, *, threshold: float, max_updates: int, lr: float,
             momentum: float = 0.0, strict_break: bool = False, return_best: bool = True,
             workspace=None, stream=None) -> dict:
    """`frames` yields (features, teacher_labels) pairs of cuda tensors ([n,c_in,h,w] bfloat16 or
    float32; [n,8h,8w] int32).  `head_params` (float32 cuda tensor) is updated in place on key
    frames.  Returns per-frame scores before training, which frames were key frames, the
    optimiser steps each took, the score the training call reported, and the frame rate."""
    import torch

    ws = workspace if workspace is not None else new_workspace(desc, head_params.device)
    velocity = torch.zeros_like(head_params) if momentum != 0.0 else None
    pred = None
    conf = torch.empty((desc.n_classes, desc.n_classes), dtype=torch.int64, device=head_params.device)
    miou = torch.empty(1, dtype=torch.float64, device=head_params.device)
    scores, key, updates, trained = [], [], [], []
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    n_frames = 0
    for features, labels in frames:
        if pred is None:
            pred = torch.empty(labels.shape, dtype=torch.uint8, device=labels.device)
        st_head_forward(desc, features, head_params, pred=pred, workspace=ws, stream=stream)
        st_miou(pred, labels, desc.n_classes, desc.ignore_index, confusion=conf, miou=miou, stream=stream)
        score = float(miou.item())          # the schedule is decided on the host
        scores.append(score)
        is_key = score < threshold
        key.append(is_key)
        if is_key:
            taken, best = st_partial_distill(desc, features, labels, head_params, max_updates, lr,
                                             momentum=momentum, velocity=velocity, threshold=threshold,
                                             strict_break=strict_break, return_best=return_best,
                                             workspace=ws, stream=stream)
            updates.append(taken)
            trained.append(best)
        else:
            updates.append(0)
            trained.append(None)
        n_frames += 1
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    return dict(scores=scores, key_frames=key, updates=updates, trained_scores=trained,
                frames_per_s=n_frames / dt if dt > 0 else float("nan"), n_key_frames=sum(key))

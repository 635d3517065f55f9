#!/usr/bin/env python3
"""Benchmark of the partial-distillation hot path on one MI355X.

One bench "step" is one st_partial_distill call on the 1280x720 key-frame workload: feature
packing, 8 optimiser steps (9 forwards, 8 partial backwards, 8 updates) and 9 loss/metric
passes, with all inputs already resident in HBM.  `value` is optimiser steps per second.

Protocol: W warm-up calls; then K = --steps calls between device synchronisations (host clock,
`wall`), every call between a pair of HIP events on the calling stream, continued until at least
--min-timed (30) calls are timed.  `ms_per_step` is the median per-call time between the events
(`ms_per_call` gives min / p90 / max), `value` = optimiser steps per call over it.  The head's
re-initialisation (one device copy) runs between the calls, outside the event pairs (inside the
host-clock region).

Prints ONE JSON line.  Extra objects:
  roofline      the kernel with the longest launches (kernels within 10 % of it count as tied and the
                tie goes to the matrix-core kernel), its algorithmic work per
                launch over its average launch duration (HIP events on the launch stream, taken
                during the timed region), against the chip's published peak; the other kernels
                of a step follow in `other_kernels`
  configs       the 1920x1080 key frame and the batch of four frames, same protocol
  clip, clip_learnable   the temporal-clip schedule: frames per second, key-frame count, time of a
                key frame and of a frame that is none
  paper_recipe  the same key frame trained as in the paper's experiments (Section 5.2): Adam on the
                loss weighted x5 near objects, the weight map made inside the timed call
  weights_pass, miou_pass, head_forward   the stand-alone entry points beside the training call
  cpu_baseline  the CPU oracle (test infrastructure, untuned) on the host cores of the machine
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_TFLOPS_BF16 = 2500.0   # MI355X dense bf16 MFMA
PEAK_TFLOPS_F32 = 157.3     # MI355X fp32 vector / matrix
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E

# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (the passes and their
# copy-kernel scale factors are recorded under profiles/).  A figure holds only for the workload and
# the kernel source it was measured on:
# (workload, kernel) -> (source file, sha256 of that file at measurement, fetched MiB, written MiB)
MEASURED_TRAFFIC = {
    ("720p", "conv12_wgrad_mfma"): ("k_wgrad_mfma.hip", "3f1113211612b411a441d3e271631c0d813b618f43bc6021537d53e99dc1f2bd", 33.76, 8.83),
    ("720p", "conv1_fwd_mfma"): ("k_conv_mfma.hip", "4fcaaea68e64f5ed6fbf36846280e453fa4afd196b9118763448bf90be1356f7", 13.75, 7.55),
    ("720p", "conv2_fwd_logits_mfma"): ("k_conv_mfma.hip", "4fcaaea68e64f5ed6fbf36846280e453fa4afd196b9118763448bf90be1356f7", 6.99, 6.13),
    ("720p", "conv2_dgrad_mfma"): ("k_conv_mfma.hip", "4fcaaea68e64f5ed6fbf36846280e453fa4afd196b9118763448bf90be1356f7", 10.45, 3.77),
    ("720p", "upsample_ce_grad"): ("k_loss.hip", "424dc624335d093c3f6a4e8de9fe08d0b1e2d3f6305e078e10999d0c9a77d705", 4.73, 4.71),
    ("720p", "upsample_ce"): ("k_loss.hip", "424dc624335d093c3f6a4e8de9fe08d0b1e2d3f6305e078e10999d0c9a77d705", 3.09, 1.79),
    ("720p", "conv3_bwd_mfma"): ("k_conv3_mfma.hip", "d34a21526a2abea318af286f76d053408f182efe714831ab42011bb3a90ac2a3", 13.22, 9.81),
    ("1080p", "conv12_wgrad_mfma"): ("k_wgrad_mfma.hip", "3f1113211612b411a441d3e271631c0d813b618f43bc6021537d53e99dc1f2bd", 73.85, 8.83),
    ("1080p", "conv1_fwd_mfma"): ("k_conv_mfma.hip", "4fcaaea68e64f5ed6fbf36846280e453fa4afd196b9118763448bf90be1356f7", 23.48, 16.59),
    ("1080p", "conv2_fwd_logits_mfma"): ("k_conv_mfma.hip", "4fcaaea68e64f5ed6fbf36846280e453fa4afd196b9118763448bf90be1356f7", 11.83, 13.48),
    ("1080p", "conv2_dgrad_mfma"): ("k_conv_mfma.hip", "4fcaaea68e64f5ed6fbf36846280e453fa4afd196b9118763448bf90be1356f7", 19.69, 8.29),
    ("1080p", "upsample_ce_grad"): ("k_loss.hip", "424dc624335d093c3f6a4e8de9fe08d0b1e2d3f6305e078e10999d0c9a77d705", 10.07, 11.14),
    ("1080p", "upsample_ce"): ("k_loss.hip", "424dc624335d093c3f6a4e8de9fe08d0b1e2d3f6305e078e10999d0c9a77d705", 6.48, 4.02),
    ("1080p", "conv3_bwd_mfma"): ("k_conv3_mfma.hip", "d34a21526a2abea318af286f76d053408f182efe714831ab42011bb3a90ac2a3", 27.57, 21.56),
    ("batch4", "conv12_wgrad_mfma"): ("k_wgrad_mfma.hip", "3f1113211612b411a441d3e271631c0d813b618f43bc6021537d53e99dc1f2bd", 268.59, 17.78),
    ("batch4", "conv1_fwd_mfma"): ("k_conv_mfma.hip", "4fcaaea68e64f5ed6fbf36846280e453fa4afd196b9118763448bf90be1356f7", 51.96, 60.38),
    ("batch4", "conv2_fwd_logits_mfma"): ("k_conv_mfma.hip", "4fcaaea68e64f5ed6fbf36846280e453fa4afd196b9118763448bf90be1356f7", 40.96, 52.83),
    ("batch4", "conv2_dgrad_mfma"): ("k_conv_mfma.hip", "4fcaaea68e64f5ed6fbf36846280e453fa4afd196b9118763448bf90be1356f7", 68.98, 30.19),
    ("batch4", "upsample_ce_grad"): ("k_loss.hip", "424dc624335d093c3f6a4e8de9fe08d0b1e2d3f6305e078e10999d0c9a77d705", 30.14, 22.21),
    ("batch4", "upsample_ce"): ("k_loss.hip", "424dc624335d093c3f6a4e8de9fe08d0b1e2d3f6305e078e10999d0c9a77d705", 23.46, 7.61),
    ("batch4", "conv3_bwd_mfma"): ("k_conv3_mfma.hip", "d34a21526a2abea318af286f76d053408f182efe714831ab42011bb3a90ac2a3", 71.54, 80.27),
}


def measured_traffic(kernel, workload):
    """HBM bytes per launch of `kernel` on `workload`, or None when there is no measurement for
    the kernel source as it stands."""
    import hashlib
    entry = MEASURED_TRAFFIC.get((workload, kernel))
    if entry is None:
        return None
    src, digest, fetch_mib, write_mib = entry
    path = os.path.join(ROOT, "paper_2003_10735_amd", "csrc", src)
    try:
        with open(path, "rb") as fh:
            if hashlib.sha256(fh.read()).hexdigest() != digest:
                return None
    except OSError:
        return None
    return round((fetch_mib + write_mib) * 1048576.0)


def kernel_work(wl):
    """Algorithmic work per launch of each kernel family: name prefix -> (bound, amount, unit).
    Convolutions count 2 * M * N * K flops of the contraction the layer defines; streaming
    kernels count the bytes the method must move; the fused up-sampling + cross-entropy kernel
    is arithmetic-bound on the vector ALUs and counts, per frame pixel and class, the float32
    operations of the definition: bilinear interpolation (3 fma = 6), running maximum (1),
    exp(z - max) (2), sum (1) -- 10 for the loss alone -- plus, with the gradient, the
    normalisation (1) and the adjoint of the interpolation (4 fma = 8): 19."""
    M = wl.n * wl.h * wl.w
    C = wl.n_classes
    P = wl.n * wl.H * wl.W
    conv1 = 2.0 * M * wl.c1 * 9 * wl.c_in
    conv2 = 2.0 * M * wl.c2 * 9 * wl.c1
    conv3 = 2.0 * M * C * wl.c2
    return {
        "conv1_fwd": ("mfma", conv1), "conv12_wgrad": ("mfma", conv1 + conv2),
        "conv2_fwd": ("mfma", conv2 + conv3), "conv2_dgrad": ("mfma", conv2), "conv1_dgrad": ("mfma", conv1),
        "conv3_fwd": ("mfma", conv3), "conv3_wgrad": ("mfma", conv3), "conv3_dgrad": ("mfma", conv3),
        # the 1x1 classifier's backward is a skinny contraction (N = classes): a2 read,
        # d loss / d z read, da2 written twice (both layouts)
        "conv3_bwd": ("hbm", (6.0 * wl.c2 + 4.0 * C) * M),
        "upsample_ce_grad": ("alu", 19.0 * C * P),
        "upsample_ce": ("alu", 10.0 * C * P),
        "sgd_update": ("hbm", (22.0 if wl.momentum else 14.0) * wl.n_params),
        "adam_update": ("hbm", 30.0 * wl.n_params),
        # the launch that opens a call: features in and out (twice on the matrix-core path: both
        # layouts), labels in, U^T of the labels out, parameters in and out
        "pack+label_adjoint": ("hbm", (3.0 if wl.compute == "bf16" else 2.0) * wl.n * wl.c_in * wl.h * wl.w * (2 if wl.feat_dtype == "bf16" else 4)
                               + 4.0 * P + 4.0 * C * M + 10.0 * wl.n_params),
    }


def call_flops(wl):
    M = wl.n * wl.h * wl.w
    conv1 = 2.0 * M * wl.c1 * 9 * wl.c_in
    conv2 = 2.0 * M * wl.c2 * 9 * wl.c1
    conv3 = 2.0 * M * wl.n_classes * wl.c2
    fwd = conv1 + conv2 + conv3
    bwd = conv1 + 2 * conv2 + 2 * conv3     # no data-gradient for layer 1: the features are frozen
    return (wl.steps + 1) * fwd + wl.steps * bwd


def step_bytes(wl):
    """Algorithmic bytes of one optimiser step (one forward, one partial backward, one update) when
    every tensor is moved once per use: bf16 (or the compute type's) activations and operand
    weights, float32 logits, gradients and parameters, int32 labels."""
    e = 2.0 if wl.compute == "bf16" else 4.0
    M, P, C = wl.n * wl.h * wl.w, wl.n * wl.H * wl.W, wl.n_classes
    feat, a1, a2 = e * M * wl.c_in, e * M * wl.c1, e * M * wl.c2
    w1, w2 = 9.0 * wl.c1 * wl.c_in, 9.0 * wl.c2 * wl.c1
    z = 4.0 * M * C
    fwd = (feat + e * w1 + a1) + (a1 + e * w2 + a2) + (a2 + z)
    loss = 2 * z + 4.0 * P
    bwd = (a2 + z + a2) + (a2 + a1 + 4 * w2) + (a2 + e * w2 + a1) + (feat + a1 + 4 * w1)
    upd = (22.0 if wl.momentum else 14.0) * wl.n_params
    return fwd + loss + bwd + upd


def upload(feats):
    import numpy as np
    import torch
    if feats.dtype == np.uint16:
        return torch.from_numpy(feats.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(feats).cuda()


class Problem:
    """One workload's inputs, head and result buffers resident on the GPU, and the call on them."""

    def __init__(self, st, WL, wl, stream, optimizer="sgd", weighted=False, full_backward=False):
        import numpy as np
        import torch
        self.st, self.wl, self.stream = st, wl, stream
        self.desc = st.HeadDesc.of(wl)
        self.feats, self.labels, self.params0 = WL.make_features(wl), WL.make_labels(wl), WL.make_head_params(wl)
        self.f, self.lab = upload(self.feats), torch.from_numpy(self.labels).cuda()
        self.p0 = torch.from_numpy(self.params0).cuda()
        self.p = self.p0.clone()
        self.vel = torch.zeros_like(self.p) if wl.momentum else None
        self.losses = torch.zeros(wl.steps + 1, dtype=torch.float32, device="cuda")
        self.mious = torch.zeros((wl.steps + 1, wl.n), dtype=torch.float64, device="cuda")
        self.conf = torch.zeros((wl.n, wl.n_classes, wl.n_classes), dtype=torch.int64, device="cuda")
        self.ws = st.new_workspace(self.desc)
        # loss weights of Section 5.2, made on the device from the labels (5 within 4 pixels of an object)
        self.pw = st.st_object_weights(self.lab, wl.n_classes, 4, ignore_index=wl.ignore_index) if weighted else None
        self.dfeat = torch.empty((wl.n, wl.c_in, wl.h, wl.w), dtype=torch.float32, device="cuda") if full_backward else None
        self.adam = dict(m=torch.zeros_like(self.p), v=torch.zeros_like(self.p), t0=0) if optimizer == "adam" else None
        torch.cuda.synchronize()

    def reset(self):
        """The head (and the optimiser state) as before the key frame."""
        self.p.copy_(self.p0)
        if self.vel is not None:
            self.vel.zero_()
        if self.adam is not None:
            self.adam["m"].zero_()
            self.adam["v"].zero_()

    def call(self, graph=False):
        """One key frame: the head is re-initialised, then one st_partial_distill call."""
        self.reset()
        self.run(graph)

    def run(self, graph=False):
        wl, st = self.wl, self.st
        if self.adam is not None:
            st.st_partial_distill(self.desc, self.f, self.lab, self.p, wl.steps, wl.lr, adam=self.adam, losses=self.losses,
                                  mious=self.mious, confusion=self.conf, workspace=self.ws, stream=self.stream,
                                  pixel_weights=self.pw, feature_grad=self.dfeat, graph=graph)
            return
        st.st_partial_distill(self.desc, self.f, self.lab, self.p, wl.steps, wl.lr, momentum=wl.momentum, velocity=self.vel,
                              losses=self.losses, mious=self.mious, confusion=self.conf, workspace=self.ws,
                              stream=self.stream, pixel_weights=self.pw, feature_grad=self.dfeat, graph=graph)


def timed_calls(fn, n_wall, n_total, before=None):
    """Runs fn() n_total times back to back on torch's current stream with a HIP event before and
    after every call; `before()` (re-initialising the head) runs ahead of each call, outside its
    event pair.  The first n_wall calls, their `before()` included, are also bracketed by a device
    synchronisation on both sides and timed with the host clock.  Returns (wall seconds of the
    first n_wall calls, list of n_total per-call milliseconds between the events)."""
    import torch
    e0 = [torch.cuda.Event(enable_timing=True) for _ in range(n_total)]
    e1 = [torch.cuda.Event(enable_timing=True) for _ in range(n_total)]

    def one(i):
        if before is not None:
            before()
        e0[i].record()
        fn()
        e1[i].record()

    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(n_wall):
        one(i)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    for i in range(n_wall, n_total):
        one(i)
    torch.cuda.synchronize()
    return wall, [e0[i].elapsed_time(e1[i]) for i in range(n_total)]


def spread(ms):
    import numpy as np
    a = np.sort(np.asarray(ms, dtype=np.float64))
    return {"median": round(float(np.median(a)), 4), "min": round(float(a[0]), 4),
            "p90": round(float(a[min(len(a) - 1, int(np.ceil(0.9 * len(a))) - 1)]), 4), "max": round(float(a[-1]), 4),
            "n_timed": int(len(a))}


def roofline_of(wl, work, name, launches, total_ms):
    pre = max((k for k in work if name.startswith(k)), key=len)
    bound, amount = work[pre]
    avg_s = total_ms / launches * 1e-3
    if bound == "mfma":
        peak = PEAK_TFLOPS_BF16 if wl.compute == "bf16" else PEAK_TFLOPS_F32
        achieved, unit = amount / avg_s / 1e12, "TFLOP/s"
    elif bound == "alu":
        peak, achieved, unit = PEAK_TFLOPS_F32, amount / avg_s / 1e12, "TFLOP/s"
    else:
        peak, achieved, unit = PEAK_HBM_GBS, amount / avg_s / 1e9, "GB/s"
    return {"bound": bound, "kernel": name, "achieved": round(achieved, 3), "peak": peak,
            "unit": unit, "frac": round(achieved / peak, 5), "traffic": measured_traffic(name, wl.name),
            "avg_launch_us": round(avg_s * 1e6, 2), "launches": launches,
            "work_per_launch": amount}


def all_kernel_pass(st, prob, calls):
    """`calls` untimed calls launched kernel by kernel with an event pair attached to every
    dispatch: name -> (launches, total ms)."""
    import torch
    st.st_profile_reset()
    st.st_profile_filter(None)
    st.st_profile_enable(True)
    for _ in range(calls):
        prob.call()
    torch.cuda.synchronize()
    prof = st.st_profile_read()
    st.st_profile_enable(False)
    st.st_profile_reset()
    return prof


def pick_dominant(work, known):
    """The kernel with the largest share of a call's GPU time (`known`: name -> (launches, total
    ms); a kernel that runs once per call, like the one that opens it, does not win on the length
    of its single launch).  Kernels within 10 % of the largest share count as tied and a tie goes
    to the matrix-core kernel, so that the choice does not flip from box to box: single kernels
    vary by +-5 % between boxes (both candidates are reported either way, one in `roofline` and
    the others in `other_kernels`)."""
    total = {k: v[1] for k, v in known.items()}
    top = max(total.values())
    tied = [k for k in total if total[k] >= 0.90 * top]
    return max(tied, key=lambda k: (work[max((q for q in work if k.startswith(q)), key=len)][0] == "mfma", total[k]))


def config_leg(st, WL, name, stream, n_timed, use_graph):
    """Another measured configuration beside the headline: per-call time (median of n_timed calls
    between HIP events, cached launch graph), convolution TFLOP/s of the whole call against the
    MFMA peak, and the kernel with the largest share of the call against its own roof."""
    import torch
    wl = WL.WORKLOADS[name]
    prob = Problem(st, WL, wl, stream)
    prob.call()
    if use_graph:
        prob.call(graph=True)
    torch.cuda.synchronize()
    work = kernel_work(wl)
    prof = all_kernel_pass(st, prob, 2)
    known = {k: v for k, v in prof.items() if any(k.startswith(pre) for pre in work)}
    dominant = pick_dominant(work, known)
    _, ms = timed_calls(lambda: prob.run(graph=use_graph), 0, n_timed, before=prob.reset)
    sp = spread(ms)
    t_call = sp["median"] * 1e-3
    peak = PEAK_TFLOPS_BF16 if wl.compute == "bf16" else PEAK_TFLOPS_F32
    tflops = call_flops(wl) / t_call / 1e12
    gbs = step_bytes(wl) * wl.steps / t_call / 1e9
    out = {"workload": f"{wl.name}: features [{wl.n},{wl.c_in},{wl.h},{wl.w}] {wl.feat_dtype}, head "
                       f"{wl.c_in}->{wl.c1}->{wl.c2}->{wl.n_classes}, x8 to {wl.H}x{wl.W}, {wl.steps} SGD steps, "
                       f"momentum {wl.momentum}, lr {wl.lr}",
           "value": round(wl.steps / t_call, 2), "unit": "steps/s", "ms_per_call": sp, "us_per_optimiser_step":
           round(t_call / wl.steps * 1e6, 2), "conv_tflops": round(tflops, 2), "mfma_frac": round(tflops / peak, 5),
           "algorithmic_GBs": round(gbs, 1), "hbm_frac": round(gbs / PEAK_HBM_GBS, 5),
           "dominant_kernel": roofline_of(wl, work, dominant, *known[dominant]),
           "kernel_us": {k: round(v[1] / v[0] * 1e3, 2) for k, v in sorted(prof.items(), key=lambda kv: -kv[1][1])},
           "loss_first_last": [float(prob.losses[0]), float(prob.losses[-1])]}
    del prob
    torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="720p")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--min-timed", type=int, default=30,
                    help="per-call statistics (median, min, p90) are taken over at least this many timed calls, "
                         "whatever --steps says")
    ap.add_argument("--full-backward", action="store_true",
                    help="also compute d loss / d features in every backward pass (the data-gradient of "
                         "layer 1 that partial distillation leaves out): the step an unfrozen front part would "
                         "build on, for the partial-vs-full comparison; default: partial, the headline")
    ap.add_argument("--weighted-loss", action="store_true",
                    help="scale the loss of pixels within 4 px of a non-background (class 0) label by 5 "
                         "(Section 5.2 of the paper); default: unweighted, the headline configuration")
    ap.add_argument("--optimizer", choices=("sgd", "adam"), default="sgd",
                    help="sgd: the workload's optimiser (the headline configuration); adam: the "
                         "paper's optimiser (Section 5.2) with beta 0.9 / 0.999, eps 1e-8, state reset per key frame")
    ap.add_argument("--clients", type=int, default=4,
                    help="also time the grouped form: this many clients, each with a head and a key frame of "
                         "its own, trained in one call (reported beside the headline as `grouped`; 0 = skip)")
    ap.add_argument("--streams", type=int, default=3,
                    help="also time this many independent clients, each with its own key frame, head and "
                         "workspace, whose calls are issued round-robin on streams of their own (the GPU "
                         "then fills one client's launch gaps with another client's kernels); reported "
                         "beside the headline as `streams`; 0 = skip")
    ap.add_argument("--clip-frames", type=int, default=32,
                    help="also run the temporal-clip schedule on this many 720p frames (every frame: head "
                         "forward + mean IoU; a frame below the threshold is a key frame and is trained "
                         "with the early-exit form of Algorithm 1), once on the configuration's noise features "
                         "(`clip`: every frame is a key frame) and once on features that carry the labels "
                         "(`clip_learnable`: most frames are not key frames, as in the paper's videos); 0 = skip")
    ap.add_argument("--other-configs", default="1080p,batch4",
                    help="comma-separated workloads measured beside the headline (`configs` in the line); "
                         "empty = skip")
    ap.add_argument("--no-full-compare", action="store_true",
                    help="skip the partial-against-full comparison leg (`partial_vs_full`)")
    ap.add_argument("--no-graph", action="store_true",
                    help="time the calls launched kernel by kernel in the stream; default: `value` is timed "
                         "with the library's cached HIP graph (st_distill_opts.use_graph), and the "
                         "kernel-by-kernel rate is reported beside it as `stream_launch`")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="also run one plain device-to-device copy of this many MiB (outside the timed "
                         "region): the known-size reference that scales hardware byte counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: the library runs on one GPU; sharding is by video stream (one head per "
              "client per GPU, no exchange) and is not part of it. Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2003_10735_amd as st
    import workloads as WL

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    st.lib()   # fails loudly when the HIP library has not been built
    torch.cuda.set_device(0)
    wl = WL.WORKLOADS[args.workload]
    # a stream of the caller's own (the library records its launch graph on it; the NULL stream
    # cannot be captured), made torch's current stream so that every copy and event below is on it
    stream = torch.cuda.Stream()
    torch.cuda.synchronize()
    torch.cuda.set_stream(stream)
    use_adam = args.optimizer == "adam"
    variant = use_adam or args.weighted_loss or args.full_backward
    prob = Problem(st, WL, wl, stream, args.optimizer, args.weighted_loss, args.full_backward)
    desc, f, lab, p, ws = prob.desc, prob.f, prob.lab, prob.p, prob.ws
    one_call = prob.call

    use_graph = not args.no_graph
    graph_note = None
    for _ in range(max(args.warmup, 1)):
        one_call()
        if use_graph:
            try:
                one_call(graph=True)
                torch.cuda.synchronize()
            except (st.StError, RuntimeError) as exc:      # no graph on this system: time the plain launches
                use_graph = False
                graph_note = f"graph launch unavailable ({exc}); "
    torch.cuda.synchronize()
    if args.copy_probe_mib > 0:
        src = torch.ones(args.copy_probe_mib * 262144, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # which kernel dominates: three untimed calls with an event pair around every launch
    prof = all_kernel_pass(st, prob, 3)
    work = kernel_work(wl)
    known = {k: v for k, v in prof.items() if any(k.startswith(pre) for pre in work)}
    dominant = pick_dominant(work, known)
    breakdown = {k: round(v[1] / v[0] * 1e3, 2) for k, v in sorted(prof.items(), key=lambda kv: -kv[1][1])}

    # timed region, kernel-by-kernel launches, no events inside the calls
    wall_plain, ms_plain = timed_calls(prob.run, args.steps, args.steps, before=prob.reset)
    sp_plain = spread(ms_plain)
    stream_launch = {"value": round(wl.steps / (sp_plain["median"] * 1e-3), 2), "unit": "steps/s",
                     "ms_per_step": sp_plain["median"], "ms_per_call": sp_plain,
                     "note": "the same K calls launched kernel by kernel in the stream"}
    # the same timed region once more with an event pair attached to every dispatch: the roofline
    # object's duration.  (With a pair on the dominant kernel alone its start stamp is taken while
    # the kernel in front of it -- which then has no completion signal of its own -- still drains,
    # and the figure reads about 1.7 us long against the profiler's; with a pair on every dispatch
    # the two agree.)
    st.st_profile_reset()
    st.st_profile_filter(None)
    st.st_profile_enable(True)
    _, ms_events = timed_calls(prob.run, args.steps, args.steps, before=prob.reset)
    prof_timed = st.st_profile_read()
    dom = prof_timed[dominant]
    st.st_profile_enable(False)
    st.st_profile_reset()
    stream_launch["with_event_pairs"] = {"ms_per_call": spread(ms_events),
                                         "note": "the K calls the roofline object's event pairs come from "
                                                 "(a pair on every dispatch)"}
    # The headline: K calls (through the library's cached launch graph unless --no-graph) bracketed by
    # a device synchronisation on both sides for the host clock, every call between a pair of HIP
    # events on the calling stream; more calls follow until there are at least --min-timed of them.
    # `value` comes from the median per-call time between the events; the host-clock figure of
    # the K-call region stands beside it.  The head's re-initialisation (one 1.8 MB device copy)
    # runs between the calls: outside the event pairs, inside the host-clock region.
    n_total = max(args.steps, args.min_timed)
    if use_graph:
        wall, ms_calls = timed_calls(lambda: prob.run(graph=True), args.steps, n_total, before=prob.reset)
    elif n_total > args.steps:
        wall, ms_calls = timed_calls(prob.run, args.steps, n_total, before=prob.reset)
    else:
        wall, ms_calls = wall_plain, ms_plain
    sp = spread(ms_calls)
    t_call = sp["median"] * 1e-3
    ms_per_call = sp["median"]
    steps_per_s = wl.steps / t_call
    final_losses = prob.losses.cpu().numpy()

    roofline = roofline_of(wl, work, dominant, dom[0], dom[1])
    # the other kernels of a step, from the all-kernel pass (every launch carried an event pair)
    others = {k: {kk: vv for kk, vv in roofline_of(wl, work, k, v[0], v[1]).items()
                  if kk in ("bound", "achieved", "unit", "frac", "avg_launch_us", "traffic")}
              for k, v in known.items() if k != dominant}
    # the fused up-sampling + cross-entropy kernel against the other roof as well: as a streaming
    # kernel it would move 4 C bytes of logits in and 4 C bytes of gradient out per low-resolution
    # cell and 4 bytes of label per frame pixel
    for k in others:
        if k.startswith("upsample_ce"):
            cells, pixels = wl.n * wl.h * wl.w, wl.n * wl.H * wl.W
            stream_bytes = (8.0 if k.startswith("upsample_ce_grad") else 4.0) * wl.n_classes * cells + 4.0 * pixels
            gbs = stream_bytes / (others[k]["avg_launch_us"] * 1e-6) / 1e9
            others[k]["hbm_achieved_GBs"] = round(gbs, 1)
            others[k]["hbm_frac"] = round(gbs / PEAK_HBM_GBS, 5)
            others[k]["binding_roof"] = "alu" if others[k]["frac"] >= others[k]["hbm_frac"] else "hbm"

    # the stand-alone metric call (st_miou: confusion histogram + mean IoU of a class map);
    # streaming bound: 1 B prediction + 4 B label per pixel
    pred = torch.zeros((wl.n, wl.H, wl.W), dtype=torch.uint8, device="cuda")
    st.st_head_forward(desc, f, p, pred=pred, workspace=ws, stream=stream)
    conf1 = torch.empty((wl.n_classes, wl.n_classes), dtype=torch.int64, device="cuda")
    m1 = torch.empty(1, dtype=torch.float64, device="cuda")
    for _ in range(3):
        st.st_miou(pred, lab, wl.n_classes, wl.ignore_index, confusion=conf1, miou=m1, stream=stream)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 20
    e0.record()
    for _ in range(reps):
        st.st_miou(pred, lab, wl.n_classes, wl.ignore_index, confusion=conf1, miou=m1, stream=stream)
    e1.record()
    torch.cuda.synchronize()
    miou_us = e0.elapsed_time(e1) / reps * 1e3
    # the same call once more with an event pair around every launch: the histogram kernel alone
    st.st_profile_reset()
    st.st_profile_filter(None)
    st.st_profile_enable(True)
    for _ in range(reps):
        st.st_miou(pred, lab, wl.n_classes, wl.ignore_index, confusion=conf1, miou=m1, stream=stream)
    torch.cuda.synchronize()
    mprof = {k: v[1] / v[0] * 1e3 for k, v in st.st_profile_read().items()}
    st.st_profile_enable(False)
    st.st_profile_reset()
    miou_bytes = 5.0 * wl.n * wl.H * wl.W
    hist_us = mprof["confusion"]
    miou_pass = {"bound": "hbm", "kernel": "confusion", "avg_launch_us": round(hist_us, 2),
                 "achieved": round(miou_bytes / hist_us / 1e3, 1), "unit": "GB/s",
                 "frac": round(miou_bytes / hist_us / 1e3 / PEAK_HBM_GBS, 5),
                 "us_per_call": round(miou_us, 2),
                 "launch_us": {k: round(v, 2) for k, v in mprof.items()},
                 "note": "st_miou; us_per_call is the whole call issued back to back from Python, avg_launch_us "
                         "the histogram kernel between its own events; 5 B per pixel"}
    # the loss-weight map from the labels (st_object_weights, once per key frame when the weighted
    # loss of Section 5.2 is used); streaming bound: 4 B label in + 1 B weight out per pixel
    wmap = torch.empty((wl.n, wl.H, wl.W), dtype=torch.uint8, device="cuda")
    ow_call = lambda: st.st_object_weights(lab, wl.n_classes, 4, ignore_index=wl.ignore_index, weights=wmap, stream=stream)
    for _ in range(3):
        ow_call()
    _, ms_ow = timed_calls(ow_call, 0, 30)
    st.st_profile_reset()
    st.st_profile_enable(True)
    for _ in range(reps):
        ow_call()
    torch.cuda.synchronize()
    ow_us = {k: v[1] / v[0] * 1e3 for k, v in st.st_profile_read().items()}["object_weights"]
    st.st_profile_enable(False)
    st.st_profile_reset()
    ow_bytes = 5.0 * wl.n * wl.H * wl.W
    weights_pass = {"bound": "hbm", "kernel": "object_weights", "avg_launch_us": round(ow_us, 2),
                    "achieved": round(ow_bytes / ow_us / 1e3, 1), "unit": "GB/s",
                    "frac": round(ow_bytes / ow_us / 1e3 / PEAK_HBM_GBS, 5),
                    "us_per_call": round(spread(ms_ow)["median"] * 1e3, 2),
                    "note": "st_object_weights, radius 4; us_per_call is the call issued from Python between two events "
                            "(median of 30), avg_launch_us its one kernel between events attached to the dispatch; "
                            "5 B per pixel"}
    # the forward alone (what a frame that is no key frame costs a client): st_head_forward
    for _ in range(3):
        st.st_head_forward(desc, f, p, pred=pred, workspace=ws, stream=stream)
    _, ms_fwd = timed_calls(lambda: st.st_head_forward(desc, f, p, pred=pred, workspace=ws, stream=stream), 0, 30)
    head_forward = {"ms_per_call": spread(ms_fwd), "frames_per_s": round(1e3 / spread(ms_fwd)["median"], 1),
                    "note": "st_head_forward (features -> class map), inputs resident in HBM"}

    # several clients in one call (one head and one key frame each; the server of Algorithm 3):
    # the same launches carry `clients` times the work, which fills the chip better
    grouped = None
    if args.clients > 0 and wl.n == 1 and not variant:
        G = args.clients
        wg = WL.small_variant(wl, n=G)
        dg = st.HeadDesc.of(wg)
        dg.grouped = 1
    if args.clients > 0 and wl.n == 1 and not variant and st.st_workspace_bytes(dg) > 0:   # (matrix-core shapes only)
        fg = upload(WL.make_features(wg))
        lg = torch.from_numpy(WL.make_labels(wg)).cuda()
        pg0 = torch.from_numpy(np.stack([WL.make_head_params(wg, seed=wg.init_seed + 17 * i) for i in range(G)])).cuda()
        pg = pg0.clone()
        wsg = st.new_workspace(dg)
        lossg = torch.zeros((wl.steps + 1, G), dtype=torch.float32, device="cuda")

        def grouped_run():
            st.st_partial_distill(dg, fg, lg, pg, wl.steps, wl.lr, losses=lossg, workspace=wsg, stream=stream,
                                  graph=use_graph)

        for _ in range(3):
            pg.copy_(pg0)
            grouped_run()
        reps = max(5, args.steps // 4)
        _, ms_g = timed_calls(grouped_run, 0, reps, before=lambda: pg.copy_(pg0))
        tg = spread(ms_g)["median"] * 1e-3
        grouped = {"clients": G, "head_steps_per_s": round(G * wl.steps / tg, 1),
                   "us_per_step": round(tg / wl.steps * 1e6, 2), "ms_per_call": spread(ms_g),
                   "note": "one st_partial_distill call trains `clients` heads on `clients` key frames "
                           "(desc.grouped = 1); head_steps_per_s counts one optimiser step of one head"}
        del fg, lg, pg, pg0, wsg

    # independent clients on streams of their own: no special mode, just concurrent calls
    streams_leg = None
    if args.streams > 1 and wl.n == 1 and not variant:
        try:
            clients = []
            for i in range(args.streams):
                wi = WL.small_variant(wl, feat_seed=wl.feat_seed + 101 * (i + 1), label_seed=wl.label_seed + 101 * (i + 1))
                pi0 = torch.from_numpy(WL.make_head_params(wi, seed=wi.init_seed + 17 * i)).cuda()
                clients.append(dict(f=upload(WL.make_features(wi)), lab=torch.from_numpy(WL.make_labels(wi)).cuda(),
                                    p0=pi0, p=pi0.clone(),
                                    ws=st.new_workspace(desc), s=torch.cuda.Stream(),
                                    vel=None if wl.momentum == 0.0 else torch.zeros_like(pi0),
                                    losses=torch.zeros(wl.steps + 1, dtype=torch.float32, device="cuda")))

            def client_call(c):
                with torch.cuda.stream(c["s"]):
                    c["p"].copy_(c["p0"], non_blocking=True)
                st.st_partial_distill(desc, c["f"], c["lab"], c["p"], wl.steps, wl.lr, momentum=wl.momentum,
                                      velocity=c["vel"],
                                      losses=c["losses"], workspace=c["ws"], stream=c["s"], graph=use_graph)

            for _ in range(3):
                for c in clients:
                    client_call(c)
            torch.cuda.synchronize()
            reps = max(10, args.steps)
            t0 = time.perf_counter()
            for _ in range(reps):
                for c in clients:
                    client_call(c)
            torch.cuda.synchronize()
            ts = time.perf_counter() - t0
            streams_leg = {"clients": args.streams, "head_steps_per_s": round(reps * args.streams * wl.steps / ts, 1),
                           "calls": reps * args.streams,
                           "note": "independent st_partial_distill calls (one key frame, head and workspace per "
                                   "client) issued round-robin on one stream per client; the sum over the clients"}
            del clients
        except Exception as e:      # the headline line must not depend on this leg
            streams_leg = {"error": f"{type(e).__name__}: {e}"}

    # The temporal clip (Algorithms 3 and 4 around the training step): labels that move two pixels per
    # frame, features that drift.  One early-exit call per frame: it scores the head on the frame
    # (forward + mean IoU) and trains only under the threshold.  Every key-frame iteration reads its
    # metric back to the host (Algorithm 1 branches on it).  Twice: on the configuration's noise
    # features every frame is a key frame; on features that carry the labels the trained head serves
    # the following frames and most frames cost one forward pass, the regime of the paper's videos
    # (Table 5: about one frame in twenty is a key frame).
    clip = clip_learnable = None
    if args.clip_frames > 0 and wl.name == "720p" and not variant:
        from paper_2003_10735_amd.clip import run_clip
        for learnable in (False, True):
            try:
                wc = WL.WORKLOADS["clip"]
                wc = WL.small_variant(wc, extra={**wc.extra, "frames": args.clip_frames})
                dc = st.HeadDesc.of(wc)
                frames_dev = [(upload(f_np), torch.from_numpy(lab_np).cuda())
                              for f_np, lab_np in WL.clip_frames(wc, learnable=learnable)]
                thr = float(wc.extra["threshold"])
                pc = torch.from_numpy(WL.make_head_params(wc)).cuda()
                wsc = st.new_workspace(dc)
                run_clip(dc, frames_dev[:2], pc.clone(), threshold=thr, max_updates=wc.steps, lr=wc.lr,
                         momentum=wc.momentum, workspace=wsc, stream=stream)          # warm-up
                r = run_clip(dc, frames_dev, pc, threshold=thr, max_updates=wc.steps, lr=wc.lr,
                             momentum=wc.momentum, workspace=wsc, stream=stream)
                key = np.array(r["key_frames"], dtype=bool)
                fms = np.array(r["frame_ms"])
                leg = {"frames": len(frames_dev), "frames_per_s": round(r["frames_per_s"], 1),
                       "key_frames": int(r["n_key_frames"]), "non_key_fraction": round(float(1.0 - key.mean()), 4),
                       "optimiser_steps": int(sum(r["updates"])),
                       "ms_per_key_frame": round(float(np.median(fms[key])), 4) if key.any() else None,
                       "ms_per_non_key_frame": round(float(np.median(fms[~key])), 4) if (~key).any() else None,
                       "threshold": thr, "max_updates": wc.steps,
                       "first_last_score": [round(r["scores"][0], 4), round(r["scores"][-1], 4)]}
                # the same clip from the same head with the caller's word that frames are key frames
                # (a server that is only sent key frames): the first pass computes its gradients at once
                rh = run_clip(dc, frames_dev, torch.from_numpy(WL.make_head_params(wc)).cuda(), threshold=thr,
                              max_updates=wc.steps, lr=wc.lr, momentum=wc.momentum, workspace=wsc, stream=stream,
                              expect_key_frames=True)
                leg["with_key_frame_hint"] = {"frames_per_s": round(rh["frames_per_s"], 1),
                                              "same_schedule": bool(rh["key_frames"] == r["key_frames"]
                                                                    and rh["updates"] == r["updates"])}
                if learnable:
                    leg["note"] = ("features = noise + a per-class code of each cell's label (not the configuration's "
                                   "inputs): the head trained on a key frame scores above the threshold on the frames "
                                   "that follow, which then cost one forward pass + metric + one host read-back each")
                    clip_learnable = leg
                else:
                    leg["note"] = ("the configuration's inputs: noise features say nothing about the labels, so every "
                                   "frame is a key frame trained for all its steps; one early-exit call per frame")
                    clip = leg
                del frames_dev, wsc
            except Exception as e:      # the headline line must not depend on this leg
                if learnable:
                    clip_learnable = {"error": f"{type(e).__name__}: {e}"}
                else:
                    clip = {"error": f"{type(e).__name__}: {e}"}

    # the other measured configurations (their own workloads, same protocol, fewer calls)
    configs = {}
    if wl.name == "720p" and not variant:
        for name in [n for n in args.other_configs.split(",") if n]:
            try:
                configs[name] = config_leg(st, WL, name, stream, 10 if name == "batch4" else 30, use_graph)
            except Exception as e:
                configs[name] = {"error": f"{type(e).__name__}: {e}"}

    # Partial against full distillation (Section 4.2; the paper's Table 2 reports 13 ms against 18 ms
    # per step for its whole student on an RTX 2080 Ti): the same key frame with the data-gradient of
    # the first trainable layer computed as well -- what an unfrozen front part would build on.
    partial_vs_full = None
    if wl.name == "720p" and not variant and not args.no_full_compare:
        try:
            pf = Problem(st, WL, wl, stream, full_backward=True)
            pf.call()
            if use_graph:
                pf.call(graph=True)
            torch.cuda.synchronize()
            _, ms_f = timed_calls(lambda: pf.run(graph=use_graph), 0, 30, before=pf.reset)
            t_full = spread(ms_f)["median"]
            partial_vs_full = {"partial_us_per_step": round(ms_per_call / wl.steps * 1e3, 2),
                               "full_us_per_step": round(t_full / wl.steps * 1e3, 2),
                               "partial_over_full": round(ms_per_call / t_full, 4),
                               "paper_table_2": {"partial_ms": 13, "full_ms": 18, "partial_over_full": round(13 / 18, 4),
                                                 "hardware": "RTX 2080 Ti, whole student (the front part is trained too)"},
                               "note": "full = every backward pass also computes d loss / d features (one more "
                                       "convolution launch per step); here only the head exists, so only the head's "
                                       "share of the saving shows"}
            del pf
        except Exception as e:
            partial_vs_full = {"error": f"{type(e).__name__}: {e}"}

    # The training recipe of the paper's experiments (Section 5.2): Adam at learning rate 0.01 on the
    # cross-entropy weighted x5 near and within objects.  The timed call makes the weight map from
    # the labels (st_object_weights), then trains with it.
    paper_recipe = None
    if wl.name == "720p" and not variant and not args.no_full_compare:
        try:
            pr = Problem(st, WL, wl, stream, optimizer="adam", weighted=True)

            def recipe_call():
                st.st_object_weights(pr.lab, wl.n_classes, 4, factor=5, ignore_index=wl.ignore_index, weights=pr.pw,
                                     stream=stream)
                pr.run(graph=use_graph)
            pr.reset(); recipe_call(); pr.reset(); recipe_call()
            torch.cuda.synchronize()
            _, ms_r = timed_calls(recipe_call, 0, 30, before=pr.reset)
            t_r = spread(ms_r)
            paper_recipe = {"ms_per_key_frame": t_r, "value": round(wl.steps / (t_r["median"] * 1e-3), 2), "unit": "steps/s",
                            "over_headline": round(t_r["median"] / ms_per_call, 4),
                            "loss_first_last": [float(pr.losses[0]), float(pr.losses[-1])],
                            "note": "Adam (lr 0.01, beta 0.9 / 0.999, eps 1e-8) + loss weights 5 within 4 pixels of a "
                                    "non-background label, 1 elsewhere; the weight map is made inside the timed call; "
                                    f"{wl.steps} steps per key frame like the headline"}
            del pr
        except Exception as e:
            paper_recipe = {"error": f"{type(e).__name__}: {e}"}

    cpu_baseline = None
    if not args.no_cpu_baseline:
        import oracle as O
        d = O.desc_of(wl)
        f64 = WL.features_as_f64(wl, prob.feats)
        k = wl.steps if wl.name in ("tiny", "720p") else 1
        tc0 = time.perf_counter()
        O.partial_distill(d, f64, prob.labels, prob.params0.astype(np.float64), k, wl.lr, momentum=wl.momentum)
        tc1 = time.perf_counter()
        cpu_baseline = {"value": round(k / (tc1 - tc0), 4), "unit": "steps/s", "cores": O.num_threads(),
                        "kind": "oracle",
                        "sample": f"the same {wl.name} key frame, {k} optimiser step(s) "
                                  f"({k + 1} forwards), float64, {tc1 - tc0:.1f} s"}

    peak = PEAK_TFLOPS_BF16 if wl.compute == "bf16" else PEAK_TFLOPS_F32
    out = {
        "metric": "key-frame partial-distill steps/sec at 1280x720 (fwd+bwd+update)",
        "value": round(steps_per_s, 2), "unit": "steps/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_call, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16" if wl.compute == "bf16" else "f32",
        "data": "synthetic",
        "config": {"workload": f"{wl.name}: features [{wl.n},{wl.c_in},{wl.h},{wl.w}] {wl.feat_dtype}, head "
                               f"{wl.c_in}->{wl.c1}->{wl.c2}->{wl.n_classes}, x8 to {wl.H}x{wl.W}, "
                               f"{wl.steps} {'Adam' if args.optimizer == 'adam' else 'SGD'} steps per key frame (one bench step = one key frame)",
                   "optimiser_steps_per_call": wl.steps, "lr": wl.lr, "momentum": wl.momentum, "optimizer": args.optimizer, "weighted_loss": bool(args.weighted_loss), "full_backward": bool(args.full_backward)},
        "step_definition": "one bench step = one st_partial_distill call = one key frame = "
                           f"{wl.steps} optimiser steps ({wl.steps + 1} forwards, {wl.steps} partial backwards, {wl.steps} updates); "
                           "ms_per_step is the median time of such a call between HIP events on the calling stream (the head is re-initialised between the calls, outside the events); "
                           "`value` counts optimiser steps",
        "ms_per_key_frame": round(ms_per_call, 4),
        "ms_per_optimiser_step": round(ms_per_call / wl.steps, 5),
        "ms_per_call": sp,
        "wall": {"ms_per_step": round(wall / args.steps * 1e3, 4), "value": round(args.steps * wl.steps / wall, 2),
                 "note": "host clock around the first K = `steps` calls, device synchronised on both sides"},
        "key_frames_per_s": round(1.0 / t_call, 3),
        "conv_tflops": round(call_flops(wl) / t_call / 1e12, 3),
        # the whole call against both roofs (a call of k steps has k + 1 forwards; its bytes are
        # counted as k steps' worth, a slight under-count)
        "whole_call": {"tflops": round(call_flops(wl) / t_call / 1e12, 3),
                       "mfma_frac": round(call_flops(wl) / t_call / 1e12 / peak, 5),
                       "algorithmic_GBs": round(step_bytes(wl) * wl.steps / t_call / 1e9, 1),
                       "hbm_frac": round(step_bytes(wl) * wl.steps / t_call / 1e9 / PEAK_HBM_GBS, 5),
                       "algorithmic_MB_per_step": round(step_bytes(wl) / 1e6, 2)},
        "loss_first_last": [float(final_losses[0]), float(final_losses[-1])],
        "kernel_us": breakdown,
        "roofline": roofline,
        "other_kernels": others,
        "miou_pass": miou_pass,
        "weights_pass": weights_pass,
        "head_forward": head_forward,
        "launch": "cached HIP graph (st_distill_opts.use_graph)" if use_graph
                  else (graph_note or "") + "kernel by kernel in the stream",
        "stream_launch": stream_launch,
        "grouped": grouped,
        "streams": streams_leg,
        "clip": clip,
        "clip_learnable": clip_learnable,
        "configs": configs,
        "partial_vs_full": partial_vs_full,
        "paper_recipe": paper_recipe,
        "cpu_baseline": cpu_baseline,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()

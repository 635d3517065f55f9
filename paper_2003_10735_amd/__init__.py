"""Thin Python binding of libshadowtutor_head.so (hand-written HIP for MI355X / gfx950).

Argument marshalling only: torch tensors supply device memory and the stream; every step of
the partial-distillation path runs inside the library's kernels.  There is no CPU fallback:
if the shared library is missing, importing the entry points raises.

Function names mirror the C ABI declared in include/shadowtutor_head.h.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libshadowtutor_head.so")

ST_OK = 0
ST_ERR_NULL, ST_ERR_SHAPE, ST_ERR_ARG, ST_ERR_WORKSPACE, ST_ERR_HIP, ST_ERR_NO_DEVICE, ST_ERR_TOO_LARGE = -1, -2, -3, -4, -5, -6, -7
ST_NOALLOC_MAX_WORKSPACE_MIB = 96
ST_OBJECT_WEIGHTS_MAX_RADIUS = 32
ST_F32, ST_BF16 = 0, 1
ST_NCHW, ST_NHWC = 0, 1
ST_COMPUTE_F32, ST_COMPUTE_BF16 = 0, 1
ST_OPTIM_SGD, ST_OPTIM_ADAM = 0, 1

EXPORTS = ["st_num_params", "st_workspace_bytes", "st_head_forward", "st_head_forward_noalloc", "st_partial_distill",
           "st_miou", "st_object_weights", "st_strerror", "st_last_hip_error", "st_version",
           "st_get_workspace_layout", "st_profile_enable", "st_profile_filter", "st_profile_reset", "st_profile_read",
           "st_next_stride", "st_schedule_bounds", "st_schedule_total_time",
           "st_graph_cache_clear", "st_graph_cache_size", "st_metric_polling"]


class StHeadDesc(C.Structure):
    _fields_ = [(k, C.c_int32) for k in ("n", "c_in", "h", "w", "c1", "c2", "n_classes", "upscale",
                                          "feat_dtype", "feat_layout", "compute", "ignore_index",
                                          "grouped")]


class StDistillOpts(C.Structure):
    _fields_ = [("momentum", C.c_float), ("velocity", C.c_void_p), ("threshold", C.c_double),
                ("strict_break", C.c_int32), ("return_best", C.c_int32),
                ("optimizer", C.c_int32), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("adam_m", C.c_void_p), ("adam_v", C.c_void_p), ("adam_t0", C.c_int32),
                ("pixel_weights", C.c_void_p), ("feature_grad", C.c_void_p), ("use_graph", C.c_int32),
                ("best_params", C.c_void_p), ("expect_key_frame", C.c_int32)]


class StScheduleParams(C.Structure):
    _fields_ = [(k, C.c_double) for k in ("t_si", "t_sd", "t_ti", "t_net", "s_net", "min_stride",
                                          "max_stride", "max_updates")]


class StScheduleBounds(C.Structure):
    _fields_ = [(k, C.c_double) for k in ("t_c_lower", "t_c_upper", "traffic_lower", "traffic_upper",
                                          "throughput_lower", "throughput_upper")]


class StDistillResult(C.Structure):
    _fields_ = [("losses", C.c_void_p), ("mious", C.c_void_p), ("confusion", C.c_void_p),
                ("pred", C.c_void_p), ("steps_taken", C.c_int32), ("best_metric", C.c_double),
                ("first_metric", C.c_double)]


class StWorkspaceLayout(C.Structure):
    _fields_ = [(k, C.c_size_t) for k in ("feat", "a1", "a2", "da1", "da2", "z", "g", "theta",
                                           "grad", "elem_size", "total", "row_pitch", "grad_copies",
                                           "grad_stride")] + [("splits", C.c_size_t * 3)]


class StKernelStat(C.Structure):
    _fields_ = [("name", C.c_char * 48), ("launches", C.c_int64), ("total_ms", C.c_double)]


class DistillReturn(tuple):
    """(steps_taken, best_metric or None) of st_partial_distill; with a threshold also
    `.first_metric`, the metric before any update."""
    first_metric = None


class StError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().st_strerror(status).decode()
        extra = f" (hipError {lib().st_last_hip_error()})" if status == ST_ERR_HIP else ""
        super().__init__(f"{where}: {msg}{extra} [status {status}]")


_LIB = None


def lib():
    """The loaded shared library.  Raises if it has not been built (no fallback exists)."""
    global _LIB
    if _LIB is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2003_10735_amd.build` "
                "(hipcc, gfx950).  There is no CPU fallback.")
        L = C.CDLL(LIB_PATH)
        L.st_num_params.restype = C.c_size_t
        L.st_num_params.argtypes = [C.POINTER(StHeadDesc)]
        L.st_workspace_bytes.restype = C.c_size_t
        L.st_workspace_bytes.argtypes = [C.POINTER(StHeadDesc)]
        L.st_head_forward.restype = C.c_int
        L.st_head_forward.argtypes = [C.POINTER(StHeadDesc), C.c_void_p, C.c_void_p, C.c_void_p,
                                      C.c_void_p, C.c_void_p, C.c_void_p]
        L.st_head_forward_noalloc.restype = C.c_int
        L.st_head_forward_noalloc.argtypes = [C.POINTER(StHeadDesc), C.c_void_p, C.c_void_p, C.c_void_p,
                                              C.c_void_p, C.c_void_p]
        L.st_partial_distill.restype = C.c_int
        L.st_partial_distill.argtypes = [C.POINTER(StHeadDesc), C.c_void_p, C.c_void_p, C.c_void_p,
                                         C.c_int32, C.c_float, C.POINTER(StDistillOpts),
                                         C.POINTER(StDistillResult), C.c_void_p, C.c_void_p]
        L.st_miou.restype = C.c_int
        L.st_miou.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int32, C.c_int32, C.c_void_p,
                              C.c_void_p, C.c_void_p]
        L.st_object_weights.restype = C.c_int
        L.st_object_weights.argtypes = [C.c_void_p] + [C.c_int32] * 8 + [C.c_void_p, C.c_void_p]
        L.st_strerror.restype = C.c_char_p
        L.st_strerror.argtypes = [C.c_int]
        L.st_last_hip_error.restype = C.c_int
        L.st_version.restype = C.c_char_p
        L.st_get_workspace_layout.restype = C.c_int
        L.st_get_workspace_layout.argtypes = [C.POINTER(StHeadDesc), C.POINTER(StWorkspaceLayout)]
        L.st_next_stride.restype = C.c_double
        L.st_next_stride.argtypes = [C.c_double] * 5
        L.st_schedule_bounds.restype = C.c_int
        L.st_schedule_bounds.argtypes = [C.POINTER(StScheduleParams), C.POINTER(StScheduleBounds)]
        L.st_schedule_total_time.restype = C.c_double
        L.st_schedule_total_time.argtypes = [C.POINTER(StScheduleParams)] + [C.c_double] * 4
        L.st_graph_cache_size.restype = C.c_int
        L.st_profile_enable.argtypes = [C.c_int]
        L.st_profile_filter.argtypes = [C.c_char_p]
        L.st_profile_read.restype = C.c_int
        L.st_profile_read.argtypes = [C.POINTER(StKernelStat), C.c_int]
        _LIB = L
    return _LIB


@dataclass
class HeadDesc:
    n: int
    c_in: int
    h: int
    w: int
    c1: int
    c2: int
    n_classes: int
    feat_dtype: int = ST_BF16
    compute: int = ST_COMPUTE_BF16
    ignore_index: int = -1
    upscale: int = 8
    feat_layout: int = ST_NCHW
    grouped: int = 0        # 1: n heads, one per frame; per-head arrays are [n, ...]

    def c(self) -> StHeadDesc:
        return StHeadDesc(self.n, self.c_in, self.h, self.w, self.c1, self.c2, self.n_classes,
                          self.upscale, self.feat_dtype, self.feat_layout, self.compute,
                          self.ignore_index, self.grouped)

    @staticmethod
    def of(wl) -> "HeadDesc":
        """Descriptor of a workloads.Workload."""
        return HeadDesc(wl.n, wl.c_in, wl.h, wl.w, wl.c1, wl.c2, wl.n_classes,
                        ST_BF16 if wl.feat_dtype == "bf16" else ST_F32,
                        ST_COMPUTE_BF16 if wl.compute == "bf16" else ST_COMPUTE_F32,
                        wl.ignore_index)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def _check(status: int, where: str):
    if status != ST_OK:
        raise StError(status, where)


def st_num_params(desc: HeadDesc) -> int:
    d = desc.c()
    return int(lib().st_num_params(C.byref(d)))


def st_workspace_bytes(desc: HeadDesc) -> int:
    d = desc.c()
    return int(lib().st_workspace_bytes(C.byref(d)))


def st_get_workspace_layout(desc: HeadDesc) -> dict:
    d, out = desc.c(), StWorkspaceLayout()
    _check(lib().st_get_workspace_layout(C.byref(d), C.byref(out)), "st_get_workspace_layout")
    return {k: ([int(v) for v in getattr(out, k)] if k == "splits" else int(getattr(out, k)))
            for k, _ in StWorkspaceLayout._fields_}


def new_workspace(desc: HeadDesc, device="cuda"):
    """A device buffer of st_workspace_bytes(desc) bytes (torch allocations are 256-byte aligned)."""
    import torch
    nbytes = st_workspace_bytes(desc)
    if nbytes == 0:
        raise StError(ST_ERR_SHAPE, "st_workspace_bytes")
    return torch.empty(nbytes, dtype=torch.uint8, device=device)


def st_head_forward(desc: HeadDesc, features, head_params, logits_lowres=None, pred=None,
                    workspace=None, stream=None):
    """features [n,c_in,h,w] (float32 or bfloat16 cuda tensor), head_params float32 [num_params]
    ([n, num_params] for a grouped descriptor).  Fills logits_lowres [n,C,h,w] float32 and/or pred [n,8h,8w] uint8 when given."""
    d = desc.c()
    ws = workspace if workspace is not None else new_workspace(desc, features.device)
    _check(lib().st_head_forward(C.byref(d), _ptr(features), _ptr(head_params), _ptr(logits_lowres),
                                 _ptr(pred), _ptr(ws), _stream(stream)), "st_head_forward")
    return logits_lowres, pred


def st_head_forward_noalloc(desc: HeadDesc, features, head_params, logits_lowres=None, pred=None, stream=None):
    """st_head_forward on the library's built-in scratch: no workspace argument, no allocation."""
    d = desc.c()
    _check(lib().st_head_forward_noalloc(C.byref(d), _ptr(features), _ptr(head_params), _ptr(logits_lowres),
                                         _ptr(pred), _stream(stream)), "st_head_forward_noalloc")
    return logits_lowres, pred


def st_partial_distill(desc: HeadDesc, features, teacher_labels, head_params, steps: int, lr: float,
                       momentum: float = 0.0, velocity=None, threshold: float = 0.0,
                       strict_break: bool = True, return_best: bool = False, losses=None,
                       mious=None, confusion=None, pred=None, workspace=None, stream=None,
                       adam=None, pixel_weights=None, feature_grad=None, graph=False, best_params=None,
                       expect_key_frame=False):
    """Runs the library's st_partial_distill; head_params (and the optimiser state) are updated
    in place.  `adam` = dict(m=, v=, t0=0, beta1=0.9, beta2=0.999, eps=1e-8) selects Adam;
    `pixel_weights` (uint8 [n,8h,8w]) scales every pixel's loss; `feature_grad` (float32
    [n,c_in,h,w]) receives d loss / d features of the last backward pass; `best_params` (float32,
    like head_params) receives Algorithm 1's best parameters when a threshold is given.
    With a grouped descriptor head_params and the optimiser state are [n, num_params] and losses
    [steps+1, n].  graph=True launches the call through the library's cached HIP graph
    (st_distill_opts.use_graph).  expect_key_frame=True (with a threshold) makes the first pass compute its
    gradients at once instead of scoring first (st_distill_opts.expect_key_frame).
    Returns (steps_taken, best_metric or None); with a threshold the returned tuple also carries
    `.first_metric`, the metric before any update."""
    d = desc.c()
    ws = workspace if workspace is not None else new_workspace(desc, features.device)
    use_opts = (momentum != 0.0 or threshold > 0.0 or velocity is not None or adam is not None
                or pixel_weights is not None or feature_grad is not None or graph or best_params is not None
                or expect_key_frame)
    opts = StDistillOpts(momentum, _ptr(velocity), threshold, 1 if strict_break else 0,
                         1 if return_best else 0, ST_OPTIM_SGD, 0.0, 0.0, 0.0, None, None, 0,
                         _ptr(pixel_weights), _ptr(feature_grad), 1 if graph else 0, _ptr(best_params),
                         1 if expect_key_frame else 0)
    if adam is not None:
        opts.optimizer = ST_OPTIM_ADAM
        opts.beta1, opts.beta2 = adam.get("beta1", 0.9), adam.get("beta2", 0.999)
        opts.eps = adam.get("eps", 1e-8)
        opts.adam_m, opts.adam_v = _ptr(adam["m"]), _ptr(adam["v"])
        opts.adam_t0 = int(adam.get("t0", 0))
    res = StDistillResult(_ptr(losses), _ptr(mious), _ptr(confusion), _ptr(pred), 0, 0.0)
    st = lib().st_partial_distill(C.byref(d), _ptr(features), _ptr(teacher_labels), _ptr(head_params),
                                  steps, lr, C.byref(opts) if use_opts else None, C.byref(res),
                                  _ptr(ws), _stream(stream))
    _check(st, "st_partial_distill")
    ret = DistillReturn((int(res.steps_taken), (float(res.best_metric) if threshold > 0.0 else None)))
    ret.first_metric = float(res.first_metric) if threshold > 0.0 else None
    return ret


def st_miou(pred, labels, n_classes: int, ignore_index: int = -1, confusion=None, miou=None,
            stream=None):
    """pred uint8 [..], labels int32 [..] cuda tensors.  Returns (confusion int64 [C,C], miou float64 [1])."""
    import torch
    if confusion is None:
        confusion = torch.empty((n_classes, n_classes), dtype=torch.int64, device=pred.device)
    if miou is None:
        miou = torch.empty(1, dtype=torch.float64, device=pred.device)
    _check(lib().st_miou(_ptr(pred), _ptr(labels), pred.numel(), n_classes, ignore_index,
                         _ptr(confusion), _ptr(miou), _stream(stream)), "st_miou")
    return confusion, miou


def st_object_weights(labels, n_classes: int, radius: int, factor: int = 5, background: int = 0,
                      ignore_index: int = -1, weights=None, stream=None):
    """labels int32 [n, H, W] cuda tensor -> uint8 [n, H, W] loss weights (`factor` within `radius`
    pixels of an object label, 1 elsewhere): the `pixel_weights` of st_partial_distill."""
    import torch
    n, H, W = labels.shape
    if weights is None:
        weights = torch.empty((n, H, W), dtype=torch.uint8, device=labels.device)
    _check(lib().st_object_weights(_ptr(labels), n, H, W, n_classes, background, ignore_index, radius, factor,
                                   _ptr(weights), _stream(stream)), "st_object_weights")
    return weights


def st_graph_cache_clear():
    lib().st_graph_cache_clear()


def st_graph_cache_size() -> int:
    return int(lib().st_graph_cache_size())


def st_metric_polling(on: bool):
    lib().st_metric_polling(1 if on else 0)


def st_profile_enable(on: bool):
    lib().st_profile_enable(1 if on else 0)


def st_profile_filter(substring):
    lib().st_profile_filter(None if substring is None else substring.encode())


def st_profile_reset():
    lib().st_profile_reset()


def st_profile_read(max_stats: int = 64) -> dict:
    arr = (StKernelStat * max_stats)()
    n = lib().st_profile_read(arr, max_stats)
    if n < 0:
        raise StError(n, "st_profile_read")
    return {arr[i].name.decode(): (int(arr[i].launches), float(arr[i].total_ms)) for i in range(n)}


def st_next_stride(stride, metric, threshold, min_stride, max_stride) -> float:
    return float(lib().st_next_stride(stride, metric, threshold, min_stride, max_stride))


def st_schedule_bounds(**params) -> dict:
    """Keyword arguments: the fields of st_schedule_params.  Returns the six bounds."""
    p = StScheduleParams(**{k: float(v) for k, v in params.items()})
    out = StScheduleBounds()
    _check(lib().st_schedule_bounds(C.byref(p), C.byref(out)), "st_schedule_bounds")
    return {k: getattr(out, k) for k, _ in StScheduleBounds._fields_}


def st_schedule_total_time(n_frames, n_distill_steps, n_key_frames, t_c, **params) -> float:
    p = StScheduleParams(**{k: float(v) for k, v in params.items()})
    return float(lib().st_schedule_total_time(C.byref(p), n_frames, n_distill_steps, n_key_frames, t_c))


def st_version() -> str:
    return lib().st_version().decode()

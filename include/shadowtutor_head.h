/*
 * shadowtutor_head.h -- C ABI of the MI355X (gfx950) partial-distillation library.
 *
 * The library runs, on one GPU, the server-side student-training step of ShadowTutor
 * restricted to the trainable tail ("head") of the student segmentation network:
 *
 *   Forward          head convolutions + x8 bilinear up-sampling to the frame's resolution
 *                    (Algorithm 1, "Forward"; Section 2.2: output has the input's spatial size)
 *   ComputeMetric    mean IoU of the predicted class map against the teacher's labels (Eq. 1)
 *   ComputeLoss      mean per-pixel cross-entropy against the teacher's hard labels
 *                    (Algorithm 1, "ComputeLoss"; Section 5.2), optionally weighted per pixel
 *   PartialBackward  chain rule from the loss down to the first trainable layer and no
 *                    further: the frozen front part's output (the feature map) is an input
 *                    and never receives a gradient (Section 4.2)
 *   OptimStep        gradient descent, optionally with momentum, or Adam (Algorithm 1,
 *                    "OptimStep"; Section 5.2)
 *
 * The head is  conv3x3(c_in->c1)+bias+ReLU,  conv3x3(c1->c2)+bias+ReLU,  conv1x1(c2->n_classes)
 * +bias,  x8 bilinear up-sampling (pixel centres at half-integers, edge replication).
 *
 * Conventions
 *   - Every tensor pointer is a DEVICE pointer owned by the caller unless it says HOST.  The
 *     library neither frees nor keeps any of them after the call returns.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the default stream).
 *     Calls return without synchronising, except st_partial_distill with a positive
 *     `threshold`, whose loop exits are decided on the host (every iteration hands its metric to
 *     the host through a small page-locked buffer the library keeps per calling thread) and which
 *     has finished when it returns.  (From the second read on, the stream
 *     already computes the iteration's gradients while the host waits; when the loop ends there
 *     they are left unused in the workspace and no parameter has changed.  A call whose first
 *     metric already reaches the threshold -- the frame is no key frame -- costs one forward
 *     pass and writes none of the caller's parameter or optimiser vectors.)
 *   - Dense row-major layouts: features [n, c_in, h, w] (or [n, h, w, c_in] with feat_layout =
 *     ST_NHWC); labels / pred [n, 8h, 8w]; low-resolution logits [n, n_classes, h, w].
 *   - head_params is one flat float32 vector: W1 (OIHW) | b1 | W2 (OIHW) | b2 | W3 (OI) | b3.
 *     It is what the server sends back to the client after training ("UpdatedPart").
 *   - Every function returns ST_OK (0) or a negative st_status; nothing throws or aborts.
 *     Arguments are validated on the host before any GPU work is enqueued.
 *   - `workspace` is caller-owned device scratch of at least st_workspace_bytes(desc) bytes,
 *     256-byte aligned; its contents on entry do not matter and two calls may not share one
 *     workspace concurrently.
 */
#ifndef SHADOWTUTOR_HEAD_H
#define SHADOWTUTOR_HEAD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum st_status {
    ST_OK = 0,
    ST_ERR_NULL = -1,      /* a required pointer is NULL */
    ST_ERR_SHAPE = -2,     /* non-positive or unsupported dimension, upscale != 8 */
    ST_ERR_ARG = -3,       /* steps < 0, non-finite lr / momentum, bad enum value */
    ST_ERR_WORKSPACE = -4, /* workspace NULL or misaligned */
    ST_ERR_HIP = -5,       /* a HIP runtime call failed (st_last_hip_error() tells which) */
    ST_ERR_NO_DEVICE = -6, /* no usable GPU in this process */
    ST_ERR_TOO_LARGE = -7  /* st_head_forward_noalloc: the shape needs more than its built-in scratch */
} st_status;

enum { ST_F32 = 0, ST_BF16 = 1 };                 /* st_head_desc.feat_dtype */
enum { ST_NCHW = 0, ST_NHWC = 1 };                /* st_head_desc.feat_layout */
enum { ST_COMPUTE_F32 = 0, ST_COMPUTE_BF16 = 1 }; /* st_head_desc.compute */

/* Shape of one training problem.
 * compute = ST_COMPUTE_F32: every convolution in float32 (reference-precision path).
 * compute = ST_COMPUTE_BF16: convolution operands (features, weights, activations and the
 *   back-propagated gradients) are rounded to bfloat16, products accumulate in float32 on the
 *   matrix cores; master weights, optimiser arithmetic, logits, loss and weight gradients stay
 *   float32.  Shapes with c_in and c1 multiples of 64 and c2 one of 64, 128, 256 run on the
 *   matrix-core kernels; every other shape runs on plain tiled kernels
 *   with the same rounding points (same results up to the order of float32 additions).
 * Limits: upscale == 8; 2 <= n_classes <= 32; labels outside [0, n_classes) are skipped like
 * ignore_index (they count neither in the loss nor in the metric).
 *
 * grouped = 0: one head, trained on a mini-batch of n frames (one loss over all of them).
 * grouped = 1: n clients in one call (the server of Algorithm 3 serves one student per client):
 *   n heads of the same shape, head f sees frame f only.  Every per-head array then holds n
 *   consecutive blocks: head_params, velocity, adam_m, adam_v are [n, st_num_params] and losses is
 *   [steps + 1, n]; the result of head f is what a call with n = 1 on frame f alone gives.  All
 *   heads take the same number of steps with the same learning rate: threshold must be <= 0, and
 *   feature_grad NULL (ST_ERR_ARG otherwise).  Runs on the matrix-core kernels only
 *   (ST_ERR_SHAPE for compute / shapes that do not, see above). */
typedef struct st_head_desc {
    int32_t n, c_in, h, w;     /* feature map [n, c_in, h, w]                         */
    int32_t c1, c2, n_classes; /* conv3x3 c_in->c1, conv3x3 c1->c2, conv1x1 c2->classes */
    int32_t upscale;           /* 8                                                   */
    int32_t feat_dtype;        /* ST_F32 | ST_BF16: element type of `features`        */
    int32_t feat_layout;       /* ST_NCHW: features [n, c_in, h, w]; ST_NHWC: [n, h, w, c_in] */
    int32_t compute;           /* ST_COMPUTE_F32 | ST_COMPUTE_BF16                    */
    int32_t ignore_index;      /* label value to skip; -1 = none                      */
    int32_t grouped;           /* 0: one head for all n frames; 1: n heads, one per frame */
} st_head_desc;

/* Options of st_partial_distill (NULL = plain gradient descent, fixed step count). */
typedef struct st_distill_opts {
    float momentum;       /* mu in v <- mu v + g, theta <- theta - lr v; 0 = plain descent   */
    float* velocity;      /* in/out, st_num_params floats, same order as head_params;
                             required when momentum != 0 (zero it before the first key frame) */
    double threshold;     /* THRESHOLD of Algorithm 1 (compared with the float64 metric);
                             <= 0 runs exactly `steps` updates                               */
    int32_t strict_break; /* 1: leave the loop when metric > threshold (as printed);
                             0: when metric >= threshold                                     */
    int32_t return_best;  /* with threshold > 0 -- 1: head_params receives best_student of
                             Algorithm 1 (strictly-better rule); 0: the last parameters.
                             Only the parameters are rolled back to the best iteration: the
                             optimiser state (velocity, adam_m, adam_v), out->pred,
                             out->confusion and entry steps_taken of losses / mious always
                             describe the last pass (Algorithm 1 returns parameters and metric
                             only; the metric of the returned ones is out->best_metric)      */
    /* Optimiser (Algorithm 1, OptimStep).  ST_OPTIM_SGD: the descent above.  ST_OPTIM_ADAM: the
     * optimiser of the paper's experiments (Section 5.2, learning rate 0.01); the paper gives
     * no further constants, the published defaults are beta1 0.9, beta2 0.999, eps 1e-8.
     * Step t = adam_t0 + 1, adam_t0 + 2, ..:
     *   m <- beta1 m + (1 - beta1) g,  v <- beta2 v + (1 - beta2) g^2,
     *   theta <- theta - lr (m / (1 - beta1^t)) / (sqrt(v / (1 - beta2^t)) + eps).
     * momentum must be 0 with Adam. */
    int32_t optimizer;    /* ST_OPTIM_SGD | ST_OPTIM_ADAM                                    */
    float beta1, beta2, eps;
    float* adam_m;        /* in/out, st_num_params floats each, same order as head_params;   */
    float* adam_v;        /* required with ST_OPTIM_ADAM (zero them before the first step)   */
    int32_t adam_t0;      /* optimiser steps already taken on this state (>= 0)              */
    /* Loss weighting (Section 5.2: the cross-entropy of pixels near and within non-background
     * objects is scaled by 5).  DEVICE pointer to one uint8 weight per pixel, [n, 8h, 8w], or NULL
     * for weight 1 everywhere.  Which pixels count as "near" is the caller's decision.  The loss
     * is the weighted mean  sum w_p CE_p / sum w_p  over the valid pixels; the metric ignores
     * the weights. */
    const uint8_t* pixel_weights;
    /* Full backward pass, for comparison with partial distillation (Section 4.2) or for a caller
     * that owns an unfrozen front part: DEVICE pointer to float32 [n, c_in, h, w] (in this order
     * whatever feat_layout says), or NULL.  When
     * given, every backward pass also computes d loss / d features (the data-gradient of the
     * first layer, which partial distillation leaves out); the tensor holds that of the last
     * backward pass of the call (untouched if no step is taken).  On the matrix-core path this
     * needs c1 in multiples of 64 (ST_ERR_SHAPE otherwise). */
    float* feature_grad;
    /* Launch through a HIP graph.  A step is a handful of short kernels, and in a stream every launch
     * costs more dispatch time than it does inside a graph.  With use_graph = 1 and threshold <= 0
     * the library records the call's launches into a graph the first time it sees this exact call
     * (same descriptor, pointers, step count, learning rate and options, same device), keeps the
     * instantiated graph in a small per-process cache (the oldest of 8 is dropped) and launches it
     * on `stream`; later identical calls only launch the cached graph.  The kernels, their order
     * and their results are those of the plain call; the buffers are read when the graph runs, so
     * their contents may change between calls.  Needs a stream created by the caller (with the
     * NULL stream, while that stream is being captured by the caller, or while st_profile_enable
     * is on, the call runs as if use_graph were 0).  Instantiating a graph allocates host and
     * driver memory; st_graph_cache_clear() releases it. */
    int32_t use_graph;
    /* With threshold > 0: DEVICE pointer to st_num_params floats (same order as head_params) that
     * receives best_student of Algorithm 1 whatever return_best says -- so a caller can have the
     * last parameters in head_params and the best ones here -- or NULL.  Ignored without a
     * threshold (there the last parameters are the result). */
    float* best_params;
    /* With threshold > 0: 1 tells the library that the frame is very likely a key frame (a server
     * that is only sent key frames, Algorithm 3).  The first pass then computes its gradients and
     * queues the backward pass at once, as every later pass does, instead of scoring the head first
     * and looking at the metric before anything else is queued; a key frame saves a loss pass and
     * a wait of the host, a frame whose first metric already reaches the threshold wastes one
     * backward pass.  Results are the same either way.  0: score first (the default). */
    int32_t expect_key_frame;
} st_distill_opts;
enum { ST_OPTIM_SGD = 0, ST_OPTIM_ADAM = 1 };

/* Outputs of st_partial_distill.  The struct lives in HOST memory; the arrays are DEVICE
 * pointers and each may be NULL.  Entry i of losses / mious describes the parameters before
 * update i+1, entry `steps_taken` the returned ones (k updates = k+1 forwards). */
typedef struct st_distill_result {
    float* losses;       /* [steps + 1]; grouped: [steps + 1, n]            */
    double* mious;       /* [steps + 1, n]  per-frame mean IoU              */
    int64_t* confusion;  /* [n, C, C] of the last forward; row = label, column = prediction */
    uint8_t* pred;       /* [n, 8h, 8w] class map of the last forward       */
    int32_t steps_taken; /* HOST, written by the call (== steps unless threshold > 0) */
    double best_metric;  /* HOST, written only when threshold > 0           */
    double first_metric; /* HOST, written only when threshold > 0: the metric (mean over the frames)
                            before any update, the one Algorithm 1 first compares with THRESHOLD */
} st_distill_result;

/* Number of float32 values in one head's parameters:
 * c1*c_in*9 + c1 + c2*c1*9 + c2 + n_classes*c2 + n_classes.  0 if desc is NULL or invalid. */
size_t st_num_params(const st_head_desc* desc);

/* Bytes of device scratch the calls below need for this shape.  0 if desc is invalid. */
size_t st_workspace_bytes(const st_head_desc* desc);

/* Forward (Algorithm 1, "Forward"): features -> low-resolution logits and/or the predicted
 * class map (lowest index among the largest up-sampled logits).
 *   features       [n, c_in, h, w], float32 or bfloat16 as desc says; read only
 *   head_params    st_num_params floats (grouped: n such blocks); read only
 *   logits_lowres  [n, n_classes, h, w] float32, or NULL
 *   pred           [n, 8h, 8w] uint8, or NULL                                              */
int st_head_forward(const st_head_desc* desc, const void* features, const float* head_params,
                    float* logits_lowres, uint8_t* pred, void* workspace, void* stream);

/* st_head_forward for callers that cannot allocate device memory and have no workspace to pass:
 * code under HIP graph capture, tight serving loops (most frames of a stream are not key frames
 * and only need this forward), harnesses that forbid hipMalloc.  Same arguments, kernels and
 * results as st_head_forward, but the workspace is a device array built into the library:
 * ST_NOALLOC_MAX_WORKSPACE_MIB MiB per GPU the library runs on, held from the first call on that
 * GPU until the process ends (enough for the 1280x720 head 256 -> 128 -> 128 -> 19, which needs
 * 75 MiB).  The call allocates nothing, on the device or through any library; shapes with
 * st_workspace_bytes(desc) above the limit are refused with ST_ERR_TOO_LARGE before any GPU work.
 * The first call on a device looks the array's address up (hipGetSymbolAddress); make that call
 * outside a capture.  Every call on a GPU uses that GPU's one array: calls that overlap on one
 * GPU (two streams, two threads) race -- serialise them.  The event profile (st_profile_enable)
 * does not see this call's launches. */
#define ST_NOALLOC_MAX_WORKSPACE_MIB 96
int st_head_forward_noalloc(const st_head_desc* desc, const void* features, const float* head_params,
                            float* logits_lowres, uint8_t* pred, void* stream);

/* Student training on one key frame (Algorithm 1 restricted to the head, Section 4.2):
 * `steps` times { loss, partial backward, optimiser step }, with a forward + metric before the
 * first and after every update.  features are never written and get no gradient.
 *   teacher_labels [n, 8h, 8w] int32 hard labels (the teacher's segmentation result)
 *   head_params    in/out, updated in place
 *   steps          >= 0 (0: forward + metric only; MAX_UPDATES when threshold > 0)
 *   lr             learning rate, finite
 * The loss is the mean over all valid pixels of all n frames (grouped: of the head's own frame);
 * the metric is per frame (the loop exits of Algorithm 1 use the mean over frames). */
int st_partial_distill(const st_head_desc* desc, const void* features,
                       const int32_t* teacher_labels, float* head_params, int32_t steps,
                       float lr, const st_distill_opts* opts, st_distill_result* out,
                       void* workspace, void* stream);

/* Mean IoU (Eq. 1) of a class map against labels: IoU_c = |pred_c & label_c| / |pred_c | label_c|
 * averaged over the classes present in the labels (0 when none is).
 *   pred [n_pixels] uint8, labels [n_pixels] int32
 *   confusion [C, C] int64 out (row = label, column = prediction), overwritten; required
 *   miou  one double out (device); 1 <= n_classes <= 256; labels outside [0, n_classes) and
 *         predictions >= n_classes are not counted; three short launches, no workspace       */
int st_miou(const uint8_t* pred, const int32_t* labels, int64_t n_pixels, int32_t n_classes,
            int32_t ignore_index, int64_t* confusion, double* miou, void* stream);

/* Loss weights from the teacher's label map (Section 5.2: the cross-entropy of pixels near and within
 * non-background objects is scaled by a factor of 5): weights = `factor` on every pixel that has, in
 * its own frame, a pixel with an object label at most `radius` columns and at most `radius` rows
 * away (itself included; the neighbourhood is cut off at the frame's edges), 1 on every other pixel.
 * The paper gives the factor and not what "near" means: the radius is the caller's choice.  A label
 * is an object when it lies in [0, n_classes) and is neither `background` nor `ignore_index`.
 *   labels   [n, height, width] int32, read only
 *   weights  [n, height, width] uint8 out, overwritten: what st_distill_opts.pixel_weights takes
 *   0 <= radius <= ST_OBJECT_WEIGHTS_MAX_RADIUS, 1 <= factor <= 255 (ST_ERR_ARG otherwise);
 *   1 <= n <= 65535, 1 <= height, width <= 2^19, n_classes >= 1 (ST_ERR_SHAPE otherwise).
 * One launch on `stream`, no workspace; labels and weights must not overlap. */
#define ST_OBJECT_WEIGHTS_MAX_RADIUS 32
int st_object_weights(const int32_t* labels, int32_t n, int32_t height, int32_t width, int32_t n_classes,
                      int32_t background, int32_t ignore_index, int32_t radius, int32_t factor, uint8_t* weights,
                      void* stream);

/* ---- scheduling arithmetic around the training step (host only, no GPU work) ------------- */

/* Key-frame striding, Algorithm 2: the ratio of the next stride to the current one is linear in
 * the metric through (0, 0) and (THRESHOLD, 1) below the threshold, and through (THRESHOLD, 1)
 * and (1, 2) from it on; the new stride is clamped to [min_stride, max_stride].
 * Returns NaN unless 0 < threshold < 1, min_stride <= max_stride and the inputs are numbers. */
double st_next_stride(double stride, double metric, double threshold, double min_stride, double max_stride);

/* Quantities of Section 4.4 (Table 1's notation).  Times in seconds; s_net in any unit of data
 * (the traffic bounds come out in that unit per second). */
typedef struct st_schedule_params {
    double t_si;        /* latency of student inference                          */
    double t_sd;        /* latency of one distillation step                      */
    double t_ti;        /* latency of teacher inference                          */
    double t_net;       /* network latency associated with one key frame         */
    double s_net;       /* networked data size associated with one key frame     */
    double min_stride, max_stride, max_updates;
} st_schedule_params;

typedef struct st_schedule_bounds_out {
    double t_c_lower, t_c_upper;                /* Eq. 2  */
    double traffic_lower, traffic_upper;        /* Eqs. 8, 12 */
    double throughput_lower, throughput_upper;  /* Eqs. 13, 14 (frames per second) */
} st_schedule_bounds_out;

/* Fills *out from *p.  ST_ERR_NULL / ST_ERR_ARG (negative or non-finite entries, min_stride <= 0,
 * max_stride < min_stride, t_si <= 0). */
int st_schedule_bounds(const st_schedule_params* p, st_schedule_bounds_out* out);

/* Eq. 3: total time to process n_frames with n_key_frames key frames, n_distill_steps
 * distillation steps and t_c seconds for the min_stride frames after each key frame.
 * (Eq. 4 is n_key_frames * s_net over it, Eq. 9 n_frames over it.)  NaN if p is NULL. */
double st_schedule_total_time(const st_schedule_params* p, double n_frames, double n_distill_steps,
                              double n_key_frames, double t_c);

/* Destroys every cached launch graph (see st_distill_opts.use_graph).  Synchronises the device. */
void st_graph_cache_clear(void);

/* Number of launch graphs in the cache. */
int st_graph_cache_size(void);

/* Human-readable text for a status code (static storage, never NULL). */
const char* st_strerror(int status);

/* The hipError_t (as int) of the most recent ST_ERR_HIP on this thread, else 0. */
int st_last_hip_error(void);

/* Library version, "major.minor". */
const char* st_version(void);

/* ---- introspection for tests and tools (no part of the training path) -------------------- */

/* Byte offsets of the library's internal buffers inside `workspace`, so that a test can look
 * at intermediate tensors after a call.  Offsets are 0 for buffers this shape does not use. */
typedef struct st_workspace_layout {
    size_t feat;      /* features, position-major [n, h+2, row_pitch, c_in], zero border    */
    size_t a1, a2;    /* activations after ReLU, same layout, c1 / c2 channels              */
    size_t da1, da2;  /* back-propagated gradients (after the ReLU mask), same layout       */
    size_t z;         /* low-resolution logits [n, C, h, w] float32                         */
    size_t g;         /* d loss / d z        [n, C, h, w] float32                           */
    size_t theta;     /* master parameters, internal order (3x3 weights as [o][kh][kw][i])  */
    size_t grad;      /* parameter gradient, internal order, as partial sums: grad_copies   */
                      /* copies grad_stride floats apart (the weight-gradient kernels split  */
                      /* the positions; a layer may use fewer copies than grad_copies: the   */
                      /* unused ones are not written).  On the matrix-core path the          */
                      /* classifier's share lies elsewhere (one slot per block).             */
    size_t elem_size; /* bytes per activation element: 4 (float32 path) or 2 (bfloat16)     */
    size_t total;     /* == st_workspace_bytes                                              */
    size_t row_pitch; /* cells per padded row: w + 2 rounded up to a multiple of 8          */
    size_t grad_copies, grad_stride;      /* see grad                                        */
    size_t splits[3]; /* copies the 3x3 layers 1, 2 and (plain kernels) the classifier use   */
} st_workspace_layout;

int st_get_workspace_layout(const st_head_desc* desc, st_workspace_layout* out);

/* How st_partial_distill with a positive threshold waits for each iteration's metric.  1 (the
 * default): the host polls the page-locked buffer the bookkeeping kernel writes, so nothing sits
 * in the stream between a pass and the kernels queued behind it; a thread whose polls time out
 * (host memory that is not coherent while a kernel runs) falls back by itself.  0: the host waits
 * on an event recorded behind the bookkeeping kernel (or on the stream), as on such a platform.
 * Results are identical either way.  Process-wide; takes effect from the next iteration on. */
void st_metric_polling(int on);

/* Per-kernel timing: when enabled, every kernel launch of the calls above is bracketed by a
 * pair of HIP events on the caller's stream.  st_profile_read synchronises those events and
 * returns, for each kernel name, the launch count and the summed duration since the last
 * st_profile_reset.  Off by default; switching it on adds event overhead to every launch. */
typedef struct st_kernel_stat {
    char name[48];
    int64_t launches;
    double total_ms;
} st_kernel_stat;

void st_profile_enable(int on);
void st_profile_filter(const char* substring); /* only kernels whose name contains it; NULL = all */
void st_profile_reset(void);
int st_profile_read(st_kernel_stat* stats, int max_stats); /* returns the number written, <0 on error */

#ifdef __cplusplus
}
#endif
#endif /* SHADOWTUTOR_HEAD_H */

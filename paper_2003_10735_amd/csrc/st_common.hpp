// Shared declarations of the partial-distillation library: geometry, workspace plan, launch
// bookkeeping and small device helpers.  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stddef.h>
#include <stdint.h>

#include "../../include/shadowtutor_head.h"

namespace st {

constexpr int UP = 8;  // up-sampling factor of the head's last stage

typedef __bf16 bf16;

// ------------------------------------------------------------------ geometry
// Activations live position-major ("NHWC") on a grid padded by one zero cell on every side, so
// a 3x3 tap is a plain offset and needs no bounds test:
//   element (img, y, x, c)  ->  ((img * Hp + y + 1) * Wp + x + 1) * C + c
// The row pitch Wp is w + 2 rounded up to a multiple of 8 (extra zero columns on the right): a
// step of one row is then a multiple of 16 bytes in the channel-major copies, which keeps the
// weight-gradient kernel's 8-position windows aligned.
struct Geo {
    int n, h, w;     // frames and low-resolution grid
    int Hp, Wp;      // padded grid: h + 2 rows of pitch Wp >= w + 2
    int H, W;        // frame resolution: 8h, 8w
    int c_in, c1, c2, C;
    int ignore_index;
    int grouped;     // 1: frame f has a head (parameters, loss, pixel count) of its own
    int nhwc;        // 1: the caller's features are [n, h, w, c_in] instead of [n, c_in, h, w]
    __host__ __device__ int heads() const { return grouped ? n : 1; }
    __host__ __device__ int head_of(int img) const { return grouped ? img : 0; }
    __host__ __device__ int positions() const { return n * h * w; }
    __host__ __device__ int padded_positions() const { return n * Hp * Wp; }
    __host__ __device__ long long pixels() const { return (long long)n * H * W; }
};

inline Geo make_geo(const st_head_desc& d)
{
    Geo g;
    g.n = d.n; g.h = d.h; g.w = d.w;
    g.Hp = d.h + 2; g.Wp = (d.w + 2 + 7) / 8 * 8;
    g.H = d.h * UP; g.W = d.w * UP;
    g.c_in = d.c_in; g.c1 = d.c1; g.c2 = d.c2; g.C = d.n_classes;
    g.ignore_index = d.ignore_index;
    g.grouped = d.grouped ? 1 : 0;
    g.nhwc = d.feat_layout == ST_NHWC ? 1 : 0;
    return g;
}

// Offsets (in floats) of the six parameter blocks; identical in the caller's flat vector and in
// the internal one.  Only the order *inside* W1 and W2 differs: OIHW outside, [o][kh][kw][i]
// inside (reduction index contiguous for the implicit GEMMs).
struct ParamOffsets {
    size_t W1, b1, W2, b2, W3, b3, total;
};

inline ParamOffsets param_offsets(const Geo& g)
{
    ParamOffsets o;
    o.W1 = 0;
    o.b1 = o.W1 + (size_t)g.c1 * g.c_in * 9;
    o.W2 = o.b1 + g.c1;
    o.b2 = o.W2 + (size_t)g.c2 * g.c1 * 9;
    o.W3 = o.b2 + g.c2;
    o.b3 = o.W3 + (size_t)g.C * g.c2;
    o.total = o.b3 + g.C;
    return o;
}

// ------------------------------------------------------------------ loss-kernel tiling
// The fused up-sample + cross-entropy kernel works on tiles of LOSS_TY x LOSS_TX groups of 8x8
// frame pixels (one thread per pixel column).  A tile touches (LOSS_TY + 2) x (LOSS_TX + 2)
// low-resolution cells and leaves its share of d loss / d z for them in a slot of its own.
#ifndef ST_LOSS_TX
#define ST_LOSS_TX 32
#endif
constexpr int LOSS_TX = ST_LOSS_TX;     // 8-pixel column groups per tile (two threads per pixel column)
#ifndef ST_LOSS_TY
#define ST_LOSS_TY 1
#endif
constexpr int LOSS_TY = ST_LOSS_TY;     // 8-pixel row groups per tile
constexpr int LOSS_CW = LOSS_TX + 2;    // cells per tile row
constexpr int LOSS_CH = LOSS_TY + 2;    // cell rows per tile

struct LossTiling {
    int tiles_x, tiles_y;   // per frame
    __host__ __device__ int tiles() const { return tiles_x * tiles_y; }
};

inline LossTiling loss_tiling(const Geo& g)
{
    LossTiling t;
    t.tiles_x = (g.w + LOSS_TX - 1) / LOSS_TX;
    t.tiles_y = (g.h + LOSS_TY - 1) / LOSS_TY;
    return t;
}

// ------------------------------------------------------------------ workspace plan
struct Plan {
    Geo g;
    ParamOffsets po;
    LossTiling lt;
    bool bf16;          // compute path
    size_t esz;         // bytes per activation element
    bool mfma;          // bf16 path on the matrix-core kernels (else the plain tiled kernels)
    // With several heads (Geo::grouped) every per-head buffer holds heads() consecutive blocks:
    // theta, vel, vel2, best (head_stride floats apart), grad (grad_copies * grad_stride floats
    // apart), grad3 (blocks3 slots apart), the bfloat16 weight copies (their own size apart),
    // the pixel counters (one each).
    int splits1, splits2;   // position splits (per head) of the layer-1 / layer-2 weight-gradient kernels
    int splits3;            // the same for the classifier layer on the plain kernels (the matrix-core
                            // path leaves per-block slots instead: blocks3)
    int blocks3;            // per-block partial slots (per head) of the layer-3 backward kernel
    int grad_copies;        // max of the splits: partial gradient copies the update sums
    size_t grad_stride;     // floats between two copies (total rounded up to 16 bytes)
    size_t head_stride;     // floats between two heads' parameters (total rounded up to 16 bytes)
    int guard;          // guard rows before and after every position-major activation buffer;
                        // also the number of guard columns in front of a channel-major row
    int PPT;            // row pitch (elements) of the channel-major copies
    // byte offsets
    size_t feat, a1, a2, da1, da2;
    size_t featT, a1T, da1T, da2T;        // channel-major copies [C][PPT] for the weight-gradient kernels
    size_t grad3;                         // per-block partials of dW3 / db3
    size_t zero_begin, zero_end;          // region cleared at the start of every call
    size_t z, g_slots, gz, tadj;   // tadj: U^T of the one-hot labels, [n, C, h, w] float32
    size_t lab8;                   // the labels as bytes, [n, 8h, 8w]: the class, or 255 for a pixel that does not count
    size_t zpart; int z_parts;     // shares of the logits left by the classifier-fused convolution
    size_t theta, vel, vel2, grad, best;   // vel: velocity or Adam's m; vel2: Adam's v
    size_t wq1, wq1t, wq2, wq2t, wq3;      // bfloat16 operand copies of the weights
    size_t wq3t;                           // W3 transposed, [c2][32 classes] (zero beyond C): MFMA A fragments of its backward
    size_t loss_part, counters, conf, scal;
    size_t losses, mious;            // staging when the caller passes no result arrays
    size_t total;
};

Plan make_plan(const st_head_desc& d);

// ------------------------------------------------------------------ launch bookkeeping
// Each kernel launch goes through Launch: it records the kernel's name for the optional event
// profile and turns a launch failure into ST_ERR_HIP instead of an abort.
struct Ctx {
    hipStream_t stream;
    int status;   // first failure sticks
    bool no_profile = false;   // launches of this call never carry profile events
};

// When the event profile is on and covers `name`, hands out a start/stop event pair that the
// launch attaches to the dispatch itself (hipExtLaunchKernelGGL): the pair then times the kernel
// only and puts no extra packet into the stream.  Otherwise both come back null.
void prof_events(Ctx& c, const char* name, hipEvent_t* start, hipEvent_t* stop);
void set_hip_error(hipError_t e);
void ensure_dynamic_lds(const void* kernel, size_t bytes);

#define ST_LAUNCH(ctx, name, kernel, grid, block, shmem, ...)                                   \
    do {                                                                                        \
        if ((ctx).status == ST_OK) {                                                            \
            hipEvent_t e0_ = nullptr, e1_ = nullptr;                                            \
            st::prof_events((ctx), name, &e0_, &e1_);                                           \
            if (e0_)                                                                            \
                hipExtLaunchKernelGGL(kernel, grid, block, shmem, (ctx).stream, e0_, e1_, 0,    \
                                      __VA_ARGS__);                                             \
            else                                                                                \
                hipLaunchKernelGGL(kernel, grid, block, shmem, (ctx).stream, __VA_ARGS__);      \
            hipError_t err_ = hipGetLastError();                                                \
            if (err_ != hipSuccess) { st::set_hip_error(err_); (ctx).status = ST_ERR_HIP; }     \
        }                                                                                       \
    } while (0)

// ------------------------------------------------------------------ device helpers
__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16 v) { return (float)v; }
template <class E> __device__ __forceinline__ E from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16 from_f32<bf16>(float v) { return (bf16)v; }  // RNE

inline int cdiv(long long a, long long b) { return (int)((a + b - 1) / b); }

}  // namespace st

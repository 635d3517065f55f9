// C ABI of the partial-distillation library: argument validation, workspace planning and the
// order in which the kernels of one call are enqueued.  No kernel lives here.
#include <math.h>
#include <string.h>

#include <atomic>
#include <chrono>
#include <mutex>
#include <string>
#include <utility>
#include <vector>

#include "st_kernels.hpp"
#include "st_finish.hpp"

namespace st {

// ------------------------------------------------------------------ errors
static thread_local int g_last_hip_error = 0;
void set_hip_error(hipError_t e) { g_last_hip_error = (int)e; }

#define ST_HIP(ctx, call)                                                                   \
    do {                                                                                    \
        if ((ctx).status == ST_OK) {                                                        \
            hipError_t e_ = (call);                                                         \
            if (e_ != hipSuccess) { st::set_hip_error(e_); (ctx).status = ST_ERR_HIP; }     \
        }                                                                                   \
    } while (0)

// ------------------------------------------------------------------ event profile
struct ProfRec { const char* name; hipEvent_t start, stop; };
static std::mutex g_prof_mutex;
static bool g_prof_on = false;
static std::string g_prof_filter;   // empty: every kernel
static std::vector<ProfRec> g_prof;
static std::vector<hipEvent_t> g_event_pool;

static hipEvent_t get_event()
{
    if (!g_event_pool.empty()) { hipEvent_t e = g_event_pool.back(); g_event_pool.pop_back(); return e; }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

void prof_events(Ctx& c, const char* name, hipEvent_t* start, hipEvent_t* stop)
{
    *start = nullptr;
    *stop = nullptr;
    if (!g_prof_on || c.no_profile) return;
    std::lock_guard<std::mutex> lk(g_prof_mutex);
    if (!g_prof_filter.empty() && !strstr(name, g_prof_filter.c_str())) return;
    hipEvent_t a = get_event(), b = get_event();
    if (!a || !b) {
        if (a) g_event_pool.push_back(a);
        if (b) g_event_pool.push_back(b);
        return;
    }
    g_prof.push_back(ProfRec{name, a, b});
    *start = a;
    *stop = b;
}

// kernels that need more than 64 KB of dynamic LDS must be told once (per process and device);
// a fixed table, so that no call path allocates host memory for it
void ensure_dynamic_lds(const void* kernel, size_t bytes)
{
    static std::mutex m;
    constexpr int MAX_DONE = 256;
    static const void* done_kernel[MAX_DONE];
    static int done_device[MAX_DONE];
    static int n_done = 0;
    int dev = -1;
    (void)hipGetDevice(&dev);
    std::lock_guard<std::mutex> lk(m);
    for (int i = 0; i < n_done; ++i)
        if (done_kernel[i] == kernel && done_device[i] == dev) return;
    (void)hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (n_done < MAX_DONE) { done_kernel[n_done] = kernel; done_device[n_done] = dev; ++n_done; }
}

// ------------------------------------------------------------------ validation and plan
static int validate(const st_head_desc* d)
{
    if (!d) return ST_ERR_NULL;
    if (d->n <= 0 || d->c_in <= 0 || d->h <= 0 || d->w <= 0 || d->c1 <= 0 || d->c2 <= 0) return ST_ERR_SHAPE;
    if (d->upscale != UP) return ST_ERR_SHAPE;
    if (d->n_classes < 2 || d->n_classes > 32) return ST_ERR_SHAPE;
    if (d->feat_dtype != ST_F32 && d->feat_dtype != ST_BF16) return ST_ERR_ARG;
    if (d->feat_layout != ST_NCHW && d->feat_layout != ST_NHWC) return ST_ERR_ARG;
    if (d->compute != ST_COMPUTE_F32 && d->compute != ST_COMPUTE_BF16) return ST_ERR_ARG;
    if (d->ignore_index < -1) return ST_ERR_ARG;
    if (d->grouped != 0 && d->grouped != 1) return ST_ERR_ARG;
    // 32-bit indexing inside the kernels
    const long long cmax = std::max(std::max(d->c_in, d->c1), std::max(d->c2, d->n_classes));
    const long long pp = (long long)d->n * (d->h + 2) * (d->w + 2 + 8);
    if (pp * cmax >= (1ll << 31)) return ST_ERR_SHAPE;
    if ((long long)d->n * d->h * d->w * UP * UP >= (1ll << 31)) return ST_ERR_SHAPE;
    if ((long long)d->c1 * d->c_in * 9 >= (1ll << 28) || (long long)d->c2 * d->c1 * 9 >= (1ll << 28))
        return ST_ERR_SHAPE;
    if (d->grouped) {
        // one head per frame: matrix-core kernels only, and all heads' parameters in 32-bit reach
        if (!make_plan(*d).mfma) return ST_ERR_SHAPE;
        if ((long long)d->n * ((long long)d->c1 * d->c_in * 9 + (long long)d->c2 * d->c1 * 9) >= (1ll << 30))
            return ST_ERR_SHAPE;
    }
    return ST_OK;
}

static size_t take(size_t& off, size_t bytes)
{
    const size_t at = off;
    off += (bytes + 255) / 256 * 256;
    return at;
}

Plan make_plan(const st_head_desc& d)
{
    Plan p;
    memset(&p, 0, sizeof(p));
    p.g = make_geo(d);
    p.po = param_offsets(p.g);
    p.lt = loss_tiling(p.g);
    p.bf16 = d.compute == ST_COMPUTE_BF16;
    p.esz = p.bf16 ? 2 : 4;
    const Geo& g = p.g;
    p.mfma = p.bf16 && conv3x3_mfma_supported(g.c_in, g.c1) && conv3x3_mfma_supported(g.c1, g.c2) &&
             wgrad3x3_mfma_supported(g.c_in, g.c1) && wgrad3x3_mfma_supported(g.c1, g.c2) &&
             conv3_mfma_supported(g.c2, g.C);
    p.splits1 = p.splits2 = p.splits3 = 1;
    if (p.mfma) wgrad_splits_for(g, &p.splits1, &p.splits2);
    else generic_wgrad_splits(g, &p.splits1, &p.splits2, &p.splits3);
    p.blocks3 = p.mfma ? conv3_bwd_blocks(g) : 0;
    p.grad_copies = std::max(std::max(p.splits1, p.splits2), p.splits3);
    // guard: a 3x3 tap reaches Wp + 1 rows back/ahead of a tile that may overrun the grid by
    // up to 255 positions
    p.guard = (g.Wp + 2 + 256 + 7) / 8 * 8;
    const size_t PP = (size_t)g.padded_positions();
    p.PPT = (int)(p.guard + (PP + 15) / 16 * 16 + p.guard);
    size_t off = 256;   // offset 0 is kept unused so that "0" can mean "absent"
    // position-major activations [guard + PP + guard][C]; the offsets point at position 0.
    // Everything from zero_begin to zero_end is cleared at the start of a call (borders, guards).
    p.zero_begin = off;
    auto act = [&](int C) {
        const size_t base = take(off, (PP + 2 * (size_t)p.guard) * C * p.esz);
        return base + (size_t)p.guard * C * p.esz;
    };
    p.feat = act(g.c_in);
    p.a1 = act(g.c1);
    p.a2 = act(g.c2);
    p.da1 = act(g.c1);
    p.da2 = act(g.c2);
    if (p.mfma) {
        p.featT = take(off, (size_t)g.c_in * p.PPT * 2);
        p.a1T = take(off, (size_t)g.c1 * p.PPT * 2);
        p.da1T = take(off, (size_t)g.c1 * p.PPT * 2);
        p.da2T = take(off, (size_t)g.c2 * p.PPT * 2);
    }
    p.zero_end = off;
    const size_t hw = (size_t)g.h * g.w;
    const size_t heads = (size_t)g.heads();
    p.z = take(off, (size_t)g.n * g.C * hw * 4);
    p.gz = take(off, (size_t)g.n * g.C * hw * 4);
    p.tadj = take(off, (size_t)g.n * g.C * hw * 4);
    p.lab8 = take(off, (size_t)g.pixels());
    p.z_parts = p.mfma ? g.c2 / 64 : 0;
    if (p.mfma) p.zpart = take(off, (size_t)p.z_parts * PP * ((g.C + 3) / 4 * 4) * 4);
    p.g_slots = take(off, loss_slot_floats(g) * 4);
    p.grad_stride = (p.po.total + 3) / 4 * 4;
    p.head_stride = p.grad_stride;
    p.theta = take(off, heads * p.head_stride * 4);
    p.vel = take(off, heads * p.head_stride * 4);
    p.vel2 = take(off, heads * p.head_stride * 4);
    p.grad = take(off, heads * p.grad_stride * 4 * p.grad_copies);
    p.grad3 = take(off, heads * std::max(p.blocks3, 1) * conv3_bwd_slot_floats(g) * 4);
    p.best = take(off, heads * p.head_stride * 4);
    if (p.bf16) {
        p.wq1 = take(off, heads * (p.po.b1 - p.po.W1) * 2);
        p.wq1t = take(off, heads * (p.po.b1 - p.po.W1) * 2);
        p.wq2 = take(off, heads * (p.po.b2 - p.po.W2) * 2);
        p.wq2t = take(off, heads * (p.po.b2 - p.po.W2) * 2);
        p.wq3 = take(off, heads * (p.po.b3 - p.po.W3) * 2);
        if (p.mfma) p.wq3t = take(off, heads * (size_t)g.c2 * 32 * 2);
    }
    p.loss_part = take(off, (size_t)loss_blocks(g) * 4);
    p.counters = take(off, std::max((size_t)256, heads * 8));   // valid pixels (their weights), one count per head
    p.conf = take(off, (size_t)g.n * g.C * g.C * 8);
    p.scal = take(off, (size_t)g.n * 8);               // per-frame mean IoU of the last pass (double)
    p.total = off;
    return p;
}

static hipStream_t as_stream(void* s) { return (hipStream_t)s; }

// Page-locked host memory for the per-iteration metric of the early-exit form.  The bookkeeping
// kernel writes the per-frame metric into it directly and, behind each value, a token the host
// chose for this pass (a release store at system scope); the host polls the tokens, so nothing
// sits in the stream between the pass and the backward kernels that follow it.  The buffer is
// asked for as host-coherent memory; should the tokens not show up within a bounded wait (the
// memory turned out not to be coherent while a kernel runs), the host synchronises the stream
// instead and this thread stops polling for good.  Where the device cannot address the buffer at
// all (`dev` null) the metric is copied into it (a copy into pageable memory would go through a
// staging buffer and cost several times as much).  One buffer per calling thread, grown on demand
// and kept until the process ends; `host` null if the allocation fails (the caller then reads
// back into ordinary memory).
static std::atomic<bool> g_metric_polling{true};   // st_metric_polling

struct MetricBuffer {
    double* host = nullptr;                  // [cap] per-frame metric
    volatile unsigned long long* tok = nullptr;   // [cap] token of the pass that wrote it
    double* dev = nullptr;                   // the same two arrays as kernels address them
    unsigned long long* dev_tok = nullptr;
    size_t cap = 0;
    unsigned long long next_token = 1;       // never repeats within the buffer's life
    bool poll = true;
};

static MetricBuffer& metric_buffer(size_t count)
{
    static thread_local MetricBuffer b;
    if (count > b.cap) {
        if (b.host) (void)hipHostFree(b.host);
        b.host = b.dev = nullptr; b.tok = nullptr; b.dev_tok = nullptr; b.cap = 0;
        const size_t want = std::max(count, (size_t)512);
        void* ptr = nullptr;
        hipError_t e = hipHostMalloc(&ptr, want * 16, hipHostMallocMapped | hipHostMallocCoherent);
        if (e != hipSuccess) {
            (void)hipGetLastError();
            b.poll = false;
            e = hipHostMalloc(&ptr, want * 16, hipHostMallocDefault);
        }
        if (e != hipSuccess) { (void)hipGetLastError(); return b; }
        memset(ptr, 0, want * 16);
        b.host = (double*)ptr;
        b.tok = (volatile unsigned long long*)(b.host + want);
        b.cap = want;
        void* dptr = nullptr;
        if (hipHostGetDevicePointer(&dptr, ptr, 0) == hipSuccess) {
            b.dev = (double*)dptr;
            b.dev_tok = (unsigned long long*)(b.dev + want);
        } else (void)hipGetLastError();
    }
    return b;
}

// Waits until the first `count` tokens of the buffer equal `token`, at most `limit_us`.
static bool wait_for_tokens(const MetricBuffer& b, size_t count, unsigned long long token, double limit_us)
{
    const auto t0 = std::chrono::steady_clock::now();
    for (size_t f = 0; f < count; ++f) {
        unsigned spins = 0;
        while (b.tok[f] != token) {
            if ((++spins & 255u) == 0 &&
                std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now() - t0).count() > limit_us)
                return false;
        }
    }
    std::atomic_thread_fence(std::memory_order_acquire);
    return true;
}

// An event per calling thread and device for the same read-back: the host waits for the copy of
// the metric while the stream already runs the backward pass behind it.
static hipEvent_t readback_event()
{
    static thread_local hipEvent_t ev = nullptr;
    static thread_local int ev_device = -1;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return nullptr;
    if (ev && dev != ev_device) { (void)hipEventDestroy(ev); ev = nullptr; }
    if (!ev) {
        if (hipEventCreateWithFlags(&ev, hipEventDisableTiming) != hipSuccess) { (void)hipGetLastError(); ev = nullptr; }
        ev_device = dev;
    }
    return ev;
}

static bool aligned(const void* p, size_t a) { return ((uintptr_t)p % a) == 0; }

// ------------------------------------------------------------------ built-in scratch
// Workspace of st_head_forward_noalloc: device memory that exists from the moment the library is
// loaded, so the call itself allocates nothing.  Every GPU the library runs on holds its own copy
// until the process ends.  In host code the array's name is only a handle: the device address is
// asked for once per device (hipGetSymbolAddress, with that device current) and kept in a table;
// the kernels get that address as their workspace argument, exactly like a caller's workspace.
constexpr size_t NOALLOC_SCRATCH_BYTES = (size_t)ST_NOALLOC_MAX_WORKSPACE_MIB << 20;
static __device__ __align__(256) unsigned char scratch[NOALLOC_SCRATCH_BYTES];
constexpr int NOALLOC_MAX_DEVICES = 64;
static std::mutex g_scratch_mutex;
static char* g_scratch_ptr[NOALLOC_MAX_DEVICES];

// the current device's copy of the scratch array (ST_ERR_HIP / ST_ERR_NO_DEVICE on failure)
static int scratch_of_current_device(char** out)
{
    int dev = -1;
    const hipError_t ge = hipGetDevice(&dev);
    if (ge != hipSuccess || dev < 0 || dev >= NOALLOC_MAX_DEVICES) { set_hip_error(ge); return ST_ERR_NO_DEVICE; }
    std::lock_guard<std::mutex> lk(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) { set_hip_error(e); return ST_ERR_HIP; }
        g_scratch_ptr[dev] = (char*)ptr;
    }
    *out = g_scratch_ptr[dev];
    return ST_OK;
}

// Clears everything a call relies on being zero, in one launch: the counters, and of the
// activation buffers
//  * plain kernels: all of them (they write interior cells only and rely on zero borders);
//  * matrix-core kernels: every position of a1, a2, da1, da2 and of their channel-major copies is
//    rewritten (zeros on the border) by its producer in every pass, so only the guards in front
//    of and behind the positions need clearing -- plus the features, unless their packing role
//    covers the padded grid as well (feat_covered).
static void prepare_workspace(Ctx& c, const Plan& p, char* ws, bool feat_covered)
{
    ZeroList z;
    const Geo& g = p.g;
    const int n_regions = 2 + 8 + 2 * 2 * (g.c1 / 32 + g.c2 / 32) + 2 * (g.c_in / 32) + 3;
    if (!p.mfma || n_regions > ZeroList::MAX) {
        z.add(ws + p.zero_begin, p.zero_end - p.zero_begin);
    } else {
        const size_t PP = (size_t)g.padded_positions(), G = (size_t)p.guard;
        if (!feat_covered) {
            z.add(ws + p.feat - G * g.c_in * 2, (PP + 2 * G) * g.c_in * 2);
            z.add(ws + p.featT, (size_t)g.c_in * p.PPT * 2);
        }
        const size_t pm[5] = {p.a1, p.a2, p.da1, p.da2, p.feat};
        const int pc[5] = {g.c1, g.c2, g.c1, g.c2, g.c_in};
        const int nbuf = feat_covered ? 5 : 4;
        for (int i = 0; i < nbuf; ++i) {
            z.add(ws + pm[i] - G * pc[i] * 2, G * pc[i] * 2);
            z.add(ws + pm[i] + PP * pc[i] * 2, G * pc[i] * 2);
        }
        // channel-major copies [C/32][PPT/8][32][8]: per channel block, the column groups of the
        // head guard and those from the end of the positions (rounded down to a group) on
        const size_t tm[4] = {p.a1T, p.da1T, p.da2T, p.featT};
        const int tc[4] = {g.c1, g.c1, g.c2, g.c_in};
        const size_t blk = (size_t)p.PPT * 32 * 2;                 // bytes of one channel block
        const size_t head = G * 32 * 2;                            // guard columns (a multiple of 8)
        const size_t tail_at = (G + PP / 8 * 8) * 32 * 2;
        for (int i = 0; i < nbuf - 1; ++i)
            for (int b = 0; b < tc[i] / 32; ++b) {
                z.add(ws + tm[i] + b * blk, head);
                z.add(ws + tm[i] + b * blk + tail_at, blk - tail_at);
            }
    }
    if (p.wq3t) z.add(ws + p.wq3t, (size_t)g.heads() * g.c2 * 32 * 2);      // rows of the classes beyond C stay zero
    z.add(ws + p.counters, std::max((size_t)256, (size_t)g.heads() * 8));
    z.add(ws + p.conf, (size_t)g.n * g.C * g.C * 8);
    zero_regions(c, z);
}

// one forward pass of the head: features (already packed) -> low-resolution logits.  The plain
// path leaves the planar tensor z; the matrix-core path leaves per-channel-tile shares of the
// logits (the classifier rides along with layer 2), which the loss kernel adds up -- and writes
// to z on the way.
static void forward(Ctx& c, const Plan& p, char* ws, float* z)
{
    if (!p.mfma) { generic_forward(c, p, ws, z); return; }
    const Geo& g = p.g;
    const float* theta = (const float*)(ws + p.theta);
    conv3x3_mfma(c, "conv1_fwd_mfma", p, (const bf16*)(ws + p.feat), (const bf16*)(ws + p.wq1), theta + p.po.b1,
                 nullptr, (bf16*)(ws + p.a1), (bf16*)(ws + p.a1T), g.c_in, g.c1, 0, 1);
    conv3x3_mfma(c, "conv2_fwd_logits_mfma", p, (const bf16*)(ws + p.a1), (const bf16*)(ws + p.wq2),
                 theta + p.po.b2, nullptr, (bf16*)(ws + p.a2), nullptr, g.c1, g.c2, 0, 2,
                 (const bf16*)(ws + p.wq3), (float*)(ws + p.zpart));
}

static ZSrc z_source(const Plan& p, char* ws, float* z)
{
    ZSrc zs;
    zs.planar = z; zs.parts = nullptr; zs.n_parts = 0; zs.b3 = nullptr; zs.z_out = nullptr;
    zs.b3_stride = p.head_stride;
    if (p.mfma) {
        zs.planar = nullptr;
        zs.parts = (const float*)(ws + p.zpart); zs.n_parts = p.z_parts;
        zs.b3 = (const float*)(ws + p.theta) + p.po.b3; zs.z_out = z;
    }
    return zs;
}

// partial backward: gradients of the head's parameters only; nothing flows into the features
// (with dfeat, the caller's float32 [n, c_in, h, w] tensor, the chain rule is continued one
// more layer: what an unfrozen front part would need, and what partial distillation saves)
// finish (matrix-core path only): the bookkeeping of the pass before rides on the first launch
static void backward(Ctx& c, const Plan& p, char* ws, float* dfeat, const FinishArgs* finish = nullptr)
{
    if (!p.mfma) {
        generic_backward(c, p, ws);
        if (dfeat) generic_feature_grad(c, p, ws, dfeat);
        return;
    }
    const Geo& g = p.g;
    float* grad = (float*)(ws + p.grad);
    conv3_bwd_mfma(c, p, (const float*)(ws + p.g_slots), (const float*)(ws + p.tadj),
                   (const unsigned long long*)(ws + p.counters), (const bf16*)(ws + p.a2),
                   (const bf16*)(ws + p.wq3t), (bf16*)(ws + p.da2), (bf16*)(ws + p.da2T), (float*)(ws + p.grad3), finish);
    conv3x3_mfma(c, "conv2_dgrad_mfma", p, (const bf16*)(ws + p.da2), (const bf16*)(ws + p.wq2t), nullptr,
                 (const bf16*)(ws + p.a1), dfeat ? (bf16*)(ws + p.da1) : nullptr, (bf16*)(ws + p.da1T), g.c2, g.c1, 1, 2);
    if (dfeat)
        conv3x3_mfma(c, "conv1_dgrad_mfma", p, (const bf16*)(ws + p.da1), (const bf16*)(ws + p.wq1t), nullptr, nullptr,
                     nullptr, nullptr, g.c1, g.c_in, 3, 1, nullptr, nullptr, dfeat);
    wgrad3x3_mfma(c, p, (const bf16*)(ws + p.da1T), (const bf16*)(ws + p.featT), (const bf16*)(ws + p.da2T),
                  (const bf16*)(ws + p.a1T), grad);
}

// ------------------------------------------------------------------ cached launch graphs
// One entry per distinct st_partial_distill call (everything the recorded launches depend on).
struct GraphKey {
    st_head_desc desc;
    const void* features; const int32_t* labels; float* params;
    int32_t steps; float lr;
    st_distill_opts opts;
    float* losses; double* mious; int64_t* confusion; uint8_t* pred;
    void* workspace;
    int device;
};
struct GraphEntry { GraphKey key; hipGraph_t graph; hipGraphExec_t exec; unsigned long long last_use; };
static std::mutex g_graph_mutex;      // the cache: look-up, insert, launch
static std::mutex g_capture_mutex;    // recording + instantiating a graph
static std::vector<GraphEntry> g_graphs;
static unsigned long long g_graph_clock = 0;
constexpr size_t GRAPH_CACHE_MAX = 8;

static void destroy_entry(GraphEntry& e)
{
    if (e.exec) (void)hipGraphExecDestroy(e.exec);
    if (e.graph) (void)hipGraphDestroy(e.graph);
    e.exec = nullptr; e.graph = nullptr;
}

}  // namespace st

using namespace st;

extern "C" {

size_t st_num_params(const st_head_desc* desc)
{
    if (validate(desc) != ST_OK) return 0;
    return param_offsets(make_geo(*desc)).total;
}

size_t st_workspace_bytes(const st_head_desc* desc)
{
    if (validate(desc) != ST_OK) return 0;
    return make_plan(*desc).total;
}

int st_get_workspace_layout(const st_head_desc* desc, st_workspace_layout* out)
{
    if (!out) return ST_ERR_NULL;
    const int v = validate(desc);
    if (v != ST_OK) return v;
    const Plan p = make_plan(*desc);
    out->feat = p.feat; out->a1 = p.a1; out->a2 = p.a2; out->da1 = p.da1; out->da2 = p.da2;
    out->z = p.z; out->g = p.gz; out->theta = p.theta; out->grad = p.grad;
    out->elem_size = p.esz; out->total = p.total; out->row_pitch = (size_t)p.g.Wp;
    out->grad_copies = (size_t)p.grad_copies; out->grad_stride = p.grad_stride;
    out->splits[0] = (size_t)p.splits1; out->splits[1] = (size_t)p.splits2; out->splits[2] = (size_t)p.splits3;
    return ST_OK;
}

// the launches of a forward call: clearing, packing + parameters, the two convolutions with the
// classifier, and the pass that leaves the class map
static int head_forward_launches(const st_head_desc* desc, const Plan& p, const void* features, const float* head_params,
                                 float* logits_lowres, uint8_t* pred, char* ws, void* stream, bool no_profile)
{
    Ctx c{as_stream(stream), ST_OK, no_profile};
    prepare_workspace(c, p, ws, pack_covers_borders(p, features, desc->feat_dtype));
    call_begin(c, p, ws, features, desc->feat_dtype, head_params, false, nullptr, nullptr);
    float* z = logits_lowres ? logits_lowres : (float*)(ws + p.z);
    forward(c, p, ws, z);
    if (pred || p.mfma)
        loss_pass(c, p.g, z_source(p, ws, z), nullptr, nullptr, nullptr, pred, nullptr, nullptr, nullptr, nullptr, nullptr,
                  false, false);
    return c.status;
}

int st_head_forward(const st_head_desc* desc, const void* features, const float* head_params,
                    float* logits_lowres, uint8_t* pred, void* workspace, void* stream)
{
    const int v = validate(desc);
    if (v != ST_OK) return v;
    if (!features || !head_params) return ST_ERR_NULL;
    if (!workspace || !aligned(workspace, 256)) return ST_ERR_WORKSPACE;
    const Plan p = make_plan(*desc);
    return head_forward_launches(desc, p, features, head_params, logits_lowres, pred, (char*)workspace, stream, false);
}

int st_head_forward_noalloc(const st_head_desc* desc, const void* features, const float* head_params,
                            float* logits_lowres, uint8_t* pred, void* stream)
{
    const int v = validate(desc);
    if (v != ST_OK) return v;
    if (!features || !head_params) return ST_ERR_NULL;
    const Plan p = make_plan(*desc);
    if (p.total > NOALLOC_SCRATCH_BYTES) return ST_ERR_TOO_LARGE;
    char* ws = nullptr;
    const int sr = scratch_of_current_device(&ws);
    if (sr != ST_OK) return sr;
    // (no event profile here: handing out event pairs may create events)
    return head_forward_launches(desc, p, features, head_params, logits_lowres, pred, ws, stream, true);
}

int st_partial_distill(const st_head_desc* desc, const void* features, const int32_t* teacher_labels,
                       float* head_params, int32_t steps, float lr, const st_distill_opts* opts,
                       st_distill_result* out, void* workspace, void* stream)
{
    const int v = validate(desc);
    if (v != ST_OK) return v;
    if (!features || !teacher_labels || !head_params) return ST_ERR_NULL;
    if (steps < 0 || !isfinite(lr)) return ST_ERR_ARG;
    float mu = 0.f;
    double threshold = 0.0;
    float* velocity = nullptr;
    bool strict = true, return_best = false;
    float* best_params = nullptr;
    bool expect_key_frame = false;
    bool use_adam = false;
    float *adam_m = nullptr, *adam_v = nullptr;
    double beta1 = 0.0, beta2 = 0.0;
    float adam_eps = 0.f;
    long long adam_t0 = 0;
    const uint8_t* pixel_weights = opts ? opts->pixel_weights : nullptr;
    float* feature_grad = opts ? opts->feature_grad : nullptr;
    if (opts) {
        if (!isfinite(opts->momentum) || opts->momentum < 0.f || isnan(opts->threshold)) return ST_ERR_ARG;
        if (opts->optimizer != ST_OPTIM_SGD && opts->optimizer != ST_OPTIM_ADAM) return ST_ERR_ARG;
        if (opts->optimizer == ST_OPTIM_ADAM) {
            if (opts->momentum != 0.f) return ST_ERR_ARG;
            if (!(opts->beta1 >= 0.f && opts->beta1 < 1.f) || !(opts->beta2 >= 0.f && opts->beta2 < 1.f) ||
                !(opts->eps > 0.f) || !isfinite(opts->eps) || opts->adam_t0 < 0)
                return ST_ERR_ARG;
            if (!opts->adam_m || !opts->adam_v) return ST_ERR_NULL;
            use_adam = true;
            adam_m = opts->adam_m; adam_v = opts->adam_v;
            beta1 = opts->beta1; beta2 = opts->beta2; adam_eps = opts->eps; adam_t0 = opts->adam_t0;
        }
        mu = opts->momentum;
        velocity = opts->velocity;
        if (mu != 0.f && !velocity) return ST_ERR_NULL;
        threshold = opts->threshold;
        strict = opts->strict_break != 0;
        return_best = opts->return_best != 0;
        best_params = opts->best_params;
        expect_key_frame = opts->expect_key_frame != 0;
    }
    if (!workspace || !aligned(workspace, 256)) return ST_ERR_WORKSPACE;
    const bool early_exit = threshold > 0.0;
    // several heads take the same steps: no per-head loop exits, no feature gradient
    if (desc->grouped && (early_exit || feature_grad)) return ST_ERR_ARG;

    if (opts && opts->use_graph && !early_exit && stream && !g_prof_on) {
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(as_stream(stream), &cap) == hipSuccess && cap == hipStreamCaptureStatusNone) {
            GraphKey key;
            memset(&key, 0, sizeof(key));          // padding bytes take part in the comparison
            key.desc = *desc;                      // (all int32: no padding)
            key.features = features; key.labels = teacher_labels; key.params = head_params;
            key.steps = steps; key.lr = lr;
            // (field by field: the caller's padding bytes must not take part)
            key.opts.momentum = opts->momentum; key.opts.velocity = opts->velocity;
            key.opts.threshold = opts->threshold; key.opts.strict_break = opts->strict_break;
            key.opts.return_best = opts->return_best; key.opts.optimizer = opts->optimizer;
            key.opts.beta1 = opts->beta1; key.opts.beta2 = opts->beta2; key.opts.eps = opts->eps;
            key.opts.adam_m = opts->adam_m; key.opts.adam_v = opts->adam_v; key.opts.adam_t0 = opts->adam_t0;
            key.opts.pixel_weights = opts->pixel_weights; key.opts.feature_grad = opts->feature_grad;
            key.opts.use_graph = 1;
            key.opts.best_params = opts->best_params;
            key.opts.expect_key_frame = opts->expect_key_frame;
            if (out) { key.losses = out->losses; key.mious = out->mious; key.confusion = out->confusion; key.pred = out->pred; }
            key.workspace = workspace;
            if (hipGetDevice(&key.device) != hipSuccess) return ST_ERR_NO_DEVICE;
            // The cache is locked only to look an entry up and to insert one: recording and
            // instantiating a graph (milliseconds) runs outside that lock, so callers on other
            // streams whose graphs exist go on.
            // (A launch itself happens under the lock, so that no other thread can evict and destroy
            //  the graph between the look-up and the launch.)
            auto launch_locked = [&](GraphEntry& e) -> int {
                e.last_use = ++g_graph_clock;
                const hipError_t le = hipGraphLaunch(e.exec, as_stream(stream));
                if (le != hipSuccess) { set_hip_error(le); return ST_ERR_HIP; }
                if (out) out->steps_taken = steps;
                return ST_OK;
            };
            {
                std::lock_guard<std::mutex> lk(g_graph_mutex);
                for (auto& e : g_graphs)
                    if (memcmp(&e.key, &key, sizeof(key)) == 0) return launch_locked(e);
            }
            {
                // One recording at a time (a lock of its own: the cache stays open to look-ups and
                // launches of other callers meanwhile).
                std::lock_guard<std::mutex> recording(g_capture_mutex);
                // record the plain call's launches (nothing runs while the stream is capturing)
                st_distill_opts plain = *opts;
                plain.use_graph = 0;
                const hipError_t begin = hipStreamBeginCapture(as_stream(stream), hipStreamCaptureModeRelaxed);
                if (begin != hipSuccess) { set_hip_error(begin); return ST_ERR_HIP; }
                const int rec = st_partial_distill(desc, features, teacher_labels, head_params, steps, lr, &plain, out,
                                                   workspace, stream);
                GraphEntry e;
                e.key = key; e.graph = nullptr; e.exec = nullptr; e.last_use = 0;
                const hipError_t end = hipStreamEndCapture(as_stream(stream), &e.graph);
                if (rec != ST_OK) { destroy_entry(e); return rec; }
                if (end != hipSuccess || !e.graph) { set_hip_error(end); destroy_entry(e); return ST_ERR_HIP; }
                const hipError_t inst = hipGraphInstantiate(&e.exec, e.graph, nullptr, nullptr, 0);
                if (inst != hipSuccess) { set_hip_error(inst); destroy_entry(e); return ST_ERR_HIP; }
                std::lock_guard<std::mutex> lk(g_graph_mutex);
                GraphEntry* twin = nullptr;      // another thread recorded the same call meanwhile
                for (auto& other : g_graphs)
                    if (memcmp(&other.key, &key, sizeof(key)) == 0) twin = &other;
                if (twin) {
                    destroy_entry(e);
                    return launch_locked(*twin);
                }
                if (g_graphs.size() >= GRAPH_CACHE_MAX) {
                    // drop the least recently used one; it may still be running somewhere
                    size_t old = 0;
                    for (size_t i = 1; i < g_graphs.size(); ++i)
                        if (g_graphs[i].last_use < g_graphs[old].last_use) old = i;
                    (void)hipDeviceSynchronize();
                    destroy_entry(g_graphs[old]);
                    g_graphs.erase(g_graphs.begin() + old);
                }
                g_graphs.push_back(e);
                return launch_locked(g_graphs.back());
            }
        }
    }

    const Plan p = make_plan(*desc);
    const Geo& g = p.g;
    // (the matrix-core kernel of the feature gradient needs c1 in multiples of 64)
    if (feature_grad && p.mfma && !conv3x3_mfma_supported(g.c1, g.c_in)) return ST_ERR_SHAPE;
    char* ws = (char*)workspace;
    Ctx c{as_stream(stream), ST_OK};

    float* theta = (float*)(ws + p.theta);
    float* z = (float*)(ws + p.z);
    unsigned long long* n_valid = (unsigned long long*)(ws + p.counters);
    unsigned long long* conf = (unsigned long long*)(ws + p.conf);
    double* metric_dev = (double*)(ws + p.scal);

    prepare_workspace(c, p, ws, pack_covers_borders(p, features, desc->feat_dtype));
    if (mu != 0.f) permute_params(c, p, velocity, (float*)(ws + p.vel), 0);
    if (use_adam) {
        permute_params(c, p, adam_m, (float*)(ws + p.vel), 0);
        permute_params(c, p, adam_v, (float*)(ws + p.vel2), 0);
    }
    // features packed, theta in internal order + bfloat16 copies, U^T of the labels and the sums
    // of the weights of the valid labels: one launch
    call_begin(c, p, ws, features, desc->feat_dtype, head_params, feature_grad != nullptr, teacher_labels, pixel_weights);

    double best_metric = -1.0, first_metric = -1.0;
    std::vector<double> frame_metric;
    int taken = 0;
    // best_student of Algorithm 1: while the best parameters so far are the current ones nothing is
    // copied; the optimiser kernel that overwrites them leaves them in the workspace on its way
    bool have_best = false, best_is_theta = false;
    const bool keep_best = early_exit && (return_best || best_params);
    bool params_out_done = false;
    for (int it = 0; it <= steps; ++it) {
        const bool last = it == steps;
        forward(c, p, ws, z);
        // The first pass of the early-exit form only scores the head (loss, class map, counts):
        // most frames are not key frames and end right there.  A key frame runs the same kernel
        // once more for the gradient half, below, once the host has seen the metric.
        // (unless the caller expects a key frame: then the first pass is like every later one)
        const bool key_hint = early_exit && expect_key_frame;
        const bool score_only = early_exit && it == 0 && !key_hint;
        loss_pass(c, g, z_source(p, ws, z), (const uint8_t*)(ws + p.lab8), pixel_weights, (const float*)(ws + p.tadj),
                  (out && (last || early_exit)) ? out->pred : nullptr,
                  (float*)(ws + p.g_slots),
                  (float*)(ws + p.gz), (float*)(ws + p.loss_part), conf, n_valid, !last && !score_only, !p.mfma);
        float* loss_out = (out && out->losses) ? out->losses + (size_t)it * g.heads() : nullptr;
        double* miou_out = (out && out->mious) ? out->mious + (size_t)it * g.n : nullptr;
        long long* conf_out = (out && out->confusion && (last || early_exit)) ? (long long*)out->confusion : nullptr;
        // The bookkeeping of this pass (loss, per-frame mIoU, clearing the counts) normally rides
        // along with the optimiser kernel at the end of the step; it needs a launch of its own
        // only when no update follows or when the host must see the metric first.
        const bool finish_now = last || early_exit;
        // (the last pass of the fixed-step form also hands the parameters back in the same launch)
        const bool out_now = last && !early_exit;
        // In the early-exit form the bookkeeping also writes the per-frame metric, and behind it the
        // pass's token, straight into page-locked host memory; the host polls the token (or, where
        // that is switched off, waits on an event), so no copy sits in the stream between the pass
        // and the backward kernels that follow.
        MetricBuffer* mb = early_exit ? &metric_buffer((size_t)g.n) : nullptr;
        double* metric_host = mb ? mb->host : nullptr;
        const bool device_writes = mb && mb->host && mb->dev;
        const unsigned long long token = device_writes ? mb->next_token++ : 0;
        // From the second pass on the backward kernels are queued before the host looks at the
        // metric (below); on the matrix-core path the bookkeeping then rides on the first of them
        // instead of taking a launch of its own.
        const bool speculate = early_exit && !last && !feature_grad && (it > 0 || key_hint);
        const bool polled = device_writes && mb->poll && g_metric_polling.load(std::memory_order_relaxed);
        const bool finish_rides = speculate && polled && p.mfma;
        if (finish_now && !finish_rides)
            finish_pass(c, p, ws, loss_out, miou_out, conf_out, out_now ? head_params : nullptr,
                        device_writes ? mb->dev : nullptr, device_writes ? mb->dev_tok : nullptr, token);
        params_out_done = params_out_done || out_now;
        bool stop = last;
        // In the early-exit form the backward pass of an iteration is put into the stream before
        // the host looks at the metric: it only produces gradients (nothing the results depend on
        // changes before the optimiser step), so the stream works through it while the host waits
        // for the metric, and it is simply not used when the loop ends here.  Not before the first
        // metric, though: most frames of a video are not key frames (Table 5: about one in
        // twenty is), their call ends right there and should cost a forward pass and no more.
        // (And not with a feature gradient: that one is an output.)
        bool backward_queued = false;
        if (early_exit) {
            // Algorithm 1 decides its exits on the metric: one small read-back per iteration
            if (!device_writes) {   // no pinned buffer the device can write: copy the metric
                if (!metric_host) { frame_metric.resize(g.n); metric_host = frame_metric.data(); }
                ST_HIP(c, hipMemcpyAsync(metric_host, metric_dev, sizeof(double) * g.n, hipMemcpyDeviceToHost, c.stream));
            }
            if (polled && c.status == ST_OK) {
                if (speculate) {
                    FinishArgs fin;
                    if (finish_rides) fin = finish_args(p, ws, loss_out, miou_out, conf_out, mb->dev, mb->dev_tok, token);
                    backward(c, p, ws, nullptr, finish_rides ? &fin : nullptr);
                    backward_queued = true;
                }
                // (the wait is bounded by far more than a pass can take: 20 ms and 2 us per grid cell)
                if (!wait_for_tokens(*mb, (size_t)g.n, token, 20000.0 + 2.0 * (double)g.positions())) {
                    // not seen while the stream runs: wait for the stream, and do so from now on
                    mb->poll = false;
                    ST_HIP(c, hipStreamSynchronize(c.stream));
                    if (c.status == ST_OK && !wait_for_tokens(*mb, (size_t)g.n, token, 0.0)) c.status = ST_ERR_HIP;
                }
            } else {
                hipEvent_t ev = speculate ? readback_event() : nullptr;
                if (ev) {
                    ST_HIP(c, hipEventRecord(ev, c.stream));
                    backward(c, p, ws, nullptr);
                    backward_queued = true;
                    ST_HIP(c, hipEventSynchronize(ev));
                } else {
                    ST_HIP(c, hipStreamSynchronize(c.stream));
                }
            }
            if (c.status != ST_OK) break;
            double metric = 0.0;
            for (int f = 0; f < g.n; ++f) metric += metric_host[f];
            metric /= g.n;
            if (it == 0) {
                first_metric = metric;
                best_metric = metric;
                if (!(metric < threshold)) stop = true;   // already good enough: no update at all
                else if (keep_best) have_best = best_is_theta = true;
            } else {
                if (metric > best_metric) {
                    best_metric = metric;
                    if (keep_best) best_is_theta = true;
                }
                if (strict ? metric > threshold : metric >= threshold) stop = true;
            }
        }
        if (stop) break;
        if (score_only)   // the gradient half of the pass just scored: no counts, no loss, no class map again
            loss_pass(c, g, z_source(p, ws, z), (const uint8_t*)(ws + p.lab8), pixel_weights, (const float*)(ws + p.tadj), nullptr,
                      (float*)(ws + p.g_slots), (float*)(ws + p.gz), nullptr, nullptr, n_valid, true, !p.mfma);
        if (!backward_queued) backward(c, p, ws, feature_grad);
        AdamStep ad;
        if (use_adam) {
            // bias corrections of step t in double precision, handed to the kernel as two factors
            const double t = (double)(adam_t0 + it + 1);
            ad.beta1 = (float)beta1; ad.beta2 = (float)beta2;
            ad.one_minus_beta1 = (float)(1.0 - beta1); ad.one_minus_beta2 = (float)(1.0 - beta2);
            ad.eps = adam_eps;
            ad.step_scale = (float)((double)lr / (1.0 - pow(beta1, t)));
            ad.inv_sqrt_bc2 = (float)(1.0 / sqrt(1.0 - pow(beta2, t)));
        }
        step_end(c, p, ws, lr, mu, use_adam ? &ad : nullptr, true, !finish_now, loss_out, miou_out, conf_out, nullptr,
                 feature_grad != nullptr, best_is_theta ? (float*)(ws + p.best) : nullptr);
        best_is_theta = false;
        ++taken;
    }
    const bool best_in_workspace = have_best && !best_is_theta;   // else the current parameters are the best
    if (early_exit && best_params) permute_params(c, p, best_in_workspace ? (const float*)(ws + p.best) : theta, best_params, 1);
    if (early_exit && return_best && best_in_workspace && taken > 0)
        ST_HIP(c, hipMemcpyAsync(theta, ws + p.best, p.po.total * 4, hipMemcpyDeviceToDevice, c.stream));
    // (a call that took no update -- not a key frame -- leaves the caller's vectors as they are)
    const bool untouched = early_exit && taken == 0;
    if (!params_out_done && !untouched) permute_params(c, p, theta, head_params, 1);
    if (mu != 0.f && !untouched) permute_params(c, p, (const float*)(ws + p.vel), velocity, 1);
    if (use_adam && !untouched) {
        permute_params(c, p, (const float*)(ws + p.vel), adam_m, 1);
        permute_params(c, p, (const float*)(ws + p.vel2), adam_v, 1);
    }
    if (early_exit) ST_HIP(c, hipStreamSynchronize(c.stream));
    if (out) {
        out->steps_taken = taken;
        if (early_exit) { out->best_metric = best_metric; out->first_metric = first_metric; }
    }
    return c.status;
}

int st_miou(const uint8_t* pred, const int32_t* labels, int64_t n_pixels, int32_t n_classes,
            int32_t ignore_index, int64_t* confusion, double* miou, void* stream)
{
    if (n_pixels < 0 || n_classes < 1 || n_classes > 256) return ST_ERR_SHAPE;
    if (((!pred || !labels) && n_pixels > 0) || !confusion || !miou) return ST_ERR_NULL;
    Ctx c{as_stream(stream), ST_OK};
    confusion_and_miou(c, pred, labels, n_pixels, n_classes, ignore_index, (long long*)confusion, miou);
    return c.status;
}

int st_object_weights(const int32_t* labels, int32_t n, int32_t height, int32_t width, int32_t n_classes,
                      int32_t background, int32_t ignore_index, int32_t radius, int32_t factor, uint8_t* weights,
                      void* stream)
{
    // the grid is (column tiles, row tiles, frames): the last two dimensions hold at most 65535 blocks
    if (n < 1 || n > 65535 || height < 1 || height > (1 << 19) || width < 1 || width > (1 << 19) || n_classes < 1)
        return ST_ERR_SHAPE;
    if (radius < 0 || radius > ST_OBJECT_WEIGHTS_MAX_RADIUS || factor < 1 || factor > 255) return ST_ERR_ARG;
    if (!labels || !weights) return ST_ERR_NULL;
    Ctx c{as_stream(stream), ST_OK};
    object_weights(c, labels, n, height, width, n_classes, background, ignore_index, radius, factor, weights);
    return c.status;
}

void st_graph_cache_clear(void)
{
    std::lock_guard<std::mutex> lk(g_graph_mutex);
    if (g_graphs.empty()) return;
    (void)hipDeviceSynchronize();
    for (auto& e : g_graphs) destroy_entry(e);
    g_graphs.clear();
}

int st_graph_cache_size(void)
{
    std::lock_guard<std::mutex> lk(g_graph_mutex);
    return (int)g_graphs.size();
}

const char* st_strerror(int status)
{
    switch (status) {
    case ST_OK: return "ok";
    case ST_ERR_NULL: return "a required pointer is NULL";
    case ST_ERR_SHAPE: return "unsupported or non-positive dimension";
    case ST_ERR_ARG: return "invalid argument value";
    case ST_ERR_WORKSPACE: return "workspace missing or not 256-byte aligned";
    case ST_ERR_HIP: return "a HIP runtime call failed";
    case ST_ERR_NO_DEVICE: return "no usable GPU";
    case ST_ERR_TOO_LARGE: return "shape needs more scratch than the no-allocation entry point has built in";
    default: return "unknown status";
    }
}

int st_last_hip_error(void) { return g_last_hip_error; }

const char* st_version(void) { return "0.1"; }

void st_metric_polling(int on) { g_metric_polling.store(on != 0, std::memory_order_relaxed); }

void st_profile_enable(int on)
{
    std::lock_guard<std::mutex> lk(g_prof_mutex);
    g_prof_on = on != 0;
}

void st_profile_filter(const char* substring)
{
    std::lock_guard<std::mutex> lk(g_prof_mutex);
    g_prof_filter = substring ? substring : "";
}

void st_profile_reset(void)
{
    std::lock_guard<std::mutex> lk(g_prof_mutex);
    for (auto& r : g_prof) { g_event_pool.push_back(r.start); g_event_pool.push_back(r.stop); }
    g_prof.clear();
}

int st_profile_read(st_kernel_stat* stats, int max_stats)
{
    if (!stats || max_stats <= 0) return ST_ERR_NULL;
    std::lock_guard<std::mutex> lk(g_prof_mutex);
    int n = 0;
    for (auto& r : g_prof) {
        if (hipEventSynchronize(r.stop) != hipSuccess) return ST_ERR_HIP;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess) return ST_ERR_HIP;
        int k = 0;
        for (; k < n; ++k)
            if (strncmp(stats[k].name, r.name, sizeof(stats[k].name) - 1) == 0) break;
        if (k == n) {
            if (n == max_stats) continue;
            memset(&stats[k], 0, sizeof(stats[k]));
            strncpy(stats[k].name, r.name, sizeof(stats[k].name) - 1);
            ++n;
        }
        stats[k].launches += 1;
        stats[k].total_ms += ms;
    }
    return n;
}

}  // extern "C"

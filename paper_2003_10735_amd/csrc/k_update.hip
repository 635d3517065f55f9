// Optimiser step over the flat parameter buffer (fused with the sum of the partial weight
// gradients and the bfloat16 operand copies of the new weights), the per-step bookkeeping
// kernel (loss, per-frame mean IoU) and the stand-alone confusion-matrix / mean-IoU kernels.
#include <string.h>

#include <algorithm>

#include "st_kernels.hpp"
#include "st_mfma.hpp"
#include "st_begin.hpp"
#include "st_finish.hpp"

namespace st {

// One kernel closes a training step; its blocks play three roles (block index ranges):
//
//  (1) optimiser step over the flat parameter buffer: theta <- theta - lr * v, v <- mu * v + g
//      (mu == 0: v is not touched), or an Adam step (Section 5.2 of the paper; AdamStep).  g is the sum, in ascending order, of the partial gradients
//      the backward kernels left behind: `splits1` copies for W1/b1, `splits2` for W2/b2 and, on
//      the plain kernels, `splits3` for W3/b3 (position splits of the weight-gradient kernels,
//      `stride` floats apart).
//  (2) the same for W3/b3 when the classifier's backward kernel left one slot per block: 16
//      threads per parameter, each adding a contiguous run of the slots, then the runs in order.
//  (3) bookkeeping of the forward pass that preceded the step: block f: mean IoU of frame f from
//      its confusion counts (copied out when asked, then cleared for the next pass); one more
//      block: the tile losses added in a fixed order (float64) over the number of valid pixels.
//
// Roles (1) and (2) also refresh the bfloat16 copies of the new weights:
//   wq1, wq2, wq3 : for the forward convolutions
//   wq2t          : W2 with the roles of o and i exchanged and the taps mirrored (tap' = 8 - tap),
//                   for the data-gradient of layer 2 run as a forward convolution
//   wq1t          : the same for W1, only when the caller wants the gradient of the features
//   wq3t          : W3 transposed, [c2][32] with zero columns beyond the classes: the A fragments of
//                   the classifier's backward kernel, read straight from memory
// wq3 has theta's order.  So do wq1 and wq2 for the plain tiled kernels (frag == 0); the
// matrix-core convolutions read wq1, wq2 and wq2t in fragment order (wfrag_index).
struct UpdateArgs {
    float* theta; float* vel; float* vel2; const float* grad; size_t stride; int splits1, splits2, splits3;
    bf16* wq1; bf16* wq1t; bf16* wq2; bf16* wq2t; bf16* wq3; bf16* wq3t;
    ParamOffsets po; int c_in, c1, c2;
    int frag;        // wq1 / wq2 / wq2t in fragment order
    float lr, mu;
    int adam; AdamStep ad;   // adam != 0: vel = first moment m, vel2 = second moment v
    int do_step;     // 0: only refresh the bfloat16 copies
    // parameter hand-over riding along: with ext_in (do_step == 0) theta is first taken from the
    // caller's vector (its OIHW order); with ext_out, nb_out more blocks copy theta out to it
    const float* ext_in; float* ext_out; int nb_out;
    // role (2)
    const float* part3; int blocks3; size_t slot3; int C;
    // block ranges; vec: role (1) handles four parameters per thread over [0, W3) and nb_tail
    // blocks handle [W3, total) one by one unless role (2) does
    int nb_main, nb_tail, nb_l3, nb_finish, vec;
    // several heads (blockIdx.y): floats / elements from one head's block to the next in the
    // parameter-like vectors (theta, vel, vel2), the caller's vectors, the partial gradients,
    // the bfloat16 copies and the layer-3 slots
    size_t hs_param, hs_ext, hs_grad, hs_wq1, hs_wq2, hs_wq3, hs_part3;
    // early-exit form only: with do_step, receives theta as it was before the step (theta's order), or null
    float* save_old;
};


// index in the caller's vector (3x3 weights OIHW) of the internal parameter j ([o][kh][kw][i])
__device__ __forceinline__ size_t external_index(const UpdateArgs& a, size_t j)
{
    if (j < a.po.b1) {
        const size_t r = j - a.po.W1, i = r % a.c_in, tap = (r / a.c_in) % 9, o = r / ((size_t)a.c_in * 9);
        return a.po.W1 + (o * a.c_in + i) * 9 + tap;
    }
    if (j >= a.po.W2 && j < a.po.b2) {
        const size_t r = j - a.po.W2, i = r % a.c1, tap = (r / a.c1) % 9, o = r / ((size_t)a.c1 * 9);
        return a.po.W2 + (o * a.c1 + i) * 9 + tap;
    }
    return j;
}

// (EE: the early-exit form's extras -- save_old here, the host copy of the metric in finish_block --
//  are compiled in; the kernels of the fixed-step form never look at those fields)
template <bool EE>
__device__ __forceinline__ void apply_update(const UpdateArgs& a, size_t j, float g)
{
    float w = a.ext_in ? a.ext_in[external_index(a, j)] : a.theta[j];
    if (a.ext_in) a.theta[j] = w;
    if (a.do_step) {
        if (EE && a.save_old) a.save_old[j] = w;
        if (a.adam) {
            const float m = __builtin_fmaf(a.ad.beta1, a.vel[j], a.ad.one_minus_beta1 * g);
            const float v = __builtin_fmaf(a.ad.beta2, a.vel2[j], a.ad.one_minus_beta2 * (g * g));
            a.vel[j] = m;
            a.vel2[j] = v;
            w = w - a.ad.step_scale * m / (__fsqrt_rn(v) * a.ad.inv_sqrt_bc2 + a.ad.eps);
        } else {
            if (a.mu != 0.f) {
                const float v = __builtin_fmaf(a.mu, a.vel[j], g);
                a.vel[j] = v;
                g = v;
            }
            w = __builtin_fmaf(-a.lr, g, w);
        }
        a.theta[j] = w;
    }
    if (a.wq1) {
        const bf16 q = (bf16)w;
        if (j < a.po.b1) {
            const size_t r = j - a.po.W1;
            if (a.frag) {
                const int i = (int)(r % a.c_in), tap = (int)((r / a.c_in) % 9), o = (int)(r / ((size_t)a.c_in * 9));
                a.wq1[wfrag_index(o, tap, i, a.c_in)] = q;
                if (a.wq1t) a.wq1t[wfrag_index(i, 8 - tap, o, a.c1)] = q;
            } else a.wq1[r] = q;
        } else if (j >= a.po.W2 && j < a.po.b2) {
            const size_t r = j - a.po.W2;
            if (a.frag) {
                const int i = (int)(r % a.c1), tap = (int)((r / a.c1) % 9), o = (int)(r / ((size_t)a.c1 * 9));
                a.wq2[wfrag_index(o, tap, i, a.c1)] = q;
                a.wq2t[wfrag_index(i, 8 - tap, o, a.c2)] = q;
            } else a.wq2[r] = q;
        } else if (j >= a.po.W3 && j < a.po.b3) {
            const size_t r = j - a.po.W3;
            a.wq3[r] = q;
            if (a.wq3t) a.wq3t[(r % a.c2) * 32 + r / a.c2] = q;
        }
    }
}

// Four consecutive parameters (all block boundaries below W3 are multiples of four here, so
// the four lie in the same block).
template <bool EE>
__device__ __forceinline__ void apply_update4(const UpdateArgs& a, size_t j, f32x4 g)
{
    f32x4 w;
    if (a.ext_in) {
#pragma unroll
        for (int e = 0; e < 4; ++e) w[e] = a.ext_in[external_index(a, j + e)];
        *(f32x4*)(a.theta + j) = w;
    } else w = *(const f32x4*)(a.theta + j);
    if (a.do_step) {
        if (EE && a.save_old) *(f32x4*)(a.save_old + j) = w;
        if (a.adam) {
            const f32x4 mo = *(const f32x4*)(a.vel + j), vo = *(const f32x4*)(a.vel2 + j);
            f32x4 m, v;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                m[e] = __builtin_fmaf(a.ad.beta1, mo[e], a.ad.one_minus_beta1 * g[e]);
                v[e] = __builtin_fmaf(a.ad.beta2, vo[e], a.ad.one_minus_beta2 * (g[e] * g[e]));
                w[e] = w[e] - a.ad.step_scale * m[e] / (__fsqrt_rn(v[e]) * a.ad.inv_sqrt_bc2 + a.ad.eps);
            }
            *(f32x4*)(a.vel + j) = m;
            *(f32x4*)(a.vel2 + j) = v;
        } else {
            if (a.mu != 0.f) {
                const f32x4 vo = *(const f32x4*)(a.vel + j);
                f32x4 v;
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = __builtin_fmaf(a.mu, vo[e], g[e]);
                *(f32x4*)(a.vel + j) = v;
                g = v;
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) w[e] = __builtin_fmaf(-a.lr, g[e], w[e]);
        }
        *(f32x4*)(a.theta + j) = w;
    }
    if (a.wq1) {
        bf16x4 q;
#pragma unroll
        for (int e = 0; e < 4; ++e) q[e] = (bf16)w[e];
        if (j < a.po.b1) {
            const size_t r = j - a.po.W1;
            if (a.frag) {
                const int i = (int)(r % a.c_in), tap = (int)((r / a.c_in) % 9), o = (int)(r / ((size_t)a.c_in * 9));
                *(bf16x4*)(a.wq1 + wfrag_index(o, tap, i, a.c_in)) = q;
                if (a.wq1t) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) a.wq1t[wfrag_index(i + e, 8 - tap, o, a.c1)] = q[e];
                }
            } else *(bf16x4*)(a.wq1 + r) = q;
        } else if (j >= a.po.W2 && j < a.po.b2) {
            const size_t r = j - a.po.W2;
            if (a.frag) {
                const int i = (int)(r % a.c1), tap = (int)((r / a.c1) % 9), o = (int)(r / ((size_t)a.c1 * 9));
                *(bf16x4*)(a.wq2 + wfrag_index(o, tap, i, a.c1)) = q;
#pragma unroll
                for (int e = 0; e < 4; ++e) a.wq2t[wfrag_index(i + e, 8 - tap, o, a.c2)] = q[e];
            } else *(bf16x4*)(a.wq2 + r) = q;
        }
    }
}

template <bool EE>
__device__ __forceinline__ void step_end_block(UpdateArgs a, const FinishArgs& f, int b, int head)
{
    if (head) {
        if (a.theta) { a.theta += head * a.hs_param; a.vel += head * a.hs_param; a.vel2 += head * a.hs_param; }
        if (EE && a.save_old) a.save_old += head * a.hs_param;
        if (a.grad) a.grad += head * a.hs_grad;
        if (a.wq1) { a.wq1 += head * a.hs_wq1; a.wq2 += head * a.hs_wq2; a.wq3 += head * a.hs_wq3; }
        if (a.wq1t) a.wq1t += head * a.hs_wq1;
        if (a.wq2t) a.wq2t += head * a.hs_wq2;
        if (a.wq3t) a.wq3t += head * (size_t)a.c2 * 32;
        if (a.ext_in) a.ext_in += head * a.hs_ext;
        if (a.ext_out) a.ext_out += head * a.hs_ext;
        if (a.part3) a.part3 += head * a.hs_part3;
    }
    if (b < a.nb_main) {
        // role (1), four parameters per thread over [0, W3): the partial gradients are added in
        // ascending order of the split, four loads in flight at a time
        if (a.vec) {
            const size_t j = ((size_t)b * 256 + threadIdx.x) * 4;
            if (j >= a.po.W3) return;
            f32x4 g = {0.f, 0.f, 0.f, 0.f};
            if (a.do_step) {
                const int splits = j < a.po.W2 ? a.splits1 : a.splits2;
                const float* gp = a.grad + j;
                g = *(const f32x4*)gp;
                int s = 1;
                for (; s + 3 < splits; s += 4) {
                    const f32x4 v0 = *(const f32x4*)(gp + (size_t)s * a.stride);
                    const f32x4 v1 = *(const f32x4*)(gp + (size_t)(s + 1) * a.stride);
                    const f32x4 v2 = *(const f32x4*)(gp + (size_t)(s + 2) * a.stride);
                    const f32x4 v3 = *(const f32x4*)(gp + (size_t)(s + 3) * a.stride);
                    g = (((g + v0) + v1) + v2) + v3;
                }
                for (; s < splits; ++s) g += *(const f32x4*)(gp + (size_t)s * a.stride);
            }
            apply_update4<EE>(a, j, g);
            return;
        }
        // role (1), one parameter per thread; W3/b3 are left to role (2) when it is active
        const size_t j = (size_t)b * 256 + threadIdx.x;
        const size_t limit = a.nb_l3 ? a.po.W3 : a.po.total;
        if (j >= limit) return;
        float g = 0.f;
        if (a.do_step) {
            const int splits = j < a.po.W2 ? a.splits1 : (j < a.po.W3 ? a.splits2 : a.splits3);
            g = a.grad[j];
            for (int s = 1; s < splits; ++s) g += a.grad[(size_t)s * a.stride + j];
        }
        apply_update<EE>(a, j, g);
    } else if (b < a.nb_main + a.nb_tail) {
        // [W3, total) one by one (only when role (2) is not active)
        const size_t j = a.po.W3 + (size_t)(b - a.nb_main) * 256 + threadIdx.x;
        if (j >= a.po.total) return;
        float g = 0.f;
        if (a.do_step) {
            g = a.grad[j];
            for (int s = 1; s < a.splits3; ++s) g += a.grad[(size_t)s * a.stride + j];
        }
        apply_update<EE>(a, j, g);
    } else if (b < a.nb_main + a.nb_tail + a.nb_l3) {
        // role (2): slot layout [32 classes][c2] weights, then [32] biases.  The slots were
        // written by other compute units, so every load is a round trip to memory: the role is
        // laid out for few of them.  A block takes 16 consecutive values; its 256 threads split
        // the slots into 16 contiguous runs (thread = value + 16 * run), every thread adds its
        // run in ascending order with eight loads in flight, and the 16 partial sums of a value
        // are added in the order of the runs.
        __shared__ float run_sum[16][16];
        const int kk = threadIdx.x & 15, run = threadIdx.x >> 4;
        const int k = (b - a.nb_main - a.nb_tail) * 16 + kk;
        const int n_w = a.C * a.c2;
        const bool live = k < n_w + a.C;
        float acc = 0.f;
        if (a.do_step && live) {
            const float* src = a.part3 + (k < n_w ? (size_t)k : (size_t)32 * a.c2 + (k - n_w));
            const int per = (a.blocks3 + 15) / 16;
            const int s1 = min((run + 1) * per, a.blocks3);
            int s = run * per;
            for (; s + 8 <= s1; s += 8) {
                float v[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = src[(size_t)(s + e) * a.slot3];
#pragma unroll
                for (int e = 0; e < 8; ++e) acc += v[e];
            }
            if (s < s1) {
                // the rest of the run, again loaded together (clamped re-loads count as zero)
                float v[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) v[e] = src[(size_t)min(s + e, a.blocks3 - 1) * a.slot3];
#pragma unroll
                for (int e = 0; e < 8; ++e) acc += s + e < s1 ? v[e] : 0.f;
            }
        }
        run_sum[run][kk] = acc;
        __syncthreads();
        if (run == 0 && live) {
            float total = run_sum[0][kk];
#pragma unroll
            for (int r = 1; r < 16; ++r) total += run_sum[r][kk];
            apply_update<EE>(a, a.po.W3 + k, total);
        }
    } else if (b < a.nb_main + a.nb_tail + a.nb_l3 + a.nb_finish) {
        finish_block<EE>(f, b - a.nb_main - a.nb_tail - a.nb_l3, head);
    } else {
        // parameters back to the caller's order
        const size_t j = (size_t)(b - a.nb_main - a.nb_tail - a.nb_l3 - a.nb_finish) * 256 + threadIdx.x;
        if (j < a.po.total) a.ext_out[external_index(a, j)] = a.theta[j];
    }
}

template <bool EE>
__global__ void __launch_bounds__(256) k_step_end(UpdateArgs a, FinishArgs f)
{
    step_end_block<EE>(a, f, blockIdx.x, blockIdx.y);
}

// The launch that opens a call: three kinds of blocks that do not depend on each other,
//   first   U^T of the label map and the pixel counts (label_adjoint_block),
//   then    the caller's parameters into theta and the bfloat16 operand copies: the blocks of
//           k_step_end, head by head,
//   last    feature packing (pack_features_block).
// Run one after the other they are three short launches, each of which leaves most of the chip
// idle for most of its time.
struct BeginArgs {
    const void* features; void* feat; void* featT; int in_bf16, out_bf16, PPT, guard;
    int pack_vec;                          // the 16-byte packing role over the padded grid
    int pack_x, pack_y, nb_pack;           // pack grid: pack_x column tiles x pack_y channel tiles x rows
    const int32_t* labels; const uint8_t* wmap; float* T; unsigned long long* n_valid; int CP, nb_label;
    uint8_t* lab8;                         // the labels as bytes for the loss kernel (written by the label role)
    int nb_update, nb_update_all;          // blocks of the parameter role per head, and of all heads
    Geo g;
};

__global__ void __launch_bounds__(256) k_call_begin(BeginArgs q, UpdateArgs a, FinishArgs f)
{
    extern __shared__ __attribute__((aligned(16))) float dyn_lds[];
    int b = blockIdx.x;
    // (blocks start in index order: the label blocks, each a long chain of dependent steps, go
    //  first, the short packing blocks last)
    if (b < q.nb_label) {
        float* colsum = dyn_lds;
        unsigned int* cnt_part = (unsigned int*)(dyn_lds + q.CP * (LABEL_NCOL + 1));
        label_adjoint_block(q.labels, q.wmap, q.T, q.n_valid, q.g, b, colsum, cnt_part, q.CP, q.lab8);
        return;
    }
    b -= q.nb_label;
    if (b >= q.nb_update_all) {
        b -= q.nb_update_all;
        float (*tile)[33] = (float (*)[33])dyn_lds;
        const int bx = b % q.pack_x, by = (b / q.pack_x) % q.pack_y, bz = b / (q.pack_x * q.pack_y);
        if (q.pack_vec) {
            pack_features_vec_block((const bf16*)q.features, (bf16*)q.feat, (bf16*)q.featT, q.g, q.PPT, q.guard, bx, by, bz, (bf16*)dyn_lds);
            return;
        }
        if (q.out_bf16) {
            if (q.in_bf16) pack_features_block<bf16, bf16>((const bf16*)q.features, (bf16*)q.feat, (bf16*)q.featT, q.g, q.PPT, q.guard, bx, by, bz, tile);
            else pack_features_block<float, bf16>((const float*)q.features, (bf16*)q.feat, (bf16*)q.featT, q.g, q.PPT, q.guard, bx, by, bz, tile);
        } else {
            if (q.in_bf16) pack_features_block<bf16, float>((const bf16*)q.features, (float*)q.feat, (float*)nullptr, q.g, 0, 0, bx, by, bz, tile);
            else pack_features_block<float, float>((const float*)q.features, (float*)q.feat, (float*)nullptr, q.g, 0, 0, bx, by, bz, tile);
        }
        return;
    }
    step_end_block<false>(a, f, b % q.nb_update, b / q.nb_update);
}

FinishArgs finish_args(const Plan& p, char* ws, float* loss_out, double* miou_out, long long* conf_out,
                       double* miou_host, unsigned long long* token_host, unsigned long long token)
{
    FinishArgs f;
    f.loss_part = (const float*)(ws + p.loss_part);
    f.n_part = loss_blocks(p.g);
    f.n_valid = (const unsigned long long*)(ws + p.counters);
    f.conf = (unsigned long long*)(ws + p.conf);
    f.n = p.g.n; f.C = p.g.C;
    f.fph = p.g.n / p.g.heads();
    f.pph = f.n_part / p.g.heads();
    f.loss_out = loss_out;
    f.miou_a = (double*)(ws + p.scal);   // per-frame metric kept in the workspace (host-side loop exits)
    f.miou_b = miou_out;                 // the caller's array (may be null)
    f.miou_c = miou_host;                // host memory the device can write (may be null): the loop exits read it
    f.token_c = token_host; f.token = token;
    f.conf_out = conf_out;
    return f;
}

static void head_strides(UpdateArgs& a, const Plan& p)
{
    a.hs_param = p.head_stride;
    a.hs_ext = p.po.total;
    a.hs_grad = p.grad_stride * p.grad_copies;
    a.hs_wq1 = p.po.b1 - p.po.W1;
    a.hs_wq2 = p.po.b2 - p.po.W2;
    a.hs_wq3 = p.po.b3 - p.po.W3;
    a.hs_part3 = (size_t)p.blocks3 * conv3_bwd_slot_floats(p.g);
}

// do_step: optimiser step (else only the bfloat16 copies are refreshed);
// finish: also close the forward pass that preceded it (loss, per-frame mIoU, counts)
static int step_end_args(const Plan& p, char* ws, float lr, float mu, const AdamStep* adam, bool do_step, bool finish,
                         const float* ext_in, bool w1t, const FinishArgs& f, UpdateArgs& a, float* save_old = nullptr)
{
    a.theta = (float*)(ws + p.theta);
    a.save_old = do_step ? save_old : nullptr;
    a.vel = (float*)(ws + p.vel);
    a.vel2 = (float*)(ws + p.vel2);
    a.ext_in = do_step ? nullptr : ext_in; a.ext_out = nullptr; a.nb_out = 0;
    a.adam = adam ? 1 : 0;
    if (adam) a.ad = *adam; else memset(&a.ad, 0, sizeof(a.ad));
    a.grad = (const float*)(ws + p.grad);
    a.stride = p.grad_stride;
    a.splits1 = p.splits1;
    a.splits2 = p.splits2;
    a.splits3 = p.splits3;
    a.wq1 = p.bf16 ? (bf16*)(ws + p.wq1) : nullptr;
    a.wq1t = (p.mfma && w1t) ? (bf16*)(ws + p.wq1t) : nullptr;
    a.wq2 = p.bf16 ? (bf16*)(ws + p.wq2) : nullptr;
    a.wq2t = (p.bf16 && p.wq2t) ? (bf16*)(ws + p.wq2t) : nullptr;
    a.wq3 = p.bf16 ? (bf16*)(ws + p.wq3) : nullptr;
    a.wq3t = p.wq3t ? (bf16*)(ws + p.wq3t) : nullptr;
    a.po = p.po; a.c_in = p.g.c_in; a.c1 = p.g.c1; a.c2 = p.g.c2;
    a.frag = p.mfma ? 1 : 0;
    a.lr = lr; a.mu = mu; a.do_step = do_step ? 1 : 0;
    a.part3 = (const float*)(ws + p.grad3);
    a.blocks3 = p.blocks3; a.slot3 = conv3_bwd_slot_floats(p.g); a.C = p.g.C;
    const bool params = do_step || p.bf16 || a.ext_in;
    const bool l3 = params && p.mfma && do_step;
    // four parameters per thread when every block below W3 starts at a multiple of four and the
    // split copies keep 16-byte alignment
    a.vec = (p.po.b1 % 4 == 0 && p.po.W2 % 4 == 0 && p.po.b2 % 4 == 0 && p.po.W3 % 4 == 0) ? 1 : 0;
    if (a.vec) {
        a.nb_main = params ? cdiv(p.po.W3 / 4, 256) : 0;
        a.nb_tail = (params && !l3) ? cdiv(p.po.total - p.po.W3, 256) : 0;
    } else {
        a.nb_main = params ? cdiv(l3 ? p.po.W3 : p.po.total, 256) : 0;
        a.nb_tail = 0;
    }
    a.nb_l3 = l3 ? cdiv(p.g.C * p.g.c2 + p.g.C, 16) : 0;
    a.nb_finish = finish ? f.fph + 1 : 0;
    head_strides(a, p);
    return a.nb_main + a.nb_tail + a.nb_l3 + a.nb_finish;
}

void step_end(Ctx& c, const Plan& p, char* ws, float lr, float mu, const AdamStep* adam, bool do_step, bool finish, float* loss_out,
              double* miou_out, long long* conf_out, const float* ext_in, bool w1t, float* save_old)
{
    UpdateArgs a;
    const FinishArgs f = finish_args(p, ws, loss_out, miou_out, conf_out);
    const int blocks = step_end_args(p, ws, lr, mu, adam, do_step, finish, ext_in, w1t, f, a, save_old);
    if (blocks == 0) return;
    const bool params = do_step || p.bf16 || a.ext_in;
    const char* name = a.ext_in ? "params_in+weights_to_bf16" : do_step ? (adam ? (finish ? "adam_update+finish_pass" : "adam_update") : (finish ? "sgd_update+finish_pass" : "sgd_update")) : (params ? "weights_to_bf16" : "finish_pass");
    if (a.save_old) ST_LAUNCH(c, name, k_step_end<true>, dim3(blocks, p.g.heads()), dim3(256), 0, a, f);
    else ST_LAUNCH(c, name, k_step_end<false>, dim3(blocks, p.g.heads()), dim3(256), 0, a, f);
}

// Whether the packing role of the call-opening launch writes the whole padded grid of both feature
// buffers (then only their guards need clearing): matrix-core path, bfloat16 features whose rows
// are multiples of 16 bytes from a 16-byte aligned start, in the [n, c_in, h, w] order.
bool pack_covers_borders(const Plan& p, const void* features, int feat_dtype)
{
    return p.mfma && !p.g.nhwc && feat_dtype == ST_BF16 && p.g.w % 8 == 0 && p.g.c_in % 64 == 0 &&
           ((uintptr_t)features & 15) == 0;
}

// Opens a call in one launch: packs the features, takes the caller's parameters (OIHW order)
// into theta and the bfloat16 copies and, with labels, computes T = U^T (one-hot valid labels)
// and the pixel counts (n_valid must be clear).  The workspace must have been cleared before.
void call_begin(Ctx& c, const Plan& p, char* ws, const void* features, int feat_dtype, const float* head_params,
                bool w1t, const int32_t* labels, const uint8_t* wmap)
{
    const Geo& g = p.g;
    BeginArgs q;
    memset(&q, 0, sizeof(q));
    q.features = features; q.feat = ws + p.feat;
    q.featT = (p.bf16 && p.featT) ? ws + p.featT : nullptr;
    q.in_bf16 = feat_dtype == ST_BF16; q.out_bf16 = p.bf16 ? 1 : 0;
    q.PPT = p.PPT; q.guard = p.guard;
    q.pack_vec = pack_covers_borders(p, features, feat_dtype) ? 1 : 0;
    if (q.pack_vec) {
        q.pack_x = cdiv(g.Wp, 64); q.pack_y = g.c_in / 64;
        q.nb_pack = q.pack_x * q.pack_y * g.n * g.Hp;
    } else {
        q.pack_x = cdiv(g.w, 32); q.pack_y = cdiv(g.c_in, 32);
        q.nb_pack = q.pack_x * q.pack_y * g.n * g.h;
    }
    q.g = g;
    q.CP = (g.C + 3) / 4 * 4;
    if (labels) {
        q.labels = labels; q.wmap = wmap; q.T = (float*)(ws + p.tadj); q.lab8 = (uint8_t*)(ws + p.lab8);
        q.n_valid = (unsigned long long*)(ws + p.counters);
        q.nb_label = g.n * g.h * cdiv(g.w, LABEL_TX);
    }
    UpdateArgs a;
    const FinishArgs f = finish_args(p, ws, nullptr, nullptr, nullptr);
    q.nb_update = step_end_args(p, ws, 0.f, 0.f, nullptr, false, false, head_params, w1t, f, a);
    q.nb_update_all = q.nb_update * g.heads();
    const size_t lds = std::max(std::max((size_t)32 * 33 * sizeof(float), (size_t)64 * PACKV_PITCH * sizeof(bf16)),
                                (size_t)(q.CP * (LABEL_NCOL + 1) + 4) * sizeof(float));
    ST_LAUNCH(c, labels ? "pack+label_adjoint+params_in" : "pack+params_in", k_call_begin,
              dim3(q.nb_pack + q.nb_label + q.nb_update * g.heads()), dim3(256), lds, q, a, f);
}

// bookkeeping of a pass without an update; with ext_out the same launch hands theta back to the
// caller's vector (OIHW order)
void finish_pass(Ctx& c, const Plan& p, char* ws, float* loss_out, double* miou_out, long long* conf_out,
                 float* ext_out, double* miou_host, unsigned long long* token_host, unsigned long long token)
{
    UpdateArgs a;
    memset(&a, 0, sizeof(a));
    const FinishArgs f = finish_args(p, ws, loss_out, miou_out, conf_out, miou_host, token_host, token);
    a.nb_finish = f.fph + 1;
    head_strides(a, p);
    if (ext_out) {
        a.theta = (float*)(ws + p.theta);
        a.po = p.po; a.c_in = p.g.c_in; a.c1 = p.g.c1; a.c2 = p.g.c2;
        a.ext_out = ext_out;
        a.nb_out = cdiv(p.po.total, 256);
    }
    if (miou_host)
        ST_LAUNCH(c, ext_out ? "finish_pass+params_out" : "finish_pass", k_step_end<true>,
                  dim3(a.nb_finish + a.nb_out, p.g.heads()), dim3(256), 0, a, f);
    else
        ST_LAUNCH(c, ext_out ? "finish_pass+params_out" : "finish_pass", k_step_end<false>,
                  dim3(a.nb_finish + a.nb_out, p.g.heads()), dim3(256), 0, a, f);
}

// Mean IoU (Eq. 1) of a C x C table of counts, any C up to 256: one wavefront per class adds
// that class's row and column (exact integer sums), then a single thread adds the per-class
// ratios of the classes that occur as a label in ascending order in float64 and divides by
// their number; 0 when there is none.
constexpr int MIOU_THREADS = 1024;
__global__ void __launch_bounds__(MIOU_THREADS)
k_miou_from_counts(const unsigned long long* __restrict__ conf, int C, double* __restrict__ out)
{
    __shared__ double iou[256];
    __shared__ int present[256];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int c = wave; c < C; c += MIOU_THREADS / 64) {
        unsigned long long row = 0, col = 0;
        for (int k = lane; k < C; k += 64) { row += conf[(size_t)c * C + k]; col += conf[(size_t)k * C + c]; }
#pragma unroll
        for (int d = 32; d; d >>= 1) { row += __shfl_xor(row, d, 64); col += __shfl_xor(col, d, 64); }
        if (lane == 0) {
            const unsigned long long inter = conf[(size_t)c * C + c];
            present[c] = row != 0;
            iou[c] = row ? (double)inter / (double)(row + col - inter) : 0.0;
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        double sum = 0.0;
        int cnt = 0;
        for (int c = 0; c < C; ++c)
            if (present[c]) { sum += iou[c]; ++cnt; }
        *out = cnt ? sum / cnt : 0.0;
    }
}

// ------------------------------------------------------------------ stand-alone metric
// Confusion counts of a class map against labels.  Each block keeps its own C x C table in
// LDS and adds it to the result at the end; integer counts, so the order of additions does
// not matter.  Few, large blocks: the final additions of every block land on the same few
// cache lines.  Per trip a wavefront takes 1024 consecutive pixels as four label loads of 16
// bytes and four prediction loads of 4 bytes per lane, each instruction reading one contiguous
// stretch, all issued before the first is used.  Label maps are piecewise constant, so most
// wavefronts hold a single (label, prediction) pair: that case is detected with one ballot and
// costs one LDS addition.  Otherwise every lane merges equal neighbours among its 16 pixels
// and adds each run to the table itself; LDS resolves lanes that hit the same counter.
// Tables too large for LDS (more than 128 classes) go to the result directly, one addition
// per distinct pair of a wavefront and pixel slot.
constexpr int CONF_THREADS = 1024;
constexpr int CONF_PER_T = 16;                       // pixels of one thread per trip
constexpr int CONF_MAX_BLOCKS = 256;
template <bool LDS_TABLE>
__global__ void __launch_bounds__(CONF_THREADS)
k_confusion(const uint8_t* __restrict__ pred, const int32_t* __restrict__ labels, long long P, int C,
            int ignore, unsigned long long* __restrict__ conf)
{
    extern __shared__ unsigned int table[];
    if (LDS_TABLE) {
        for (int i = threadIdx.x; i < C * C; i += CONF_THREADS) table[i] = 0;
        __syncthreads();
    }
    const bool aligned = (((uintptr_t)labels | (uintptr_t)pred) & 15) == 0;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const long long trip = (long long)CONF_THREADS * CONF_PER_T;
    for (long long first = (long long)blockIdx.x * trip; first < P; first += (long long)gridDim.x * trip) {
        // pixel (k, j) of this lane: wbase + 256 k + 4 lane + j
        const long long wbase = first + (long long)wave * (64 * CONF_PER_T);
        if (wbase >= P) continue;
        int bins[CONF_PER_T];
        if (aligned && wbase + 64 * CONF_PER_T <= P) {
            u32x4 lv[4];
            unsigned int pv[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) lv[k] = *(const u32x4*)(labels + wbase + 256 * k + 4 * lane);
#pragma unroll
            for (int k = 0; k < 4; ++k) pv[k] = *(const unsigned int*)(pred + wbase + 256 * k + 4 * lane);
#pragma unroll
            for (int i = 0; i < CONF_PER_T; ++i) {
                const int y = (int)lv[i >> 2][i & 3];
                const int q = (int)((pv[i >> 2] >> (8 * (i & 3))) & 0xFFu);
                bins[i] = (y != ignore && y >= 0 && y < C && q < C) ? y * C + q : -1;
            }
        } else {
#pragma unroll
            for (int i = 0; i < CONF_PER_T; ++i) {
                const long long at = wbase + 256 * (i >> 2) + 4 * lane + (i & 3);
                bins[i] = -1;
                if (at < P) {
                    const int y = labels[at];
                    const int q = pred[at];
                    if (y != ignore && y >= 0 && y < C && q < C) bins[i] = y * C + q;
                }
            }
        }
        if (LDS_TABLE) {
            const int b0 = __builtin_amdgcn_readfirstlane(bins[0]);
            bool same = true;
#pragma unroll
            for (int i = 0; i < CONF_PER_T; ++i) same &= bins[i] == b0;
            if (__ballot(same) == __ballot(true)) {
                // one pair for the whole wavefront (or nothing to count)
                if (b0 >= 0 && lane == 0) atomicAdd(&table[b0], 64u * CONF_PER_T);
            } else {
                unsigned int run = 1;
#pragma unroll
                for (int i = 1; i <= CONF_PER_T; ++i) {
                    if (i < CONF_PER_T && bins[i] == bins[i - 1]) { ++run; continue; }
                    if (bins[i - 1] >= 0) atomicAdd(&table[bins[i - 1]], run);
                    run = 1;
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < CONF_PER_T; ++i) {
                const int bin = bins[i];
                unsigned long long todo = __ballot(bin >= 0);
                while (todo) {
                    const int leader = __ffsll((long long)todo) - 1;
                    const int lbin = __shfl(bin, leader, 64);
                    const unsigned long long same = __ballot(bin == lbin);
                    if (lane == leader) atomicAdd(&conf[lbin], (unsigned long long)__popcll(same));
                    todo &= ~same;
                }
            }
        }
    }
    if (LDS_TABLE) {
        __syncthreads();
        for (int i = threadIdx.x; i < C * C; i += CONF_THREADS)
            if (table[i]) atomicAdd(&conf[i], (unsigned long long)table[i]);
    }
}

void confusion_and_miou(Ctx& c, const uint8_t* pred, const int32_t* labels, long long P, int C, int ignore,
                        long long* conf, double* miou)
{
    zero_u64(c, (unsigned long long*)conf, (size_t)C * C);
    const int blocks = std::min(std::max(cdiv(P, CONF_THREADS * CONF_PER_T), 1), CONF_MAX_BLOCKS);
    const size_t lds = (size_t)C * C * 4;
    if (lds <= 64 * 1024)
        ST_LAUNCH(c, "confusion", (k_confusion<true>), dim3(blocks), dim3(CONF_THREADS), lds, pred, labels, P, C, ignore,
                  (unsigned long long*)conf);
    else
        ST_LAUNCH(c, "confusion", (k_confusion<false>), dim3(blocks), dim3(CONF_THREADS), 0, pred, labels, P, C, ignore,
                  (unsigned long long*)conf);
    ST_LAUNCH(c, "miou", k_miou_from_counts, dim3(1), dim3(MIOU_THREADS), 0, (const unsigned long long*)conf, C, miou);
}

}  // namespace st

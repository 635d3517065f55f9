// Optimiser step over the flat parameter buffer (fused with the sum of the partial weight
// gradients and the bfloat16 operand copies of the new weights), the per-step bookkeeping
// kernel (loss, per-frame mean IoU) and the stand-alone confusion-matrix / mean-IoU kernels.
#include "st_kernels.hpp"

namespace st {

// theta <- theta - lr * v,  v <- mu * v + g  (mu == 0: v is not touched).  g is the sum, in
// ascending order, of the partial gradients the backward kernels left behind: `splits1` copies
// for W1/b1 and `splits2` for W2/b2 (position splits of the weight-gradient kernels, `stride`
// floats apart); W3/b3 sit in copy 0 (k_reduce3 has already added their per-block slots).
// Also refreshes the bfloat16 copies of the new weights:
//   wq1, wq2, wq3 : same (internal) order as theta, for the forward convolutions
//   wq2t          : W2 as [i][tap'][o] with tap' the mirrored tap, for the data-gradient of layer 2
struct UpdateArgs {
    float* theta; float* vel; const float* grad; size_t stride; int splits1, splits2;
    bf16* wq1; bf16* wq2; bf16* wq2t; bf16* wq3;
    ParamOffsets po; int c1, c2;
    float lr, mu;
    int do_step;   // 0: only refresh the bfloat16 copies
};

__global__ void __launch_bounds__(256) k_update(UpdateArgs a)
{
    const size_t j = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (j >= a.po.total) return;
    float w = a.theta[j];
    if (a.do_step) {
        const int splits = j < a.po.W2 ? a.splits1 : (j < a.po.W3 ? a.splits2 : 1);
        float g = a.grad[j];
        for (int s = 1; s < splits; ++s) g += a.grad[(size_t)s * a.stride + j];
        if (a.mu != 0.f) {
            const float v = __builtin_fmaf(a.mu, a.vel[j], g);
            a.vel[j] = v;
            g = v;
        }
        w = __builtin_fmaf(-a.lr, g, w);
        a.theta[j] = w;
    }
    if (a.wq1) {
        const bf16 q = (bf16)w;
        if (j < a.po.b1) a.wq1[j - a.po.W1] = q;
        else if (j >= a.po.W2 && j < a.po.b2) {
            const size_t r = j - a.po.W2;
            a.wq2[r] = q;
            if (a.wq2t) {
                const size_t i = r % a.c1, tap = (r / a.c1) % 9, o = r / ((size_t)a.c1 * 9);
                a.wq2t[(i * 9 + (8 - tap)) * a.c2 + o] = q;
            }
        } else if (j >= a.po.W3 && j < a.po.b3) a.wq3[j - a.po.W3] = q;
    }
}

void update_params(Ctx& c, const Plan& p, char* ws, float lr, float mu, bool do_step)
{
    UpdateArgs a;
    a.theta = (float*)(ws + p.theta);
    a.vel = (float*)(ws + p.vel);
    a.grad = (const float*)(ws + p.grad);
    a.stride = p.po.total;
    a.splits1 = p.mfma ? p.splits1 : 1;
    a.splits2 = p.mfma ? p.splits2 : 1;
    a.wq1 = p.bf16 ? (bf16*)(ws + p.wq1) : nullptr;
    a.wq2 = p.bf16 ? (bf16*)(ws + p.wq2) : nullptr;
    a.wq2t = (p.bf16 && p.wq2t) ? (bf16*)(ws + p.wq2t) : nullptr;
    a.wq3 = p.bf16 ? (bf16*)(ws + p.wq3) : nullptr;
    a.po = p.po; a.c1 = p.g.c1; a.c2 = p.g.c2;
    a.lr = lr; a.mu = mu; a.do_step = do_step ? 1 : 0;
    if (!do_step && !p.bf16) return;
    ST_LAUNCH(c, do_step ? "sgd_update" : "weights_to_bf16", k_update, dim3(cdiv(p.po.total, 256)), dim3(256),
              0, a);
}

// ------------------------------------------------------------------ mean IoU from counts
// IoU_c = conf[c][c] / (row_c + col_c - conf[c][c]) for classes with row_c > 0, summed in
// ascending c in float64, divided by their number; 0 when no class is present.
__device__ double miou_of(const unsigned long long* conf, int C)
{
    double sum = 0.0;
    int present = 0;
    for (int c = 0; c < C; ++c) {
        unsigned long long row = 0, col = 0;
        for (int k = 0; k < C; ++k) { row += conf[c * C + k]; col += conf[k * C + c]; }
        if (row == 0) continue;
        const unsigned long long inter = conf[c * C + c];
        sum += (double)inter / (double)(row + col - inter);
        ++present;
    }
    return present ? sum / present : 0.0;
}

// Sum of the per-block slots of the classifier layer's backward kernel into gradient copy 0.
// One wavefront per parameter: lane l adds slots l, l+64, ... in order, then the 64 lane sums
// are added by a fixed shuffle tree.
__global__ void __launch_bounds__(256)
k_reduce3(const float* __restrict__ part, int blocks, size_t slot, float* __restrict__ gW3,
          float* __restrict__ gb3, int C, int c2)
{
    const int lane = threadIdx.x & 63;
    const int j = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int n_w = C * c2;
    if (j >= n_w + C) return;
    const size_t r = j < n_w ? (size_t)j : (size_t)32 * c2 + (j - n_w);   // slot: [32][c2] weights, [32] biases
    float acc = 0.f;
    for (int s = lane; s < blocks; s += 64) acc += part[(size_t)s * slot + r];
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_down(acc, off, 64);
    if (lane == 0) {
        if (j < n_w) gW3[j] = acc;
        else gb3[j - n_w] = acc;
    }
}

void reduce_grad3(Ctx& c, const Plan& p, char* ws)
{
    float* grad = (float*)(ws + p.grad);
    const int n = p.g.C * p.g.c2 + p.g.C;
    ST_LAUNCH(c, "reduce_grad3", k_reduce3, dim3(cdiv(n, 4)), dim3(256), 0, (const float*)(ws + p.grad3),
              p.blocks3, conv3_bwd_slot_floats(p.g), grad + p.po.W3, grad + p.po.b3, p.g.C, p.g.c2);
}

// Closes a forward pass.  Block f < n: mean IoU of frame f from its confusion counts (copied out
// when asked, then cleared for the next pass).  Block n: the tile losses added in a fixed order
// (float64) and divided by the number of valid pixels.
__global__ void __launch_bounds__(256)
k_finish_pass(const float* __restrict__ loss_part, int n_part, const unsigned long long* __restrict__ n_valid,
              unsigned long long* __restrict__ conf, int n, int C, float* loss_out, double* miou_a,
              double* miou_b, long long* conf_out)
{
    __shared__ double part[256];
    __shared__ unsigned long long cl[32 * 32];
    __shared__ double iou[32];
    __shared__ int present[32];
    const int tid = threadIdx.x;
    if ((int)blockIdx.x == n) {
        double acc = 0.0;
        const int per = (n_part + 255) / 256;
        for (int i = tid * per; i < min(n_part, (tid + 1) * per); ++i) acc += (double)loss_part[i];
        part[tid] = acc;
        __syncthreads();
        for (int s = 128; s > 0; s >>= 1) {
            if (tid < s) part[tid] += part[tid + s];
            __syncthreads();
        }
        if (tid == 0 && loss_out) {
            const unsigned long long nv = *n_valid;
            *loss_out = nv ? (float)(part[0] / (double)nv) : 0.f;
        }
        return;
    }
    const int f = blockIdx.x;
    unsigned long long* cf = conf + (size_t)f * C * C;
    for (int i = tid; i < C * C; i += 256) {
        const unsigned long long v = cf[i];
        cl[i] = v;
        if (conf_out) conf_out[(size_t)f * C * C + i] = (long long)v;
        cf[i] = 0ull;
    }
    __syncthreads();
    if (tid < C) {
        unsigned long long row = 0, col = 0;
        for (int k = 0; k < C; ++k) { row += cl[tid * C + k]; col += cl[k * C + tid]; }
        const unsigned long long inter = cl[tid * C + tid];
        present[tid] = row != 0;
        iou[tid] = row ? (double)inter / (double)(row + col - inter) : 0.0;
    }
    __syncthreads();
    if (tid == 0) {
        double sum = 0.0;
        int cnt = 0;
        for (int c = 0; c < C; ++c)
            if (present[c]) { sum += iou[c]; ++cnt; }
        const double m = cnt ? sum / cnt : 0.0;
        if (miou_a) miou_a[f] = m;
        if (miou_b) miou_b[f] = m;
    }
}

// miou_ws: per-frame metric kept in the workspace (for the host-side loop exits);
// miou_out: the caller's array (may be null)
void finish_pass(Ctx& c, const Plan& p, char* ws, float* loss_out, double* miou_out, long long* conf_out)
{
    ST_LAUNCH(c, "finish_pass", k_finish_pass, dim3(p.g.n + 1), dim3(256), 0, (const float*)(ws + p.loss_part),
              loss_blocks(p.g), (const unsigned long long*)(ws + p.counters),
              (unsigned long long*)(ws + p.conf), p.g.n, p.g.C, loss_out, (double*)(ws + p.scal), miou_out,
              conf_out);
}

// ------------------------------------------------------------------ stand-alone metric
// Confusion counts of a class map against labels.  Each block keeps its own C x C table in
// LDS.  Label maps are piecewise constant, so most wavefronts hold a single (label, prediction)
// pair: the wavefront first agrees on one bin by ballot and a single lane adds the population
// count; the few mixed wavefronts repeat that for each distinct bin.  Integer counts, so the
// order of additions does not matter.
template <bool LDS_TABLE>
__global__ void __launch_bounds__(256)
k_confusion(const uint8_t* __restrict__ pred, const int32_t* __restrict__ labels, long long P, int C,
            int ignore, unsigned long long* __restrict__ conf)
{
    extern __shared__ unsigned int table[];
    if (LDS_TABLE) {
        for (int i = threadIdx.x; i < C * C; i += 256) table[i] = 0;
        __syncthreads();
    }
    const long long stride = (long long)gridDim.x * 256;
    const long long n_iter = (P + stride - 1) / stride;
    for (long long it = 0; it < n_iter; ++it) {
        const long long i = it * stride + (long long)blockIdx.x * 256 + threadIdx.x;
        int bin = -1;
        if (i < P) {
            const int y = labels[i];
            const int q = pred[i];
            if (y != ignore && y >= 0 && y < C && q < C) bin = y * C + q;
        }
        // wavefront-level aggregation
        unsigned long long todo = __ballot(bin >= 0);
        while (todo) {
            const int leader = __ffsll((long long)todo) - 1;
            const int lbin = __shfl(bin, leader, 64);
            const unsigned long long same = __ballot(bin == lbin);
            if ((int)(threadIdx.x & 63) == leader) {
                const unsigned int cnt = (unsigned int)__popcll(same);
                if (LDS_TABLE) atomicAdd(&table[lbin], cnt);
                else atomicAdd(&conf[lbin], (unsigned long long)cnt);
            }
            todo &= ~same;
        }
    }
    if (LDS_TABLE) {
        __syncthreads();
        for (int i = threadIdx.x; i < C * C; i += 256)
            if (table[i]) atomicAdd(&conf[i], (unsigned long long)table[i]);
    }
}

__global__ void k_miou_single(const unsigned long long* conf, int C, double* out)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) *out = miou_of(conf, C);
}

void confusion_and_miou(Ctx& c, const uint8_t* pred, const int32_t* labels, long long P, int C, int ignore,
                        long long* conf, double* miou)
{
    zero_u64(c, (unsigned long long*)conf, (size_t)C * C);
    int blocks = cdiv(P, 256 * 16);
    if (blocks < 1) blocks = 1;
    if (blocks > 2048) blocks = 2048;
    const size_t lds = (size_t)C * C * 4;
    if (lds <= 64 * 1024)
        ST_LAUNCH(c, "confusion", (k_confusion<true>), dim3(blocks), dim3(256), lds, pred, labels, P, C, ignore,
                  (unsigned long long*)conf);
    else
        ST_LAUNCH(c, "confusion", (k_confusion<false>), dim3(blocks), dim3(256), 0, pred, labels, P, C, ignore,
                  (unsigned long long*)conf);
    ST_LAUNCH(c, "miou", k_miou_single, dim3(1), dim3(64), 0, (const unsigned long long*)conf, C, miou);
}

}  // namespace st

// Plain tiled GEMM kernels for every contraction of the head (forward, data-gradient and
// weight-gradient of the 3x3 and 1x1 convolutions), templated on the element type of the
// activations and weights.  With float elements this is the reference-precision path; with
// bfloat16 elements it computes what the matrix-core kernels compute (bf16 x bf16 products are
// exact in float32, sums in float32) and serves shapes those kernels do not cover.
//
//   C[m][n] = sum_k A(m, k) * B(k, n),   64 x 64 tile per block, 4 x 4 per thread, K step 16.
//
// Each problem is a small struct that says where A(m,k) and B(k,n) live -- as the sum of an offset
// that depends on the row and one that depends on k -- and where to store.
#include <algorithm>

#include "st_kernels.hpp"

namespace st {

constexpr int GB = 64, GK = 16;

template <class Prob>
__global__ void __launch_bounds__(256) k_gemm_generic(Prob p)
{
    __shared__ float As[GK][GB + 4];
    __shared__ float Bs[GK][GB + 4];
    const int tid = threadIdx.x;
    const int m0 = blockIdx.x * GB, n0 = blockIdx.y * GB;
    const int tm = (tid / 16) * 4, tn = (tid % 16) * 4;
    const int M = p.M(), N = p.N();
    // blockIdx.z: a share of the reduction range, in whole K steps (weight gradients are split over
    // the positions, each share goes to a partial copy of its own; everything else has one share)
    const int k_steps = (p.K() + GK - 1) / GK;
    const int per = (k_steps + (int)gridDim.z - 1) / (int)gridDim.z;
    const int k_begin = (int)blockIdx.z * per * GK, K = min(p.K(), ((int)blockIdx.z + 1) * per * GK);

    // A thread stages four elements of each operand per K step.  An element's address is the sum
    // of a part that depends on the row (m or n) and a part that depends on k; the thread's rows
    // never change, so their parts are computed once, and of the k parts only what the step needs.
    //   K_FAST operand: one k (tid % GK), four rows (tid / GK + 16 r)
    //   otherwise:      one row (tid % GB), four k (tid / GB + 4 r)
    const int a_kk = Prob::A_K_FAST ? tid % GK : tid / GB, a_mm = Prob::A_K_FAST ? tid / GK : tid % GB;
    const int b_kk = Prob::B_K_FAST ? tid % GK : tid / GB, b_nn = Prob::B_K_FAST ? tid / GK : tid % GB;
    long a_row[4], b_row[4];
    bool a_in[4], b_in[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        const int mm = a_mm + (Prob::A_K_FAST ? 16 * r : 0), nn = b_nn + (Prob::B_K_FAST ? 16 * r : 0);
        a_in[r] = m0 + mm < M;
        b_in[r] = n0 + nn < N;
        a_row[r] = a_in[r] ? p.am(m0 + mm) : 0;
        b_row[r] = b_in[r] ? p.bn(n0 + nn) : 0;
    }
    float ra[4], rb[4];
    // the elements of the step that starts at k0, into registers
    auto fetch = [&](int k0) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int ka = k0 + a_kk + (Prob::A_K_FAST ? 0 : 4 * r), kb = k0 + b_kk + (Prob::B_K_FAST ? 0 : 4 * r);
            ra[r] = (a_in[r] && ka < K) ? p.a_ld(a_row[r] + p.ak(ka)) : 0.f;
            rb[r] = (b_in[r] && kb < K) ? p.b_ld(b_row[r] + p.bk(kb)) : 0.f;
        }
    };
    float acc[4][4] = {};
    if (k_begin < K) fetch(k_begin);
    for (int k0 = k_begin; k0 < K; k0 += GK) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            As[a_kk + (Prob::A_K_FAST ? 0 : 4 * r)][a_mm + (Prob::A_K_FAST ? 16 * r : 0)] = ra[r];
            Bs[b_kk + (Prob::B_K_FAST ? 0 : 4 * r)][b_nn + (Prob::B_K_FAST ? 16 * r : 0)] = rb[r];
        }
        __syncthreads();
        // the next step's elements travel while this one is multiplied
        if (k0 + GK < K) fetch(k0 + GK);
#pragma unroll
        for (int kk = 0; kk < GK; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = As[kk][tm + i]; b[i] = Bs[kk][tn + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (m0 + tm + i < M && n0 + tn + j < N) p.store(m0 + tm + i, n0 + tn + j, acc[i][j], (int)blockIdx.z);
}

// position index m in [0, n*h*w) -> padded position (img, y + 1 + dy, x + 1 + dx)
__device__ __forceinline__ int padded_pos(const Geo& g, int m, int dy, int dx)
{
    const int hw = g.h * g.w;
    const int img = m / hw, r = m - img * hw;
    const int y = r / g.w, x = r - y * g.w;
    return (img * g.Hp + y + 1 + dy) * g.Wp + x + 1 + dx;
}

// ---- forward: y[pos][o] = act( b[o] + sum_{tap,i} x[pos + tap][i] * W[o][tap][i] ) ----------
template <class E, class WE, int TAPS>
struct FwdProb {
    static constexpr bool A_K_FAST = true, B_K_FAST = true;
    Geo g; int ci, co, relu;
    const E* x; const WE* W; const float* bias; E* y;
    __device__ int M() const { return g.positions(); }
    __device__ int N() const { return co; }
    __device__ int K() const { return TAPS * ci; }
    __device__ long am(int m) const { return (long)padded_pos(g, m, 0, 0) * ci; }
    __device__ long ak(int k) const
    {
        const int tap = k / ci, i = k - tap * ci;
        const int dy = TAPS == 9 ? tap / 3 - 1 : 0, dx = TAPS == 9 ? tap % 3 - 1 : 0;
        return (long)(dy * g.Wp + dx) * ci + i;
    }
    __device__ float a_ld(long at) const { return to_f32(x[at]); }
    __device__ long bn(int n) const { return (long)n * TAPS * ci; }
    __device__ long bk(int k) const { return k; }
    __device__ float b_ld(long at) const { return to_f32(W[at]); }
    __device__ void store(int m, int n, float v, int) const
    {
        v += bias[n];
        if (relu) v = fmaxf(v, 0.f);
        y[(size_t)padded_pos(g, m, 0, 0) * co + n] = from_f32<E>(v);
    }
};

// ---- data gradient: dx[pos][i] = [act[pos][i] > 0] * sum_{tap,o} dy[pos - tap][o] * W[o][tap][i]
template <class E, class WE>
struct DgradProb {
    static constexpr bool A_K_FAST = true, B_K_FAST = false;
    Geo g; int ci, co;
    const E* dy; const WE* W; const E* act; E* dx;
    __device__ int M() const { return g.positions(); }
    __device__ int N() const { return ci; }
    __device__ int K() const { return 9 * co; }
    __device__ long am(int m) const { return (long)padded_pos(g, m, 0, 0) * co; }
    __device__ long ak(int k) const
    {
        const int tap = k / co, o = k - tap * co;
        return (long)((1 - tap / 3) * g.Wp + (1 - tap % 3)) * co + o;
    }
    __device__ float a_ld(long at) const { return to_f32(dy[at]); }
    __device__ long bn(int n) const { return n; }
    __device__ long bk(int k) const
    {
        const int tap = k / co, o = k - tap * co;
        return ((long)o * 9 + tap) * ci;
    }
    __device__ float b_ld(long at) const { return to_f32(W[at]); }
    __device__ void store(int m, int n, float v, int) const
    {
        const size_t at = (size_t)padded_pos(g, m, 0, 0) * ci + n;
        dx[at] = from_f32<E>(to_f32(act[at]) > 0.f ? v : 0.f);
    }
};

// ---- data gradient of layer 1, straight into the caller's float32 NCHW tensor (no activation in
//      front of the features, so nothing gates it) ---------------------------------------------
template <class E, class WE>
struct FeatDgradProb {
    static constexpr bool A_K_FAST = true, B_K_FAST = false;
    Geo g; int ci, co;
    const E* dy; const WE* W; float* dfeat;
    __device__ int M() const { return g.positions(); }
    __device__ int N() const { return ci; }
    __device__ int K() const { return 9 * co; }
    __device__ long am(int m) const { return (long)padded_pos(g, m, 0, 0) * co; }
    __device__ long ak(int k) const
    {
        const int tap = k / co, o = k - tap * co;
        return (long)((1 - tap / 3) * g.Wp + (1 - tap % 3)) * co + o;
    }
    __device__ float a_ld(long at) const { return to_f32(dy[at]); }
    __device__ long bn(int n) const { return n; }
    __device__ long bk(int k) const
    {
        const int tap = k / co, o = k - tap * co;
        return ((long)o * 9 + tap) * ci;
    }
    __device__ float b_ld(long at) const { return to_f32(W[at]); }
    __device__ void store(int m, int n, float v, int) const
    {
        const int hw = g.h * g.w;
        const int img = m / hw, r = m - img * hw;
        dfeat[((size_t)img * ci + n) * hw + r] = v;
    }
};

// ---- weight gradient: dW[o][tap][i] = sum_pos dy[pos][o] * x[pos + tap][i] -------------------
template <class E, int TAPS>
struct WgradProb {
    static constexpr bool A_K_FAST = false, B_K_FAST = false;
    Geo g; int ci, co;
    const E* dy; const E* x; float* dW; size_t copy_stride;
    __device__ int M() const { return co; }
    __device__ int N() const { return TAPS * ci; }
    __device__ int K() const { return g.positions(); }
    __device__ long am(int m) const { return m; }
    __device__ long ak(int k) const { return (long)padded_pos(g, k, 0, 0) * co; }
    __device__ float a_ld(long at) const { return to_f32(dy[at]); }
    __device__ long bn(int n) const
    {
        const int tap = n / ci, i = n - tap * ci;
        const int dyy = TAPS == 9 ? tap / 3 - 1 : 0, dxx = TAPS == 9 ? tap % 3 - 1 : 0;
        return (long)(dyy * g.Wp + dxx) * ci + i;
    }
    __device__ long bk(int k) const { return (long)padded_pos(g, k, 0, 0) * ci; }
    __device__ float b_ld(long at) const { return to_f32(x[at]); }
    __device__ void store(int m, int n, float v, int share) const { dW[share * copy_stride + (size_t)m * TAPS * ci + n] = v; }
};

// ---- last layer (1x1) with planar float32 logits / logit gradients ---------------------------
// z[img][c][pos] = b3[c] + sum_o a2[pos][o] * W3[c][o]
template <class E, class WE>
struct LogitsProb {
    static constexpr bool A_K_FAST = true, B_K_FAST = true;
    Geo g; const E* a2; const WE* W3; const float* b3; float* z;
    __device__ int M() const { return g.positions(); }
    __device__ int N() const { return g.C; }
    __device__ int K() const { return g.c2; }
    __device__ long am(int m) const { return (long)padded_pos(g, m, 0, 0) * g.c2; }
    __device__ long ak(int k) const { return k; }
    __device__ float a_ld(long at) const { return to_f32(a2[at]); }
    __device__ long bn(int n) const { return (long)n * g.c2; }
    __device__ long bk(int k) const { return k; }
    __device__ float b_ld(long at) const { return to_f32(W3[at]); }
    __device__ void store(int m, int n, float v, int) const
    {
        const int hw = g.h * g.w, img = m / hw, r = m - img * hw;
        z[((size_t)img * g.C + n) * hw + r] = v + b3[n];
    }
};

// gq = operand copy of g (rounded to the activation element type)
template <class E>
__device__ __forceinline__ float as_operand(float v) { return to_f32(from_f32<E>(v)); }

// da2[pos][o] = [a2[pos][o] > 0] * sum_c g[img][c][pos] * W3[c][o]
template <class E, class WE>
struct LogitsDgradProb {
    static constexpr bool A_K_FAST = false, B_K_FAST = false;
    Geo g; const float* gz; const WE* W3; const E* a2; E* da2;
    __device__ int M() const { return g.positions(); }
    __device__ int N() const { return g.c2; }
    __device__ int K() const { return g.C; }
    __device__ long am(int m) const
    {
        const int hw = g.h * g.w, img = m / hw, r = m - img * hw;
        return (long)img * g.C * hw + r;
    }
    __device__ long ak(int k) const { return (long)k * g.h * g.w; }
    __device__ float a_ld(long at) const { return as_operand<E>(gz[at]); }
    __device__ long bn(int n) const { return n; }
    __device__ long bk(int k) const { return (long)k * g.c2; }
    __device__ float b_ld(long at) const { return to_f32(W3[at]); }
    __device__ void store(int m, int n, float v, int) const
    {
        const size_t at = (size_t)padded_pos(g, m, 0, 0) * g.c2 + n;
        da2[at] = from_f32<E>(to_f32(a2[at]) > 0.f ? v : 0.f);
    }
};

// dW3[c][o] = sum_pos g[c][pos] * a2[pos][o]
template <class E>
struct LogitsWgradProb {
    static constexpr bool A_K_FAST = true, B_K_FAST = false;
    Geo g; const float* gz; const E* a2; float* dW3; size_t copy_stride;
    __device__ int M() const { return g.C; }
    __device__ int N() const { return g.c2; }
    __device__ int K() const { return g.positions(); }
    __device__ long am(int m) const { return (long)m * g.h * g.w; }
    __device__ long ak(int k) const
    {
        const int hw = g.h * g.w, img = k / hw, r = k - img * hw;
        return (long)img * g.C * hw + r;
    }
    __device__ float a_ld(long at) const { return as_operand<E>(gz[at]); }
    __device__ long bn(int n) const { return n; }
    __device__ long bk(int k) const { return (long)padded_pos(g, k, 0, 0) * g.c2; }
    __device__ float b_ld(long at) const { return to_f32(a2[at]); }
    __device__ void store(int m, int n, float v, int share) const { dW3[share * copy_stride + (size_t)m * g.c2 + n] = v; }
};

template <class Prob>
static void launch(Ctx& c, const char* name, const Prob& p, int M, int N, int shares = 1)
{
    ST_LAUNCH(c, name, (k_gemm_generic<Prob>), dim3(cdiv(M, GB), cdiv(N, GB), shares), dim3(256), 0, p);
}

// Position splits of the three weight-gradient products: their outputs are small and their
// reduction runs over every position, so one share per output tile would leave most of the chip
// idle for milliseconds.  Enough shares for about a thousand blocks, at most 16 partial copies,
// at least 128 positions per share.
void generic_wgrad_splits(const Geo& g, int* splits1, int* splits2, int* splits3)
{
    auto pick = [&](int M, int N) {
        const int tiles = cdiv(M, GB) * cdiv(N, GB);
        const int by_work = std::max(1, g.positions() / 128);
        return std::max(1, std::min(std::min(cdiv(1024, tiles), 16), by_work));
    };
    *splits1 = pick(g.c1, 9 * g.c_in);
    *splits2 = pick(g.c2, 9 * g.c1);
    *splits3 = pick(g.C, g.c2);
}

// ---- bias gradients ---------------------------------------------------------------------------
// db[o] = sum over all padded positions of dy[pos][o] (the border holds zeros).  One block per
// 32 channels and share of the positions (blockIdx.y, partial copy `copy_stride` floats apart);
// 8 row-lanes per channel walk the share's positions, then a fixed-order LDS sum.
template <class E>
__global__ void __launch_bounds__(256) k_bias_grad(const E* __restrict__ dy, float* __restrict__ db, int PP, int co,
                                                   size_t copy_stride)
{
    __shared__ float part[8][33];
    const int tx = threadIdx.x % 32, ty = threadIdx.x / 32;
    const int o = blockIdx.x * 32 + tx;
    const int per = (PP + (int)gridDim.y - 1) / (int)gridDim.y;
    const int p0 = (int)blockIdx.y * per, p1 = min(PP, p0 + per);
    float acc = 0.f;
    if (o < co)
        for (int p = p0 + ty; p < p1; p += 8) acc += to_f32(dy[(size_t)p * co + o]);
    part[ty][tx] = acc;
    __syncthreads();
    if (ty == 0 && o < co) {
        float s = 0.f;
        for (int r = 0; r < 8; ++r) s += part[r][tx];
        db[blockIdx.y * copy_stride + o] = s;
    }
}

// db3[c] = sum over frames and positions of the operand copy of g[img][c][pos]; blockIdx.y: share
// of every frame's positions
template <class E>
__global__ void __launch_bounds__(256) k_bias_grad_planar(const float* __restrict__ gz, float* __restrict__ db, Geo g,
                                                          size_t copy_stride)
{
    __shared__ float part[256];
    const int c = blockIdx.x, hw = g.h * g.w;
    const int per = (hw + (int)gridDim.y - 1) / (int)gridDim.y;
    const int p0 = (int)blockIdx.y * per, p1 = min(hw, p0 + per);
    float acc = 0.f;
    for (int img = 0; img < g.n; ++img)
        for (int p = p0 + threadIdx.x; p < p1; p += 256) acc += as_operand<E>(gz[((size_t)img * g.C + c) * hw + p]);
    part[threadIdx.x] = acc;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) part[threadIdx.x] += part[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) db[blockIdx.y * copy_stride + c] = part[0];
}

// ------------------------------------------------------------------ host-side entry points
template <class E, class WE>
static void fwd_impl(Ctx& c, const Plan& p, char* ws, const WE* W1, const WE* W2, const WE* W3,
                     const float* theta, float* z)
{
    const Geo& g = p.g;
    FwdProb<E, WE, 9> p1{g, g.c_in, g.c1, 1, (const E*)(ws + p.feat), W1, theta + p.po.b1, (E*)(ws + p.a1)};
    launch(c, "conv1_fwd_generic", p1, g.positions(), g.c1);
    FwdProb<E, WE, 9> p2{g, g.c1, g.c2, 1, (const E*)(ws + p.a1), W2, theta + p.po.b2, (E*)(ws + p.a2)};
    launch(c, "conv2_fwd_generic", p2, g.positions(), g.c2);
    LogitsProb<E, WE> p3{g, (const E*)(ws + p.a2), W3, theta + p.po.b3, z};
    launch(c, "conv3_fwd_generic", p3, g.positions(), g.C);
}

template <class E, class WE>
static void feat_grad_impl(Ctx& c, const Plan& p, char* ws, const WE* W1, float* dfeat)
{
    const Geo& g = p.g;
    FeatDgradProb<E, WE> d1{g, g.c_in, g.c1, (const E*)(ws + p.da1), W1, dfeat};
    launch(c, "conv1_dgrad_generic", d1, g.positions(), g.c_in);
}

template <class E, class WE>
static void bwd_impl(Ctx& c, const Plan& p, char* ws, const WE* W2, const WE* W3, float* grad)
{
    const Geo& g = p.g;
    const float* gz = (const float*)(ws + p.gz);
    const E* a1 = (const E*)(ws + p.a1);
    const E* a2 = (const E*)(ws + p.a2);
    E* da2 = (E*)(ws + p.da2);
    E* da1 = (E*)(ws + p.da1);
    // layer 3
    LogitsWgradProb<E> w3{g, gz, a2, grad + p.po.W3, p.grad_stride};
    launch(c, "conv3_wgrad_generic", w3, g.C, g.c2, p.splits3);
    ST_LAUNCH(c, "bias3_grad", (k_bias_grad_planar<E>), dim3(g.C, p.splits3), dim3(256), 0, gz, grad + p.po.b3, g,
              p.grad_stride);
    LogitsDgradProb<E, WE> d3{g, gz, W3, a2, da2};
    launch(c, "conv3_dgrad_generic", d3, g.positions(), g.c2);
    // layer 2
    WgradProb<E, 9> w2{g, g.c1, g.c2, da2, a1, grad + p.po.W2, p.grad_stride};
    launch(c, "conv2_wgrad_generic", w2, g.c2, 9 * g.c1, p.splits2);
    ST_LAUNCH(c, "bias2_grad", (k_bias_grad<E>), dim3(cdiv(g.c2, 32), p.splits2), dim3(256), 0, (const E*)da2,
              grad + p.po.b2, g.padded_positions(), g.c2, p.grad_stride);
    DgradProb<E, WE> d2{g, g.c1, g.c2, da2, W2, a1, da1};
    launch(c, "conv2_dgrad_generic", d2, g.positions(), g.c1);
    // layer 1: parameters only -- the features are frozen, no gradient flows past this layer
    WgradProb<E, 9> w1{g, g.c_in, g.c1, da1, (const E*)(ws + p.feat), grad + p.po.W1, p.grad_stride};
    launch(c, "conv1_wgrad_generic", w1, g.c1, 9 * g.c_in, p.splits1);
    ST_LAUNCH(c, "bias1_grad", (k_bias_grad<E>), dim3(cdiv(g.c1, 32), p.splits1), dim3(256), 0, (const E*)da1,
              grad + p.po.b1, g.padded_positions(), g.c1, p.grad_stride);
}

void generic_forward(Ctx& c, const Plan& p, char* ws, float* z)
{
    const float* theta = (const float*)(ws + p.theta);
    if (p.bf16)
        fwd_impl<bf16, bf16>(c, p, ws, (const bf16*)(ws + p.wq1), (const bf16*)(ws + p.wq2),
                             (const bf16*)(ws + p.wq3), theta, z);
    else
        fwd_impl<float, float>(c, p, ws, theta + p.po.W1, theta + p.po.W2, theta + p.po.W3, theta, z);
}

// d loss / d features [n, c_in, h, w] float32 from da1 (run after generic_backward)
void generic_feature_grad(Ctx& c, const Plan& p, char* ws, float* dfeat)
{
    const float* theta = (const float*)(ws + p.theta);
    if (p.bf16) feat_grad_impl<bf16, bf16>(c, p, ws, (const bf16*)(ws + p.wq1), dfeat);
    else feat_grad_impl<float, float>(c, p, ws, theta + p.po.W1, dfeat);
}

void generic_backward(Ctx& c, const Plan& p, char* ws)
{
    const float* theta = (const float*)(ws + p.theta);
    float* grad = (float*)(ws + p.grad);
    if (p.bf16)
        bwd_impl<bf16, bf16>(c, p, ws, (const bf16*)(ws + p.wq2), (const bf16*)(ws + p.wq3), grad);
    else
        bwd_impl<float, float>(c, p, ws, theta + p.po.W2, theta + p.po.W3, grad);
}

}  // namespace st

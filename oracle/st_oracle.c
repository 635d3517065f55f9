/*
 * CPU oracle for the server-side partial-distillation step of ShadowTutor.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, direct
 * implementation in double precision that exists only so that the GPU library
 * can be checked against something independent.  It shares no code with the
 * GPU path: no headers, no kernels, no tables.  Only the test-suite, the smoke
 * check and the benchmark's "cpu_baseline" leg may call it.
 *
 * What it computes (student training, Algorithm 1 of the paper, applied to the
 * trainable tail only as Section 4.2 "Partial Knowledge Distillation" states):
 *
 *   prediction = Forward(head, frozen features)
 *   metric     = mean IoU (Eq. 1) of prediction against the teacher's labels
 *   repeat:  loss = per-pixel cross-entropy (Section 5.2), gradients by the
 *            chain rule down to the first trainable layer and no further,
 *            one optimiser step (gradient descent, optionally with momentum,
 *            or Adam as in Section 5.2), Forward, metric
 *
 * The head is conv3x3(+bias, ReLU), conv3x3(+bias, ReLU), conv1x1(+bias), then
 * an x8 bilinear up-sampling to the input resolution (Section 2.2: the output
 * has the input's spatial size).  Every loop below is the textbook definition,
 * written out; there is no blocking, fusion or reordering.  OpenMP is used only
 * over independent output elements, so results do not depend on thread count.
 *
 * Layout: all tensors are dense, row-major NCHW; weights are OIHW; the flat
 * parameter vector is W1, b1, W2, b2, W3, b3.
 *
 * Parity status: every function here is pinned by tests/test_oracle_*.py
 * (finite differences, closed forms, brute force, an independent library),
 * and so are the losses and trained weights of the k-step loop on the
 * measured workloads themselves (the same loop replayed with an independent
 * library's autograd and optimiser in float64).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define STO_UP 8 /* up-sampling factor of the head's last stage */

int sto_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------ bfloat16 rounding */
/* Round a real value to the nearest bfloat16 (ties to even), going through float32 first,
 * as a GEMM operand of the "bf16 in, fp32 accumulate" variant would be. */
static double round_bf16(double v)
{
    float f = (float)v;
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7fffffffu) > 0x7f800000u) return v; /* NaN stays */
    u += 0x7fffu + ((u >> 16) & 1u);
    u &= 0xffff0000u;
    memcpy(&f, &u, 4);
    return (double)f;
}

void sto_round_bf16(double* x, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) x[i] = round_bf16(x[i]);
}

/* ------------------------------------------------------------------ convolution (k = 1 or 3) */
/* y[n,o,:,:] = b[o] + sum_{i,kh,kw} W[o,i,kh,kw] * x[n,i, .+kh-k/2, .+kw-k/2], zero padding,
 * stride 1 (Forward of Algorithm 1 for one layer). */
void sto_conv_fwd(const double* x, const double* W, const double* b, double* y,
                  int n, int ci, int co, int h, int w, int k)
{
    const int pad = k / 2;
#pragma omp parallel for collapse(2) schedule(static)
    for (int in = 0; in < n; ++in)
        for (int o = 0; o < co; ++o) {
            double* yo = y + ((size_t)in * co + o) * h * w;
            for (int p = 0; p < h * w; ++p) yo[p] = b ? b[o] : 0.0;
            for (int i = 0; i < ci; ++i) {
                const double* xi = x + ((size_t)in * ci + i) * h * w;
                for (int kh = 0; kh < k; ++kh)
                    for (int kw = 0; kw < k; ++kw) {
                        const double wv = W[(((size_t)o * ci + i) * k + kh) * k + kw];
                        const int dy = kh - pad, dx = kw - pad;
                        const int y0 = dy < 0 ? -dy : 0, y1 = dy > 0 ? h - dy : h;
                        const int x0 = dx < 0 ? -dx : 0, x1 = dx > 0 ? w - dx : w;
                        for (int yy = y0; yy < y1; ++yy)
                            for (int xx = x0; xx < x1; ++xx)
                                yo[yy * w + xx] += wv * xi[(yy + dy) * w + xx + dx];
                    }
            }
        }
}

/* dx[n,i,y,x] = sum_{o,kh,kw} W[o,i,kh,kw] * dy[n,o, y-(kh-k/2), x-(kw-k/2)]
 * (chain rule through the layer with respect to its input). */
void sto_conv_dgrad(const double* dy, const double* W, double* dx,
                    int n, int ci, int co, int h, int w, int k)
{
    const int pad = k / 2;
#pragma omp parallel for collapse(2) schedule(static)
    for (int in = 0; in < n; ++in)
        for (int i = 0; i < ci; ++i) {
            double* dxi = dx + ((size_t)in * ci + i) * h * w;
            for (int p = 0; p < h * w; ++p) dxi[p] = 0.0;
            for (int o = 0; o < co; ++o) {
                const double* dyo = dy + ((size_t)in * co + o) * h * w;
                for (int kh = 0; kh < k; ++kh)
                    for (int kw = 0; kw < k; ++kw) {
                        const double wv = W[(((size_t)o * ci + i) * k + kh) * k + kw];
                        const int sy = kh - pad, sx = kw - pad; /* y_out = y_in - sy */
                        const int y0 = sy > 0 ? sy : 0, y1 = sy < 0 ? h + sy : h;
                        const int x0 = sx > 0 ? sx : 0, x1 = sx < 0 ? w + sx : w;
                        for (int yy = y0; yy < y1; ++yy)
                            for (int xx = x0; xx < x1; ++xx)
                                dxi[yy * w + xx] += wv * dyo[(yy - sy) * w + xx - sx];
                    }
            }
        }
}

/* dW[o,i,kh,kw] = sum_{n,y,x} dy[n,o,y,x] * x[n,i,y+kh-k/2,x+kw-k/2];  db[o] = sum dy[n,o,:,:]
 * (chain rule with respect to the layer's own parameters). */
void sto_conv_wgrad(const double* x, const double* dy, double* dW, double* db,
                    int n, int ci, int co, int h, int w, int k)
{
    const int pad = k / 2;
#pragma omp parallel for collapse(2) schedule(static)
    for (int o = 0; o < co; ++o)
        for (int i = 0; i < ci; ++i)
            for (int kh = 0; kh < k; ++kh)
                for (int kw = 0; kw < k; ++kw) {
                    const int dyy = kh - pad, dxx = kw - pad;
                    const int y0 = dyy < 0 ? -dyy : 0, y1 = dyy > 0 ? h - dyy : h;
                    const int x0 = dxx < 0 ? -dxx : 0, x1 = dxx > 0 ? w - dxx : w;
                    double acc = 0.0;
                    for (int in = 0; in < n; ++in) {
                        const double* dyo = dy + ((size_t)in * co + o) * h * w;
                        const double* xi = x + ((size_t)in * ci + i) * h * w;
                        for (int yy = y0; yy < y1; ++yy)
                            for (int xx = x0; xx < x1; ++xx)
                                acc += dyo[yy * w + xx] * xi[(yy + dyy) * w + xx + dxx];
                    }
                    dW[(((size_t)o * ci + i) * k + kh) * k + kw] = acc;
                }
    if (db) {
#pragma omp parallel for schedule(static)
        for (int o = 0; o < co; ++o) {
            double acc = 0.0;
            for (int in = 0; in < n; ++in) {
                const double* dyo = dy + ((size_t)in * co + o) * h * w;
                for (int p = 0; p < h * w; ++p) acc += dyo[p];
            }
            db[o] = acc;
        }
    }
}

/* y = max(x, 0) */
void sto_relu(double* x, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) x[i] = x[i] > 0.0 ? x[i] : 0.0;
}

/* dx = dy where the forward output was positive, else 0 (derivative 0 at the kink) */
void sto_relu_bwd(double* dy, const double* a, int64_t n)
{
    for (int64_t i = 0; i < n; ++i)
        if (!(a[i] > 0.0)) dy[i] = 0.0;
}

/* ------------------------------------------------------------------ x8 bilinear up-sampling */
/* Source coordinate of destination index d with pixel centres at half-integers:
 * src = (d + 0.5) / 8 - 0.5.  Its floor gives the first neighbour, the fraction the weight of
 * the second; both neighbours are clamped to the grid (edge replication). */
static void tap(int d, int len, int* i0, int* i1, double* frac)
{
    const double src = ((double)d + 0.5) / (double)STO_UP - 0.5;
    const double fl = floor(src);
    *frac = src - fl;
    int a = (int)fl, b = a + 1;
    if (a < 0) a = 0;
    if (b < 0) b = 0;
    if (a > len - 1) a = len - 1;
    if (b > len - 1) b = len - 1;
    *i0 = a;
    *i1 = b;
}

/* Z[n,c,Y,X] = lerp_y( lerp_x(z[y0,x0], z[y0,x1]), lerp_x(z[y1,x0], z[y1,x1]) ),
 * lerp(a, b, t) = a + t * (b - a).   planes = n * C. */
void sto_upsample8(const double* z, double* Z, int planes, int h, int w)
{
    const int H = h * STO_UP, Wd = w * STO_UP;
#pragma omp parallel for schedule(static)
    for (int pl = 0; pl < planes; ++pl) {
        const double* zp = z + (size_t)pl * h * w;
        double* Zp = Z + (size_t)pl * H * Wd;
        for (int Y = 0; Y < H; ++Y) {
            int y0, y1;
            double wy;
            tap(Y, h, &y0, &y1, &wy);
            for (int X = 0; X < Wd; ++X) {
                int x0, x1;
                double wx;
                tap(X, w, &x0, &x1, &wx);
                const double r0 = zp[y0 * w + x0] + wx * (zp[y0 * w + x1] - zp[y0 * w + x0]);
                const double r1 = zp[y1 * w + x0] + wx * (zp[y1 * w + x1] - zp[y1 * w + x0]);
                Zp[(size_t)Y * Wd + X] = r0 + wy * (r1 - r0);
            }
        }
    }
}

/* The same interpolation in float32 with a fixed operation order, each operation rounded
 * once: t = b - a; r = fma(t_weight, t, a).  The predicted class is decided on these values
 * (the precision the GPU kernels decide it in), so the order is part of the definition. */
static inline float lerp_f32(float a, float b, float t)
{
    const float d = b - a;
    return fmaf(t, d, a);
}

void sto_upsample8_f32(const float* z, float* Z, int planes, int h, int w)
{
    const int H = h * STO_UP, Wd = w * STO_UP;
#pragma omp parallel for schedule(static)
    for (int pl = 0; pl < planes; ++pl) {
        const float* zp = z + (size_t)pl * h * w;
        float* Zp = Z + (size_t)pl * H * Wd;
        for (int Y = 0; Y < H; ++Y) {
            int y0, y1;
            double wy;
            tap(Y, h, &y0, &y1, &wy);
            for (int X = 0; X < Wd; ++X) {
                int x0, x1;
                double wx;
                tap(X, w, &x0, &x1, &wx);
                const float r0 = lerp_f32(zp[y0 * w + x0], zp[y0 * w + x1], (float)wx);
                const float r1 = lerp_f32(zp[y1 * w + x0], zp[y1 * w + x1], (float)wx);
                Zp[(size_t)Y * Wd + X] = lerp_f32(r0, r1, (float)wy);
            }
        }
    }
}

/* g = U^T G: every high-resolution value is handed back to its four source cells with the
 * weights the forward interpolation used. */
void sto_upsample8_adjoint(const double* G, double* g, int planes, int h, int w)
{
    const int H = h * STO_UP, Wd = w * STO_UP;
#pragma omp parallel for schedule(static)
    for (int pl = 0; pl < planes; ++pl) {
        const double* Gp = G + (size_t)pl * H * Wd;
        double* gp = g + (size_t)pl * h * w;
        for (int p = 0; p < h * w; ++p) gp[p] = 0.0;
        for (int Y = 0; Y < H; ++Y) {
            int y0, y1;
            double wy;
            tap(Y, h, &y0, &y1, &wy);
            for (int X = 0; X < Wd; ++X) {
                int x0, x1;
                double wx;
                tap(X, w, &x0, &x1, &wx);
                const double v = Gp[(size_t)Y * Wd + X];
                gp[y0 * w + x0] += (1.0 - wy) * (1.0 - wx) * v;
                gp[y0 * w + x1] += (1.0 - wy) * wx * v;
                gp[y1 * w + x0] += wy * (1.0 - wx) * v;
                gp[y1 * w + x1] += wy * wx * v;
            }
        }
    }
}

/* ------------------------------------------------------------------ prediction, loss, metric */
/* pred[n,p] = lowest index among the largest of Zf[n,:,p] (float32 values). */
void sto_argmax_f32(const float* Zf, uint8_t* pred, int n, int C, int64_t P)
{
#pragma omp parallel for schedule(static)
    for (int64_t q = 0; q < (int64_t)n * P; ++q) {
        const int in = (int)(q / P);
        const int64_t p = q % P;
        const float* base = Zf + (size_t)in * C * P + p;
        int best = 0;
        float bv = base[0];
        for (int c = 1; c < C; ++c) {
            const float v = base[(size_t)c * P];
            if (v > bv) { bv = v; best = c; }
        }
        pred[q] = (uint8_t)best;
    }
}

static int label_valid(int32_t y, int C, int ignore_index)
{
    return y != ignore_index && y >= 0 && y < C;
}

/* Per-pixel cross-entropy of softmax(Z[:,p]) against the hard label y_p over the valid pixels
 * of all n frames (ComputeLoss of Algorithm 1), each pixel scaled by an integer weight w_p
 * (Section 5.2: the loss of pixels near and within non-background objects is scaled by 5; which
 * pixels those are is the caller's business, it passes the map; weights == NULL means 1
 * everywhere).  The loss is the weighted mean  sum_p w_p CE_p / sum_p w_p  over the valid
 * pixels, and, when G != NULL, G[n,c,p] = w_p (softmax_c - [c == y_p]) / sum w is its
 * derivative (zero on ignored pixels).  Returns the loss; *w_sum_out receives sum w (the
 * number of valid pixels when unweighted).  sum w == 0 gives 0. */
double sto_softmax_ce_w(const double* Z, const int32_t* labels, const uint8_t* weights, double* G,
                        int n, int C, int64_t P, int ignore_index, int64_t* w_sum_out)
{
    int64_t w_sum = 0;
    for (int64_t q = 0; q < (int64_t)n * P; ++q)
        if (label_valid(labels[q], C, ignore_index)) w_sum += weights ? weights[q] : 1;
    if (w_sum_out) *w_sum_out = w_sum;
    const double inv = w_sum > 0 ? 1.0 / (double)w_sum : 0.0;

    /* one partial sum per row-sized chunk, then a serial sum: independent of thread count */
    const int64_t chunk = 1024;
    const int64_t total = (int64_t)n * P;
    const int64_t n_chunks = (total + chunk - 1) / chunk;
    double* part = (double*)calloc((size_t)(n_chunks > 0 ? n_chunks : 1), sizeof(double));
#pragma omp parallel for schedule(static)
    for (int64_t ch = 0; ch < n_chunks; ++ch) {
        double acc = 0.0;
        const int64_t q1 = (ch + 1) * chunk < total ? (ch + 1) * chunk : total;
        for (int64_t q = ch * chunk; q < q1; ++q) {
            const int in = (int)(q / P);
            const int64_t p = q % P;
            const double* zb = Z + (size_t)in * C * P + p;
            double* gb = G ? G + (size_t)in * C * P + p : NULL;
            const int32_t y = labels[q];
            if (!label_valid(y, C, ignore_index)) {
                if (gb) for (int c = 0; c < C; ++c) gb[(size_t)c * P] = 0.0;
                continue;
            }
            const double wp = weights ? (double)weights[q] : 1.0;
            double m = zb[0];
            for (int c = 1; c < C; ++c) if (zb[(size_t)c * P] > m) m = zb[(size_t)c * P];
            double s = 0.0;
            for (int c = 0; c < C; ++c) s += exp(zb[(size_t)c * P] - m);
            const double lse = m + log(s);
            acc += wp * (lse - zb[(size_t)y * P]);
            if (gb)
                for (int c = 0; c < C; ++c)
                    gb[(size_t)c * P] = wp * (exp(zb[(size_t)c * P] - lse) - (c == y ? 1.0 : 0.0)) * inv;
        }
        part[ch] = acc;
    }
    double loss = 0.0;
    for (int64_t ch = 0; ch < n_chunks; ++ch) loss += part[ch];
    free(part);
    return loss * inv;
}

/* the unweighted mean (every weight 1) */
double sto_softmax_ce(const double* Z, const int32_t* labels, double* G,
                      int n, int C, int64_t P, int ignore_index, int64_t* n_valid_out)
{
    return sto_softmax_ce_w(Z, labels, NULL, G, n, C, P, ignore_index, n_valid_out);
}

/* conf[y, pred] += 1 over valid pixels (row = label, column = prediction). */
void sto_confusion(const uint8_t* pred, const int32_t* labels, int64_t P, int C,
                   int ignore_index, int64_t* conf)
{
    memset(conf, 0, sizeof(int64_t) * (size_t)C * C);
    for (int64_t p = 0; p < P; ++p) {
        const int32_t y = labels[p];
        if (!label_valid(y, C, ignore_index)) continue;
        if (pred[p] < C) conf[(size_t)y * C + pred[p]] += 1;
    }
}

/* Mean IoU (Eq. 1): IoU_c = |pred_c ∩ label_c| / |pred_c ∪ label_c|, averaged over the classes
 * that occur in the label.  Returns the number of such classes; no such class gives 0. */
int sto_miou(const int64_t* conf, int C, double* miou)
{
    double sum = 0.0;
    int present = 0;
    for (int c = 0; c < C; ++c) {
        int64_t row = 0, col = 0;
        for (int j = 0; j < C; ++j) { row += conf[(size_t)c * C + j]; col += conf[(size_t)j * C + c]; }
        if (row == 0) continue;
        const int64_t inter = conf[(size_t)c * C + c];
        sum += (double)inter / (double)(row + col - inter);
        ++present;
    }
    *miou = present ? sum / present : 0.0;
    return present;
}

/* ------------------------------------------------------------------ optimiser step */
/* v <- mu v + g;  theta <- theta - lr v   (mu = 0: plain gradient descent, v may be NULL) */
void sto_sgd(double* theta, const double* grad, double* vel, int64_t n, double lr, double mu)
{
    for (int64_t i = 0; i < n; ++i) {
        double step = grad[i];
        if (vel) { vel[i] = mu * vel[i] + grad[i]; step = vel[i]; }
        theta[i] -= lr * step;
    }
}

/* Adam, the optimiser of the paper's experiments (Section 5.2: learning rate 0.01).  The
 * paper gives no further constants; the caller passes them (the published defaults are
 * beta1 = 0.9, beta2 = 0.999, eps = 1e-8).  Step t = 1, 2, .. of the published algorithm:
 *   m <- beta1 m + (1 - beta1) g          v <- beta2 v + (1 - beta2) g^2
 *   mhat = m / (1 - beta1^t)              vhat = v / (1 - beta2^t)
 *   theta <- theta - lr mhat / (sqrt(vhat) + eps)                                        */
void sto_adam(double* theta, const double* grad, double* m, double* v, int64_t n, double lr,
              double beta1, double beta2, double eps, int64_t t)
{
    const double bc1 = 1.0 - pow(beta1, (double)t), bc2 = 1.0 - pow(beta2, (double)t);
    for (int64_t i = 0; i < n; ++i) {
        m[i] = beta1 * m[i] + (1.0 - beta1) * grad[i];
        v[i] = beta2 * v[i] + (1.0 - beta2) * grad[i] * grad[i];
        const double mhat = m[i] / bc1, vhat = v[i] / bc2;
        theta[i] -= lr * mhat / (sqrt(vhat) + eps);
    }
}

/* One optimiser description for the loops below.  kind 0: gradient descent with optional
 * momentum (state s1 = velocity); kind 1: Adam (s1 = m, s2 = v, t0 = steps taken before). */
typedef struct {
    int32_t kind;
    double lr, mu, beta1, beta2, eps;
    int64_t t0;
} sto_optim;

static void optim_step(const sto_optim* o, double* theta, const double* grad, double* s1, double* s2,
                       int64_t n, int64_t step_in_call)
{
    if (o->kind == 1) sto_adam(theta, grad, s1, s2, n, o->lr, o->beta1, o->beta2, o->eps, o->t0 + step_in_call);
    else sto_sgd(theta, grad, o->mu != 0.0 ? s1 : NULL, n, o->lr, o->mu);
}

/* ------------------------------------------------------------------ the head and the loop */
typedef struct {
    int32_t n, c_in, h, w;
    int32_t c1, c2, n_classes;
    int32_t ignore_index;  /* -1: none */
    int32_t bf16_operands; /* 1: round every convolution operand to bfloat16 first */
    const uint8_t* pixel_weights; /* [n, 8h, 8w] loss weight of every pixel, or NULL: all 1 */
} sto_desc;

typedef struct {
    size_t W1, b1, W2, b2, W3, b3, total;
} sto_offsets;

static sto_offsets offsets(const sto_desc* d)
{
    sto_offsets o;
    o.W1 = 0;
    o.b1 = o.W1 + (size_t)d->c1 * d->c_in * 9;
    o.W2 = o.b1 + d->c1;
    o.b2 = o.W2 + (size_t)d->c2 * d->c1 * 9;
    o.W3 = o.b2 + d->c2;
    o.b3 = o.W3 + (size_t)d->n_classes * d->c2;
    o.total = o.b3 + d->n_classes;
    return o;
}

int64_t sto_num_params(const sto_desc* d) { return (int64_t)offsets(d).total; }

static double* dalloc(size_t n) { return (double*)malloc(sizeof(double) * (n ? n : 1)); }

static double* operand_copy(const double* src, size_t n, int bf16)
{
    double* c = dalloc(n);
    memcpy(c, src, sizeof(double) * n);
    if (bf16) sto_round_bf16(c, (int64_t)n);
    return c;
}

typedef struct {
    double *Wq1, *Wq2, *Wq3; /* weights as the convolutions see them */
    double *a1, *a2, *z;     /* activations (a1, a2 after ReLU, rounded if bf16_operands) */
} fwd_state;

static void forward_lowres(const sto_desc* d, const double* f, const double* th, fwd_state* s)
{
    const sto_offsets o = offsets(d);
    const size_t hw = (size_t)d->h * d->w;
    const int q = d->bf16_operands;
    s->Wq1 = operand_copy(th + o.W1, o.b1 - o.W1, q);
    s->Wq2 = operand_copy(th + o.W2, o.b2 - o.W2, q);
    s->Wq3 = operand_copy(th + o.W3, o.b3 - o.W3, q);
    s->a1 = dalloc((size_t)d->n * d->c1 * hw);
    s->a2 = dalloc((size_t)d->n * d->c2 * hw);
    s->z = dalloc((size_t)d->n * d->n_classes * hw);
    sto_conv_fwd(f, s->Wq1, th + o.b1, s->a1, d->n, d->c_in, d->c1, d->h, d->w, 3);
    sto_relu(s->a1, (int64_t)d->n * d->c1 * hw);
    if (q) sto_round_bf16(s->a1, (int64_t)d->n * d->c1 * hw);
    sto_conv_fwd(s->a1, s->Wq2, th + o.b2, s->a2, d->n, d->c1, d->c2, d->h, d->w, 3);
    sto_relu(s->a2, (int64_t)d->n * d->c2 * hw);
    if (q) sto_round_bf16(s->a2, (int64_t)d->n * d->c2 * hw);
    sto_conv_fwd(s->a2, s->Wq3, th + o.b3, s->z, d->n, d->c2, d->n_classes, d->h, d->w, 1);
}

static void free_state(fwd_state* s)
{
    free(s->Wq1); free(s->Wq2); free(s->Wq3); free(s->a1); free(s->a2); free(s->z);
}

/* prediction map from low-resolution logits: interpolate in float32 (fixed order), argmax */
static void predict(const sto_desc* d, const double* z, uint8_t* pred)
{
    const size_t hw = (size_t)d->h * d->w;
    const size_t nz = (size_t)d->n * d->n_classes * hw;
    const int64_t P = (int64_t)hw * STO_UP * STO_UP;
    float* zf = (float*)malloc(sizeof(float) * nz);
    float* Zf = (float*)malloc(sizeof(float) * nz * STO_UP * STO_UP);
    for (size_t i = 0; i < nz; ++i) zf[i] = (float)z[i];
    sto_upsample8_f32(zf, Zf, d->n * d->n_classes, d->h, d->w);
    sto_argmax_f32(Zf, pred, d->n, d->n_classes, P);
    free(zf);
    free(Zf);
}

/* Forward of the head: low-resolution logits z [n,C,h,w] (may be NULL) and the predicted
 * class map pred [n,8h,8w] (may be NULL). */
void sto_head_forward(const sto_desc* d, const double* features, const double* params,
                      double* z_out, uint8_t* pred)
{
    fwd_state s;
    forward_lowres(d, features, params, &s);
    if (z_out) memcpy(z_out, s.z, sizeof(double) * (size_t)d->n * d->n_classes * d->h * d->w);
    if (pred) predict(d, s.z, pred);
    free_state(&s);
}

/* Loss of the head at `params`, and (grad != NULL) its gradient with respect to the head's
 * parameters only: back-propagation stops at the first trainable layer, so no gradient with
 * respect to the features is ever formed (Section 4.2).  Also returns, when asked, the
 * prediction map, per-frame confusion matrices [n,C,C] and per-frame mean IoU [n]. */
double sto_loss_and_grad_full(const sto_desc* d, const double* features, const int32_t* labels,
                              const double* params, double* grad, double* dfeatures, uint8_t* pred_out,
                              int64_t* conf_out, double* miou_out)
{
    const sto_offsets o = offsets(d);
    const int C = d->n_classes;
    const size_t hw = (size_t)d->h * d->w;
    const int64_t P = (int64_t)hw * STO_UP * STO_UP;
    const int q = d->bf16_operands;
    fwd_state s;
    forward_lowres(d, features, params, &s);

    /* metric of this forward */
    if (pred_out || conf_out || miou_out) {
        uint8_t* pred = pred_out ? pred_out : (uint8_t*)malloc((size_t)d->n * P);
        int64_t* conf = (int64_t*)malloc(sizeof(int64_t) * (size_t)C * C);
        predict(d, s.z, pred);
        for (int in = 0; in < d->n; ++in) {
            sto_confusion(pred + (size_t)in * P, labels + (size_t)in * P, P, C, d->ignore_index, conf);
            if (conf_out) memcpy(conf_out + (size_t)in * C * C, conf, sizeof(int64_t) * (size_t)C * C);
            if (miou_out) sto_miou(conf, C, miou_out + in);
        }
        free(conf);
        if (!pred_out) free(pred);
    }

    /* loss on the up-sampled logits */
    const size_t nZ = (size_t)d->n * C * (size_t)P;
    double* Z = dalloc(nZ);
    double* G = grad ? dalloc(nZ) : NULL;
    sto_upsample8(s.z, Z, d->n * C, d->h, d->w);
    const double loss = sto_softmax_ce_w(Z, labels, d->pixel_weights, G, d->n, C, P, d->ignore_index, NULL);
    free(Z);

    if (grad) {
        double* g = dalloc((size_t)d->n * C * hw);
        sto_upsample8_adjoint(G, g, d->n * C, d->h, d->w);
        free(G);
        double* gq = operand_copy(g, (size_t)d->n * C * hw, q);
        /* layer 3 (1x1): parameters, then the input gradient masked by ReLU of layer 2.
         * Weight and bias gradients both sum the same (operand) copy of g. */
        sto_conv_wgrad(s.a2, gq, grad + o.W3, grad + o.b3, d->n, d->c2, C, d->h, d->w, 1);
        double* da2 = dalloc((size_t)d->n * d->c2 * hw);
        sto_conv_dgrad(gq, s.Wq3, da2, d->n, d->c2, C, d->h, d->w, 1);
        sto_relu_bwd(da2, s.a2, (int64_t)d->n * d->c2 * hw);
        if (q) sto_round_bf16(da2, (int64_t)d->n * d->c2 * hw);
        /* layer 2 (3x3) */
        sto_conv_wgrad(s.a1, da2, grad + o.W2, grad + o.b2, d->n, d->c1, d->c2, d->h, d->w, 3);
        double* da1 = dalloc((size_t)d->n * d->c1 * hw);
        sto_conv_dgrad(da2, s.Wq2, da1, d->n, d->c1, d->c2, d->h, d->w, 3);
        sto_relu_bwd(da1, s.a1, (int64_t)d->n * d->c1 * hw);
        if (q) sto_round_bf16(da1, (int64_t)d->n * d->c1 * hw);
        /* layer 1 (3x3): parameters only; the features are frozen, nothing flows past here */
        sto_conv_wgrad(features, da1, grad + o.W1, grad + o.b1, d->n, d->c_in, d->c1, d->h, d->w, 3);
        /* what partial distillation leaves out (Section 4.2): the gradient with respect to the
         * features, which an unfrozen front part would need to continue the chain rule */
        if (dfeatures) sto_conv_dgrad(da1, s.Wq1, dfeatures, d->n, d->c_in, d->c1, d->h, d->w, 3);
        free(da1); free(da2); free(gq); free(g);
    }
    free_state(&s);
    return loss;
}

double sto_loss_and_grad(const sto_desc* d, const double* features, const int32_t* labels,
                         const double* params, double* grad, uint8_t* pred_out,
                         int64_t* conf_out, double* miou_out)
{
    return sto_loss_and_grad_full(d, features, labels, params, grad, NULL, pred_out, conf_out, miou_out);
}

/* k optimiser steps with a fixed step count (Algorithm 1's loop body without the exits):
 * losses[i], mious[i*n + frame] describe the parameters before update i+1; entry k the final
 * ones (k steps = k+1 forwards).  params (and velocity when mu != 0) are updated in place.
 * conf_final [n,C,C] and pred_final [n,8h,8w] (both optional) belong to the final forward. */
void sto_partial_distill_opt(const sto_desc* d, const double* features, const int32_t* labels,
                             double* params, const sto_optim* opt, double* s1, double* s2, int steps,
                             double* losses, double* mious, int64_t* conf_final, uint8_t* pred_final)
{
    const size_t np = offsets(d).total;
    double* grad = dalloc(np);
    for (int it = 0; it <= steps; ++it) {
        const int last = it == steps;
        losses[it] = sto_loss_and_grad(d, features, labels, params, last ? NULL : grad,
                                       last ? pred_final : NULL, last ? conf_final : NULL,
                                       mious + (size_t)it * d->n);
        if (last) break;
        optim_step(opt, params, grad, s1, s2, (int64_t)np, it + 1);
    }
    free(grad);
}

void sto_partial_distill(const sto_desc* d, const double* features, const int32_t* labels,
                         double* params, double* velocity, int steps, double lr, double mu,
                         double* losses, double* mious, int64_t* conf_final, uint8_t* pred_final)
{
    const sto_optim o = {0, lr, mu, 0.0, 0.0, 0.0, 0};
    sto_partial_distill_opt(d, features, labels, params, &o, velocity, NULL, steps, losses, mious,
                            conf_final, pred_final);
}

/* Student training exactly as Algorithm 1 states it: skip when the first metric already
 * reaches THRESHOLD, at most max_updates steps, keep the best-scoring parameters (strictly
 * better), leave the loop once the metric exceeds THRESHOLD (strict_break != 0: '>' as the
 * paper prints; 0: '>=').  The metric is the mean over frames of the per-frame mean IoU.
 * On return params holds best_student; returns the number of updates taken;
 * *best_metric receives the matching metric; metrics[0..updates] the trace. */
int sto_train_opt(const sto_desc* d, const double* features, const int32_t* labels,
                  double* params, const sto_optim* opt, double* s1, double* s2, int max_updates,
                  double threshold, int strict_break, double* best_metric, double* metrics)
{
    const size_t np = offsets(d).total;
    double* grad = dalloc(np);
    double* best = dalloc(np);
    double* fm = dalloc((size_t)d->n);
    int updates = 0;

    sto_loss_and_grad(d, features, labels, params, grad, NULL, NULL, fm);
    double metric = 0.0;
    for (int in = 0; in < d->n; ++in) metric += fm[in];
    metric /= d->n;
    double bm = metric;
    if (metrics) metrics[0] = metric;
    memcpy(best, params, sizeof(double) * np);
    if (bm < threshold) {
        for (int i = 1; i <= max_updates; ++i) {
            optim_step(opt, params, grad, s1, s2, (int64_t)np, i);
            ++updates;
            sto_loss_and_grad(d, features, labels, params, grad, NULL, NULL, fm);
            metric = 0.0;
            for (int in = 0; in < d->n; ++in) metric += fm[in];
            metric /= d->n;
            if (metrics) metrics[i] = metric;
            if (metric > bm) { bm = metric; memcpy(best, params, sizeof(double) * np); }
            if (strict_break ? metric > threshold : metric >= threshold) break;
        }
    }
    memcpy(params, best, sizeof(double) * np);
    *best_metric = bm;
    free(grad); free(best); free(fm);
    return updates;
}

int sto_train(const sto_desc* d, const double* features, const int32_t* labels,
              double* params, double* velocity, int max_updates, double lr, double mu,
              double threshold, int strict_break, double* best_metric, double* metrics)
{
    const sto_optim o = {0, lr, mu, 0.0, 0.0, 0.0, 0};
    return sto_train_opt(d, features, labels, params, &o, velocity, NULL, max_updates, threshold,
                         strict_break, best_metric, metrics);
}

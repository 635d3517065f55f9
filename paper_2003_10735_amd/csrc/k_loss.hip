// Fused x8 bilinear up-sampling + per-pixel softmax cross-entropy + its gradient with respect
// to the low-resolution logits + predicted class + confusion counts, in one pass over the
// labels.  The up-sampled logits (n x C x 8h x 8w) are never written to memory.
//
// Interpolation (pixel centres at half-integers, edge replication): for a destination index
// 8q + j the two source cells and the weight of the second are
//     j <  4:  cells q-1, q      weight (2j + 9) / 16
//     j >= 4:  cells q,   q+1    weight (2j - 7) / 16
// and lerp(a, b, t) is evaluated as fma(t, b - a, a), first along x, then along y, every
// operation rounded once in float32.  The predicted class is decided on exactly these values.
//
// Work split: one 256-thread block per tile of LOSS_TY x LOSS_TX groups of 8 x 8 pixels, one
// thread per pixel column.  A tile touches (LOSS_TY + 2) x (LOSS_TX + 2) low-resolution cells;
// its share of d loss / d z for those cells goes to a slot of its own, and a second small
// kernel adds the (at most four) slots that meet in a cell in a fixed order.  No floating-point
// atomics anywhere: results do not change from run to run.
#include "st_kernels.hpp"

namespace st {

// fixed order, separately rounded: d = b - a;  r = fma(t, d, a)
__device__ __forceinline__ float lerp1(float a, float b, float t)
{
    const float d = __fsub_rn(b, a);
    return __builtin_fmaf(t, d, a);
}

// sum over the 8 lanes of an aligned group of 8 (all 8 lanes receive it), fixed order
__device__ __forceinline__ float group8_sum(float v)
{
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0xB1, 0xF, 0xF, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x4E, 0xF, 0xF, true));
    v += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), 0x141, 0xF, 0xF, true));
    return v;
}

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    return v;
}

// number of valid labels (constant over the steps of one call)
__global__ void __launch_bounds__(256)
k_count_valid(const int32_t* __restrict__ labels, long long P, int C, int ignore, unsigned long long* out)
{
    __shared__ unsigned int part[4];
    unsigned int cnt = 0;
    for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < P; i += (long long)gridDim.x * 256) {
        const int y = labels[i];
        cnt += (y != ignore && y >= 0 && y < C) ? 1u : 0u;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) cnt += __shfl_down(cnt, off, 64);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = cnt;
    __syncthreads();
    if (threadIdx.x == 0) atomicAdd(out, (unsigned long long)(part[0] + part[1] + part[2] + part[3]));
}

template <int CP, bool GRAD>
__global__ void __launch_bounds__(256)
k_loss(const float* __restrict__ z, const int32_t* __restrict__ labels, uint8_t* __restrict__ pred,
       float* __restrict__ slots, float* __restrict__ loss_part, unsigned long long* __restrict__ conf,
       const unsigned long long* __restrict__ n_valid, Geo g, LossTiling lt)
{
    constexpr int CW = LOSS_CW, CH = LOSS_CH, CWP = CW + 1;
    __shared__ float zt[CP][CH][CWP];                 // logits of the touched cells
    __shared__ float contrib[GRAD ? CP : 1][CH][LOSS_TX][3];  // per column group: left/centre/right cell
    __shared__ unsigned int conf_l[32 * 32];          // label x prediction counts of this tile
    __shared__ float wsum[4];

    const int tid = threadIdx.x;
    const int tile = blockIdx.x % lt.tiles(), img = blockIdx.x / lt.tiles();
    const int tile_x = tile % lt.tiles_x, tile_y = tile / lt.tiles_x;
    const int C = g.C, hw = g.h * g.w;
    const int cx0 = tile_x * LOSS_TX - 1, cy0 = tile_y * LOSS_TY - 1;  // cell of local (0, 0)

    // ---- stage the touched cells (edge replication = clamped read); padded classes get a
    //      large negative logit: they never win, their softmax term is exactly 0
    for (int i = tid; i < CP * CH * CW; i += 256) {
        const int lc = i % CW, r = (i / CW) % CH, c = i / (CW * CH);
        const int cx = min(max(cx0 + lc, 0), g.w - 1), cy = min(max(cy0 + r, 0), g.h - 1);
        zt[c][r][lc] = c < C ? z[((size_t)img * C + c) * hw + cy * g.w + cx] : -1e30f;
    }
    for (int i = tid; i < C * C; i += 256) conf_l[i] = 0;
    __syncthreads();

    const int j = tid & 7, tq = tid >> 3;
    const int X = (tile_x * LOSS_TX + tq) * 8 + j;
    const bool col_ok = X < g.W;
    const float fx = (j < 4 ? 2 * j + 9 : 2 * j - 7) * 0.0625f;
    const int cl = tq + (j >= 4 ? 1 : 0);
    const float inv_n = [&] {
        const unsigned long long nv = n_valid ? *n_valid : 0ull;
        return nv ? 1.0f / (float)nv : 0.f;
    }();
    // weights of this column towards the left / centre / right cell of its group
    const float wl = j < 4 ? 1.f - fx : 0.f, wc = j < 4 ? fx : 1.f - fx, wr = j < 4 ? 0.f : fx;

    float loss_acc = 0.f;
    const int32_t* lab_img = labels ? labels + (size_t)img * g.H * g.W : nullptr;
    uint8_t* pred_img = pred ? pred + (size_t)img * g.H * g.W : nullptr;

#pragma unroll 1
    for (int gy = 0; gy < LOSS_TY; ++gy) {
        const int qy = tile_y * LOSS_TY + gy;   // row group
        if (qy >= g.h) break;                   // uniform over the block
        float Hm[CP], H0[CP], Hp[CP];           // x-interpolated logits on cell rows qy-1, qy, qy+1
#pragma unroll
        for (int c = 0; c < CP; ++c) {
            Hm[c] = lerp1(zt[c][gy][cl], zt[c][gy][cl + 1], fx);
            H0[c] = lerp1(zt[c][gy + 1][cl], zt[c][gy + 1][cl + 1], fx);
            Hp[c] = lerp1(zt[c][gy + 2][cl], zt[c][gy + 2][cl + 1], fx);
        }
        float Vm[GRAD ? CP : 1], V0[GRAD ? CP : 1], Vp[GRAD ? CP : 1];
        if (GRAD) {
#pragma unroll
            for (int c = 0; c < CP; ++c) { Vm[c] = 0.f; V0[c] = 0.f; Vp[c] = 0.f; }
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float fy = (i < 4 ? 2 * i + 9 : 2 * i - 7) * 0.0625f;
            const int Y = qy * 8 + i;
            float Z[CP];
#pragma unroll
            for (int c = 0; c < CP; ++c) Z[c] = i < 4 ? lerp1(Hm[c], H0[c], fy) : lerp1(H0[c], Hp[c], fy);
            // prediction: lowest index among the largest
            float m = Z[0];
            int best = 0;
#pragma unroll
            for (int c = 1; c < CP; ++c)
                if (Z[c] > m) { m = Z[c]; best = c; }
            if (pred_img && col_ok) pred_img[(size_t)Y * g.W + X] = (uint8_t)best;
            if (lab_img) {
                const int y = col_ok ? lab_img[(size_t)Y * g.W + X] : -1;
                const bool valid = col_ok && y != g.ignore_index && y >= 0 && y < C;
                float s = 0.f, zym = 0.f;   // zym = Z_y - m
#pragma unroll
                for (int c = 0; c < CP; ++c) {
                    const float t = Z[c] - m;
                    zym = (c == y) ? t : zym;
                    Z[c] = __builtin_amdgcn_exp2f(t * 1.44269504088896341f);
                    s += Z[c];
                }
                // -log softmax_y = log(sum exp(Z - m)) - (Z_y - m)
                const float nll = __builtin_amdgcn_logf(s) * 0.693147180559945309f - zym;
                if (valid) {
                    loss_acc += nll;
                    atomicAdd(&conf_l[y * C + best], 1u);
                }
                if (GRAD) {
                    const float rs = valid ? __builtin_amdgcn_rcpf(s) : 0.f;
#pragma unroll
                    for (int c = 0; c < CP; ++c) {
                        const float G = valid ? __builtin_fmaf(Z[c], rs, c == y ? -1.f : 0.f) : 0.f;
                        if (i < 4) { Vm[c] = fmaf(1.f - fy, G, Vm[c]); V0[c] = fmaf(fy, G, V0[c]); }
                        else       { V0[c] = fmaf(1.f - fy, G, V0[c]); Vp[c] = fmaf(fy, G, Vp[c]); }
                    }
                }
            }
        }
        if (GRAD) {
            // hand the column sums to the three cells of this column group (adjoint of the
            // x-interpolation), reduced over the group's 8 columns
#pragma unroll
            for (int c = 0; c < CP; ++c) {
#pragma unroll
                for (int r = 0; r < 3; ++r) {
                    const float v = r == 0 ? Vm[c] : (r == 1 ? V0[c] : Vp[c]);
                    const float L = group8_sum(v * wl), M = group8_sum(v * wc), R = group8_sum(v * wr);
                    if (j == 0) {
                        float* dst = &contrib[c][gy + r][tq][0];
                        if (gy == 0 || r == 2) { dst[0] = L; dst[1] = M; dst[2] = R; }
                        else { dst[0] += L; dst[1] += M; dst[2] += R; }
                    }
                }
            }
        }
    }

    // ---- loss of this tile: wave sums, then the four waves in order
    loss_acc = wave_sum(loss_acc);
    if ((tid & 63) == 0) wsum[tid >> 6] = loss_acc;
    __syncthreads();
    if (tid == 0 && loss_part) loss_part[blockIdx.x] = ((wsum[0] + wsum[1]) + wsum[2]) + wsum[3];
    if (conf && lab_img)
        for (int i = tid; i < C * C; i += 256)
            if (conf_l[i]) atomicAdd(&conf[(size_t)img * C * C + i], (unsigned long long)conf_l[i]);

    if (GRAD) {
        // rows of `contrib` a short last tile never wrote must read as zero
        const int rows_done = min(LOSS_TY, g.h - tile_y * LOSS_TY);   // row groups processed
        // ---- cell totals: column group lc gives its left part, lc-1 its centre, lc-2 its right
        float* slot = slots + (size_t)blockIdx.x * CP * CH * CW;
        // 1) gather into zt (reused as the output tile)
        __syncthreads();
        for (int i = tid; i < CP * CH * CW; i += 256) {
            const int lc = i % CW, r = (i / CW) % CH, c = i / (CW * CH);
            float v = 0.f;
            if (r < rows_done + 2) {
                if (lc < LOSS_TX) v += contrib[c][r][lc][0];
                if (lc >= 1 && lc - 1 < LOSS_TX) v += contrib[c][r][lc - 1][1];
                if (lc >= 2) v += contrib[c][r][lc - 2][2];
            }
            zt[c][r][lc] = v;
        }
        __syncthreads();
        // 2) fold cells outside the grid onto the border cell they replicate, scale, store
        for (int i = tid; i < CP * CH * CW; i += 256) {
            const int lc = i % CW, r = (i / CW) % CH, c = i / (CW * CH);
            const int cx = cx0 + lc, cy = cy0 + r;
            float v = 0.f;
            if (cx >= 0 && cx < g.w && cy >= 0 && cy < g.h) {
                v = zt[c][r][lc];
                const bool fl = cx == 0 && lc >= 1, fr = cx == g.w - 1 && lc + 1 < CW;
                const bool fu = cy == 0 && r >= 1, fd = cy == g.h - 1 && r + 1 < CH;
                if (fl) v += zt[c][r][lc - 1];
                if (fr) v += zt[c][r][lc + 1];
                if (fu) {
                    v += zt[c][r - 1][lc];
                    if (fl) v += zt[c][r - 1][lc - 1];
                    if (fr) v += zt[c][r - 1][lc + 1];
                }
                if (fd) {
                    v += zt[c][r + 1][lc];
                    if (fl) v += zt[c][r + 1][lc - 1];
                    if (fr) v += zt[c][r + 1][lc + 1];
                }
                v *= inv_n;
            }
            slot[i] = v;
        }
    }
}

// g[img][c][cy][cx] = sum of the slots of the tiles that touch the cell, tile rows first
template <int CP>
__global__ void __launch_bounds__(256)
k_assemble_g(const float* __restrict__ slots, float* __restrict__ gz, Geo g, LossTiling lt)
{
    constexpr int CW = LOSS_CW, CH = LOSS_CH;
    const int idx = blockIdx.x * 256 + threadIdx.x;
    const int hw = g.h * g.w;
    if (idx >= g.n * g.C * hw) return;
    const int cx = idx % g.w, cy = (idx / g.w) % g.h, c = (idx / hw) % g.C, img = idx / (hw * g.C);
    float v = 0.f;
    // tiles whose cell window [t*T - 1, t*T + T] contains the cell: the last candidate is
    // (cell + 1) / T, and a window of T + 2 cells can overlap at most 3 tiles
    const int ty_hi = min((cy + 1) / LOSS_TY, lt.tiles_y - 1), tx_hi = min((cx + 1) / LOSS_TX, lt.tiles_x - 1);
    for (int ty = max(ty_hi - 2, 0); ty <= ty_hi; ++ty) {
        const int r = cy - (ty * LOSS_TY - 1);
        if (r < 0 || r >= CH) continue;
        for (int tx = max(tx_hi - 2, 0); tx <= tx_hi; ++tx) {
            const int lc = cx - (tx * LOSS_TX - 1);
            if (lc < 0 || lc >= CW) continue;
            const size_t tile = (size_t)img * lt.tiles() + ty * lt.tiles_x + tx;
            v += slots[((tile * CP + c) * CH + r) * CW + lc];
        }
    }
    gz[idx] = v;
}

static int padded_classes(int C) { return (C + 3) / 4 * 4; }

size_t loss_slot_floats(const Geo& g)
{
    const LossTiling lt = loss_tiling(g);
    return (size_t)g.n * lt.tiles() * padded_classes(g.C) * LOSS_CH * LOSS_CW;
}

int loss_blocks(const Geo& g) { return g.n * loss_tiling(g).tiles(); }

void count_valid(Ctx& c, const Geo& g, const int32_t* labels, unsigned long long* out)
{
    const long long P = g.pixels();
    int blocks = cdiv(P, 256 * 8);
    if (blocks > 1024) blocks = 1024;
    ST_LAUNCH(c, "count_valid", k_count_valid, dim3(blocks), dim3(256), 0, labels, P, g.C, g.ignore_index, out);
}

template <int CP>
static void loss_launch(Ctx& c, const Geo& g, const float* z, const int32_t* labels, uint8_t* pred,
                        float* slots, float* gz, float* loss_part, unsigned long long* conf,
                        const unsigned long long* n_valid, bool grad)
{
    const LossTiling lt = loss_tiling(g);
    const int blocks = g.n * lt.tiles();
    if (grad) {
        ST_LAUNCH(c, "upsample_ce_grad", (k_loss<CP, true>), dim3(blocks), dim3(256), 0, z, labels, pred,
                  slots, loss_part, conf, n_valid, g, lt);
        ST_LAUNCH(c, "assemble_dz", (k_assemble_g<CP>), dim3(cdiv((long long)g.n * g.C * g.h * g.w, 256)),
                  dim3(256), 0, (const float*)slots, gz, g, lt);
    } else {
        ST_LAUNCH(c, "upsample_ce", (k_loss<CP, false>), dim3(blocks), dim3(256), 0, z, labels, pred,
                  slots, loss_part, conf, n_valid, g, lt);
    }
}

void loss_pass(Ctx& c, const Geo& g, const float* z, const int32_t* labels, uint8_t* pred, float* slots,
               float* gz, float* loss_part, unsigned long long* conf, const unsigned long long* n_valid,
               bool grad)
{
    switch (padded_classes(g.C)) {
    case 4: loss_launch<4>(c, g, z, labels, pred, slots, gz, loss_part, conf, n_valid, grad); break;
    case 8: loss_launch<8>(c, g, z, labels, pred, slots, gz, loss_part, conf, n_valid, grad); break;
    case 12: loss_launch<12>(c, g, z, labels, pred, slots, gz, loss_part, conf, n_valid, grad); break;
    case 16: loss_launch<16>(c, g, z, labels, pred, slots, gz, loss_part, conf, n_valid, grad); break;
    case 20: loss_launch<20>(c, g, z, labels, pred, slots, gz, loss_part, conf, n_valid, grad); break;
    case 24: loss_launch<24>(c, g, z, labels, pred, slots, gz, loss_part, conf, n_valid, grad); break;
    case 28: loss_launch<28>(c, g, z, labels, pred, slots, gz, loss_part, conf, n_valid, grad); break;
    case 32: loss_launch<32>(c, g, z, labels, pred, slots, gz, loss_part, conf, n_valid, grad); break;
    default: c.status = ST_ERR_SHAPE; break;
    }
}

}  // namespace st

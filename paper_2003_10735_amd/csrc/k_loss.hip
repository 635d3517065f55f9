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
// What depends on the labels but not on the logits is computed once per call
// (label_adjoint_block, a role of the launch that opens a call): with U the up-sampling operator
// and Y the one-hot label map,
//     T = U^T Y                      (exact in float32: sums of multiples of 1/256)
// Then, with P the softmax of the up-sampled logits on the valid pixels,
//     d loss / d z = (U^T P - T) / N_valid
//     loss         = ( sum_valid logsumexp  -  <T, z> ) / N_valid        (U z is linear in z)
// so the per-step kernel needs no per-class label test at all: per pixel and class it does one
// fma (interpolate), max/compare (prediction), fma + exp, add, and two fmas (U^T along y).
//
// Work split: one 512-thread block per tile of 1 x LOSS_TX groups of 8 x 8 pixels, two threads
// per pixel column (four pixels each).  A tile touches 3 x (LOSS_TX + 2) low-resolution cells;
// its share of U^T P for those cells goes to a slot of its own, and the consumer adds the (at
// most four) slots that meet in a cell in a fixed order.  No floating-point atomics anywhere:
// results do not change from run to run.
#include "st_kernels.hpp"
#include "st_mfma.hpp"

namespace st {

// fixed order, separately rounded: d = b - a;  r = fma(t, d, a)
__device__ __forceinline__ float lerp1(float a, float b, float t)
{
    const float d = __fsub_rn(b, a);
    return __builtin_fmaf(t, d, a);
}

template <int CTRL>
__device__ __forceinline__ float dpp_add(float v)
{
    return v + __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xF, 0xF, true));
}
// sum over the 4 lanes of a quad / the 8 lanes of an aligned group of 8 (every lane gets it)
__device__ __forceinline__ float quad_sum(float v) { return dpp_add<0x4E>(dpp_add<0xB1>(v)); }
__device__ __forceinline__ float group8_sum(float v) { return dpp_add<0x141>(quad_sum(v)); }

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    return v;
}

constexpr int LOSS_THREADS = 2 * 8 * LOSS_TX;   // two threads per pixel column of the tile

// (up to 24 padded classes the kernel is held to 128 registers, so that two blocks share a
//  compute unit: the phases of one then fill the barriers and memory waits of the other)
// CP: classes rounded up to a multiple of four (the layout of the logit shares, of the staged
// cells and of the slots); CA: the number of classes itself, CP - 3 .. CP -- the per-pixel
// arithmetic runs over exactly these, so a padded class costs no instruction.
template <int CP, int CA, bool GRAD>
__global__ void __launch_bounds__(LOSS_THREADS, (CP <= 24 ? 4 : 2))
k_loss(ZSrc zs, const uint8_t* __restrict__ labels, const uint8_t* __restrict__ wmap, const float* __restrict__ T,
       uint8_t* __restrict__ pred, float* __restrict__ slots, float* __restrict__ loss_part,
       unsigned long long* __restrict__ conf, Geo g, LossTiling lt, int n_tiles)
{
    static_assert(LOSS_TY == 1, "one row group per tile: the two halves of a block split its 8 pixel rows");
    constexpr int CW = LOSS_CW, CH = LOSS_CH, CWP = CW + 1, NT = LOSS_THREADS;
    __shared__ float zt[CP][CH][CWP];                 // logits of the touched cells
    // per half, class, cell row (upper / lower of the half) and column group: what the group hands
    // to its (left, centre, right, unused) cells; written once, never read-modify-written
    __shared__ __attribute__((aligned(16))) float contrib[GRAD ? 2 : 1][GRAD ? CP : 1][2][LOSS_TX][4];
    __shared__ unsigned int conf_l[32 * 32];          // label x prediction counts of this tile
    __shared__ float wsum[NT / 64];

    const int tid = threadIdx.x;
    // XCD-aware tile order: consecutive blocks go to different XCDs, each with an L2 of its own.
    // Every XCD gets a contiguous run of tiles (a band of rows), so the three tiles that stage the
    // same row of cells run on one XCD and two of them find the row in its L2.
    const int per_xcd = (n_tiles + 7) >> 3;
    const int bid = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if ((int)(blockIdx.x >> 3) >= per_xcd || bid >= n_tiles) return;
    const int tile = bid % lt.tiles(), img = bid / lt.tiles();
    const int tile_x = tile % lt.tiles_x, qy = tile / lt.tiles_x;   // qy: row group = cell row
    const int C = g.C, hw = g.h * g.w;
    const int cx0 = tile_x * LOSS_TX - 1, cy0 = qy - 1;  // cell of local (0, 0)

    // ---- stage the touched cells (edge replication = clamped read); padded classes get a
    //      large negative logit: they never win, their softmax term is exactly 0.
    //      All global loads of the prologue are issued before anything waits for one of them.
    constexpr int NZ = (CP * CH * CW + NT - 1) / NT;
    constexpr int QC = CP / 4;                            // 16-byte chunks of a cell's row of CP classes
    constexpr int NZQ = (CH * CW * QC + NT - 1) / NT;
    float zv[NZ];
    f32x4 zr[NZQ][4], bq[NZQ];
    if (zs.parts) {
        const size_t PP = (size_t)g.padded_positions();
#pragma unroll
        for (int k = 0; k < NZQ; ++k) {
            const int i = min(tid + k * NT, CH * CW * QC - 1);
            const int cell = i / QC, chunk = i - cell * QC;
            const int lc = cell % CW, r = cell / CW;
            const int cx = min(max(cx0 + lc, 0), g.w - 1), cy = min(max(cy0 + r, 0), g.h - 1);
            const size_t mp = ((size_t)img * g.Hp + cy + 1) * g.Wp + cx + 1;
            // one, two or four shares (64, 128, 256 channels); within a group of two an absent
            // share re-reads the last one (it is then not added), so that the loads of a group are
            // issued together.  Only loaded here: the sums wait until every load of the prologue
            // is on its way.
            const float* zp = zs.parts + mp * CP + chunk * 4;
            const size_t share = PP * CP;
            zr[k][0] = *(const f32x4*)zp;
            zr[k][1] = *(const f32x4*)(zp + (zs.n_parts > 1 ? share : 0));
            if (zs.n_parts > 2) {
                zr[k][2] = *(const f32x4*)(zp + 2 * share);
                zr[k][3] = *(const f32x4*)(zp + 3 * share);
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) bq[k][e] = zs.b3[g.head_of(img) * zs.b3_stride + min(chunk * 4 + e, C - 1)];
        }
    } else {
#pragma unroll
        for (int k = 0; k < NZ; ++k) {
            const int i = min(tid + k * NT, CP * CH * CW - 1);
            const int lc = i % CW, r = (i / CW) % CH, c = i / (CW * CH);
            const int cx = min(max(cx0 + lc, 0), g.w - 1), cy = min(max(cy0 + r, 0), g.h - 1);
            zv[k] = zs.planar[((size_t)img * C + min(c, C - 1)) * hw + cy * g.w + cx];
        }
    }
    // T over the cells this tile owns, for the  - <T, z>  part of the loss (see the header)
    constexpr int NTT = (32 * LOSS_TX + NT - 1) / NT;
    float tv[NTT];
    const bool want_tz = T && loss_part;
#pragma unroll
    for (int k = 0; k < NTT; ++k) tv[k] = 0.f;
    if (want_tz) {
        // (clamped addresses: the values of cells and classes that do not exist are dropped below)
#pragma unroll
        for (int k = 0; k < NTT; ++k) {
            const int i = tid + k * NT;
            const int lc = i % LOSS_TX, c = i / LOSS_TX;
            const int cx = tile_x * LOSS_TX + lc;
            tv[k] = T[((size_t)img * C + min(c, C - 1)) * hw + qy * g.w + min(cx, g.w - 1)];
        }
    }
    for (int i = tid; i < C * C; i += NT) conf_l[i] = 0;

    // Two threads per pixel column: `half` 0 takes the upper four pixels of the 8 (they
    // interpolate between cell rows qy-1 and qy), half 1 the lower four (rows qy and qy+1).
    // The per-thread instruction stream is the critical path of this kernel, so it is kept short.
    const int half = tid >= NT / 2 ? 1 : 0, t = tid - half * (NT / 2);
    const int j = t & 7, tq = t >> 3;
    const int X = (tile_x * LOSS_TX + tq) * 8 + j;
    const bool col_ok = X < g.W;
    const float fx = (j < 4 ? 2 * j + 9 : 2 * j - 7) * 0.0625f;
    const int cl = tq + (j >= 4 ? 1 : 0);
    // weights of this column towards its group's outer cell (left for j < 4, right for j >= 4)
    // and towards the centre cell
    float w_side = j < 4 ? 1.f - fx : fx, w_mid = j < 4 ? fx : 1.f - fx;
    {
        // edge replication: at the first / last column group the cell outside the grid is the
        // border cell itself, so its weight goes to the centre cell
        const int q = tile_x * LOSS_TX + tq;
        if ((q == 0 && j < 4) || (q == g.w - 1 && j >= 4)) { w_mid += w_side; w_side = 0.f; }
    }
    const uint8_t* lab_img = labels ? labels + (size_t)img * g.H * g.W : nullptr;
    uint8_t* pred_img = pred ? pred + (size_t)img * g.H * g.W : nullptr;
    const int Yb = qy * 8 + half * 4;    // first of this thread's four pixel rows
    // labels of this thread's 4 pixels, fetched before the barrier
    int lab4[4] = {255, 255, 255, 255};
    int wraw[4] = {1, 1, 1, 1};              // loss weight of each pixel
    if (lab_img) {
        const size_t at = (size_t)Yb * g.W + min(X, g.W - 1);
#pragma unroll
        for (int i = 0; i < 4; ++i) lab4[i] = lab_img[at + (size_t)i * g.W];
        if (wmap) {
            const uint8_t* wm = wmap + (size_t)img * g.H * g.W;
#pragma unroll
            for (int i = 0; i < 4; ++i) wraw[i] = wm[at + (size_t)i * g.W];
        }
    }
    // ---- every load of the prologue is issued; from here on their values are used
    float w4[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        lab4[i] = col_ok ? lab4[i] : 255;
        w4[i] = col_ok ? (float)wraw[i] : 0.f;
    }
    if (want_tz) {
#pragma unroll
        for (int k = 0; k < NTT; ++k) {
            const int i = tid + k * NT;
            if (i / LOSS_TX >= C || tile_x * LOSS_TX + i % LOSS_TX >= g.w) tv[k] = 0.f;
        }
    }
    if (zs.parts) {
#pragma unroll
        for (int k = 0; k < NZQ; ++k) {
            const int i = tid + k * NT;
            const int cell = i / QC, chunk = i - cell * QC;
            const int lc = cell % CW, r = cell / CW;
            // the shares in ascending order (each addition rounded on its own), then the bias
            f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                acc[e] = __builtin_fmaf(1.f, zr[k][0][e], acc[e]);
                if (zs.n_parts > 1) acc[e] = __builtin_fmaf(1.f, zr[k][1][e], acc[e]);
            }
            if (zs.n_parts > 2) {
#pragma unroll
                for (int e = 0; e < 4; ++e) acc[e] = __builtin_fmaf(1.f, zr[k][3][e], __builtin_fmaf(1.f, zr[k][2][e], acc[e]));
            }
            if (i < CH * CW * QC) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int c = chunk * 4 + e;
                    zt[c][r][lc] = c < C ? acc[e] + bq[k][e] : -1e30f;
                }
            }
        }
    } else {
#pragma unroll
        for (int k = 0; k < NZ; ++k) {
            const int i = tid + k * NT;
            const int lc = i % CW, r = (i / CW) % CH, c = i / (CW * CH);
            if (i < CP * CH * CW) zt[c][r][lc] = c < C ? zv[k] : -1e30f;
        }
    }
    __syncthreads();
    // the logits of this tile's own cells, as used below, for whoever wants the planar tensor
    if (zs.parts && zs.z_out) {
        for (int i = tid; i < C * LOSS_TX; i += NT) {
            const int lc = i % LOSS_TX, c = i / LOSS_TX;
            const int cx = tile_x * LOSS_TX + lc;
            if (cx < g.w) zs.z_out[((size_t)img * C + c) * hw + qy * g.w + cx] = zt[c][1][lc + 1];
        }
    }

    float loss_acc = 0.f;
#pragma unroll
    for (int k = 0; k < NTT; ++k) {
        const int i = tid + k * NT;
        const int lc = i % LOSS_TX, c = min(i / LOSS_TX, CP - 1);
        loss_acc -= tv[k] * zt[c][1][lc + 1];     // tv is 0 where the cell or class does not exist
    }

    // x-interpolated logits on this half's upper cell row and their difference to the lower one
    // (the y interpolation is fma(fy, difference, upper row): same roundings as lerp1)
    float Hu[CA], D[CA];
#pragma unroll
    for (int c = 0; c < CA; ++c) {
        Hu[c] = lerp1(zt[c][half][cl], zt[c][half][cl + 1], fx);
        const float Hl = lerp1(zt[c][half + 1][cl], zt[c][half + 1][cl + 1], fx);
        D[c] = __fsub_rn(Hl, Hu[c]);
    }
    float Vu[GRAD ? CA : 1], Vl[GRAD ? CA : 1];    // U^T along y: upper / lower cell row of the half
    if (GRAD) {
#pragma unroll
        for (int c = 0; c < CA; ++c) { Vu[c] = 0.f; Vl[c] = 0.f; }
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        // weight of the lower cell row: (9, 11, 13, 15) / 16 in the upper half, (1, 3, 5, 7) / 16 below
        const float fy = half ? (2 * i + 1) * 0.0625f : (2 * i + 9) * 0.0625f;
        const int Y = Yb + i;
        float Z[CA];
#pragma unroll
        for (int c = 0; c < CA; ++c) Z[c] = __builtin_fmaf(fy, D[c], Hu[c]);
        // prediction: the largest logit, lowest index among equals
        float m = Z[0];
#pragma unroll
        for (int c = 1; c < CA; ++c) m = fmaxf(m, Z[c]);
        // (when nothing compares equal to the maximum -- NaN logits -- the answer is class 0)
        int best = 0;
#pragma unroll
        for (int c = CA - 1; c >= 0; --c) best = Z[c] == m ? c : best;
        if (pred_img && col_ok) pred_img[(size_t)Y * g.W + X] = (uint8_t)best;
        if (lab_img) {
            const int y = lab4[i];
            const bool valid = y < C;     // (255: ignored, no class index, or off the frame)
            const float mb = -m * 1.44269504088896341f;
            float sum = 0.f;
#pragma unroll
            for (int c = 0; c < CA; ++c) {
                Z[c] = __builtin_amdgcn_exp2f(__builtin_fmaf(Z[c], 1.44269504088896341f, mb));
                sum += Z[c];
            }
            if (valid) {
                loss_acc += w4[i] * __builtin_fmaf(__builtin_amdgcn_logf(sum), 0.693147180559945309f, m);
                atomicAdd(&conf_l[y * C + best], 1u);
            }
            if (GRAD) {
                const float rs = valid ? w4[i] * __builtin_amdgcn_rcpf(sum) : 0.f;
                const float wa = (1.f - fy) * rs, wb = fy * rs;
#pragma unroll
                for (int c = 0; c < CA; ++c) {
                    Vu[c] = __builtin_fmaf(wa, Z[c], Vu[c]);
                    Vl[c] = __builtin_fmaf(wb, Z[c], Vl[c]);
                }
            }
        }
    }
    if (GRAD) {
        // edge replication for the first / last row group: the cell row outside the grid is the
        // border row itself
        if (qy == 0 && half == 0) {
#pragma unroll
            for (int c = 0; c < CA; ++c) { Vl[c] += Vu[c]; Vu[c] = 0.f; }
        }
        if (qy == g.h - 1 && half == 1) {
#pragma unroll
            for (int c = 0; c < CA; ++c) { Vu[c] += Vl[c]; Vl[c] = 0.f; }
        }
        // adjoint of the x interpolation, reduced over the group's 8 columns: columns 0-3 feed
        // the left and the centre cell, columns 4-7 the centre and the right cell
        float2* my_contrib = (float2*)&contrib[half][0][0][tq][0] + (j >> 2);
#pragma unroll
        for (int c = 0; c < CA; ++c) {
#pragma unroll
            for (int r = 0; r < 2; ++r) {
                const float v = r == 0 ? Vu[c] : Vl[c];
                float side = quad_sum(v * w_side);   // lanes 0-3: left cell, lanes 4-7: right cell
                float mid = group8_sum(v * w_mid);
                // (the sums are complete before the branch: inside it the cross-lane operand and
                //  its addition would be two instructions)
                asm volatile("" : "+v"(side), "+v"(mid));
                // lane 0 of the group writes (left, centre), lane 4 writes (right, unused)
                if ((j & 3) == 0) my_contrib[(c * 2 + r) * (LOSS_TX * 2)] = make_float2(side, j == 0 ? mid : 0.f);
            }
        }
    }

    // ---- loss of this tile: wave sums, then the waves in order
    loss_acc = wave_sum(loss_acc);
    if ((tid & 63) == 0) wsum[tid >> 6] = loss_acc;
    __syncthreads();
    if (tid == 0 && loss_part) {
        float acc = wsum[0];
#pragma unroll
        for (int w = 1; w < NT / 64; ++w) acc += wsum[w];
        loss_part[bid] = acc;
    }
    if (conf && lab_img)
        for (int i = tid; i < C * C; i += NT)
            if (conf_l[i]) atomicAdd(&conf[(size_t)img * C * C + i], (unsigned long long)conf_l[i]);

    if (GRAD) {
        float* slot = slots + (size_t)bid * CP * CH * CW;
        // cell totals: column group lc gives its left part, lc-1 its centre part, lc-2 its right
        // part; cell row 0 comes from the upper half, row 2 from the lower half, row 1 from both
        // (upper half first).  Cells outside the grid received nothing (their weight went to the
        // border cells above).
        // A thread keeps one cell (row r, column lc) and walks over the classes, NT / (CH * CW) of
        // them per trip of the block: everything that depends on the cell is computed once.
        constexpr int CELLS = CH * CW, CSTEP = NT / CELLS;
        const int cg = tid / CELLS, cell = tid - cg * CELLS;
        const int r = cell / CW, lc = cell - r * CW;
        const int hfA = r == 2 ? 1 : 0, rrA = r - hfA;        // first contributing (half, row of the half)
        const bool pairB = r == 1;                             // row 1 also gets the lower half's row 0
        const bool s0 = lc < LOSS_TX, s1 = lc >= 1 && lc <= LOSS_TX, s2 = lc >= 2;
        const int i0 = min(lc, LOSS_TX - 1) * 4, i1 = min(max(lc - 1, 0), LOSS_TX - 1) * 4 + 1, i2 = max(lc - 2, 0) * 4 + 2;
        if (cg < CSTEP) {
#pragma unroll
            for (int k = 0; k < (CP + CSTEP - 1) / CSTEP; ++k) {
                const int c = cg + k * CSTEP;
                if (c >= CP) break;
                float v = 0.f;
                if (c < CA) {                                  // (a padded class: nothing was handed over)
                    const float* A = &contrib[hfA][c][rrA][0][0];
                    const float a0 = A[i0], a1 = A[i1], a2 = A[i2];
                    v += s0 ? a0 : 0.f;
                    v += s1 ? a1 : 0.f;
                    v += s2 ? a2 : 0.f;
                    if (pairB) {
                        const float* B = &contrib[1][c][0][0][0];
                        const float b0 = B[i0], b1 = B[i1], b2 = B[i2];
                        v += s0 ? b0 : 0.f;
                        v += s1 ? b1 : 0.f;
                        v += s2 ? b2 : 0.f;
                    }
                }
                slot[c * CELLS + cell] = v;
            }
        }
    }
}

// g[img][c][cy][cx] = ( sum of the slots of the tiles that touch the cell, tile rows first,  - T ) / N_valid
template <int CP>
__global__ void __launch_bounds__(256)
k_assemble_g(const float* __restrict__ slots, const float* __restrict__ T,
             const unsigned long long* __restrict__ n_valid, float* __restrict__ gz, Geo g, LossTiling lt)
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
    const unsigned long long nv = *n_valid;
    const float inv_n = nv ? 1.0f / (float)nv : 0.f;
    gz[idx] = (v - T[idx]) * inv_n;
}

static int padded_classes(int C) { return (C + 3) / 4 * 4; }

size_t loss_slot_floats(const Geo& g)
{
    const LossTiling lt = loss_tiling(g);
    return (size_t)g.n * lt.tiles() * padded_classes(g.C) * LOSS_CH * LOSS_CW;
}

int loss_blocks(const Geo& g) { return g.n * loss_tiling(g).tiles(); }

template <int CP, int CA>
static void loss_launch(Ctx& c, const Geo& g, const ZSrc& zs, const uint8_t* labels, const uint8_t* wmap,
                        const float* T,
                        uint8_t* pred, float* slots, float* gz, float* loss_part, unsigned long long* conf,
                        const unsigned long long* n_valid, bool grad, bool assemble)
{
    const LossTiling lt = loss_tiling(g);
    const int n_tiles = g.n * lt.tiles();
    const int blocks = (n_tiles + 7) / 8 * 8;      // whole rounds over the eight XCDs
    if (grad) {
        ST_LAUNCH(c, "upsample_ce_grad", (k_loss<CP, CA, true>), dim3(blocks), dim3(LOSS_THREADS), 0, zs, labels, wmap, T, pred,
                  slots, loss_part, conf, g, lt, n_tiles);
        // the matrix-core backward kernel adds the slots itself; the plain path wants g assembled
        if (assemble)
            ST_LAUNCH(c, "assemble_dz", (k_assemble_g<CP>), dim3(cdiv((long long)g.n * g.C * g.h * g.w, 256)),
                      dim3(256), 0, (const float*)slots, T, n_valid, gz, g, lt);
    } else {
        ST_LAUNCH(c, "upsample_ce", (k_loss<CP, CA, false>), dim3(blocks), dim3(LOSS_THREADS), 0, zs, labels, wmap, T, pred, slots,
                  loss_part, conf, g, lt, n_tiles);
    }
}

#define ST_FOR_CP(CALL)                                                                       \
    switch (padded_classes(g.C)) {                                                            \
    case 4: CALL(4); break;                                                                   \
    case 8: CALL(8); break;                                                                   \
    case 12: CALL(12); break;                                                                 \
    case 16: CALL(16); break;                                                                 \
    case 20: CALL(20); break;                                                                 \
    case 24: CALL(24); break;                                                                 \
    case 28: CALL(28); break;                                                                 \
    case 32: CALL(32); break;                                                                 \
    default: c.status = ST_ERR_SHAPE; break;                                                  \
    }

void loss_pass(Ctx& c, const Geo& g, const ZSrc& zs, const uint8_t* labels, const uint8_t* wmap, const float* T,
               uint8_t* pred,
               float* slots, float* gz, float* loss_part, unsigned long long* conf,
               const unsigned long long* n_valid, bool grad, bool assemble)
{
#define ST_ARGS c, g, zs, labels, wmap, T, pred, slots, gz, loss_part, conf, n_valid, grad, assemble
#define ST_CALL(CP)                                                                           \
    switch (CP - g.C) {                                                                       \
    case 0: loss_launch<CP, CP>(ST_ARGS); break;                                              \
    case 1: loss_launch<CP, CP - 1>(ST_ARGS); break;                                          \
    case 2: loss_launch<CP, CP - 2>(ST_ARGS); break;                                          \
    default: loss_launch<CP, CP - 3>(ST_ARGS); break;                                         \
    }
    ST_FOR_CP(ST_CALL)
#undef ST_CALL
#undef ST_ARGS
}

}  // namespace st

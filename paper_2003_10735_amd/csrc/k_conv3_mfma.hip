// The 1x1 classifier layer on the matrix cores (bfloat16 operands, float32 accumulation).
//
// Forward:   z[img][c][pos] = b3[c] + sum_o a2[pos][o] * W3[c][o]            (float32, planar)
// Backward:  da2[pos][o]    = [a2[pos][o] > 0] * sum_c g[c][pos] * W3[c][o]
//            dW3[c][o]      = sum_pos g[c][pos] * a2[pos][o]
//            db3[c]         = sum_pos g[c][pos]
// with g = d loss / d z rounded to bfloat16 where it enters a product.  The class dimension
// (<= 32) is padded to one 32-row MFMA tile with zeros.
#include <string.h>

#include "st_kernels.hpp"
#include "st_mfma.hpp"
#include "st_finish.hpp"

namespace st {

typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

bool conv3_mfma_supported(int c2, int C) { return (c2 == 64 || c2 == 128 || c2 == 256) && C <= 32; }

// ------------------------------------------------------------------ backward
// One block = C3B_BP consecutive padded positions (g is zero on the border).  The block first
// forms g = d loss / d z for its cells from what the loss kernel left behind -- the per-tile slots
// of U^T softmax (added in a fixed order: tile rows first), minus U^T of the one-hot labels, over
// N_valid -- rounds it to bfloat16 and stages it in LDS in both orientations.  W3 comes transposed
// and padded to 32 classes from the optimiser kernel ([channel][32]), so its MFMA A fragments are
// 16-byte loads straight from memory.
// Then
//   wavefront w computes da2 for positions 32 (w % 2) .. +31 and half of the channel tiles
//   (K = classes),
//   wavefront w computes dW3 for channel tiles w, w+4, ..  over all positions (K = positions),
// so no sum crosses wavefronts.  Partial dW3 / db3 go to one slot per block; the optimiser
// kernel adds the slots in order (only the rows of real classes are stored).  The block's a2
// tile is loaded once, position-major, before the first barrier (its latency overlaps the
// staging of g) and kept in LDS: the ReLU mask is read from it directly, the dW3 operand
// through the transposing LDS read.
// The work per position is small and every phase is a chain of dependent memory round trips, so
// the block is kept small: the grid then covers the whole chip and each chain is short.
constexpr int C3B_BP = 64;

// (one or two wavefronts per SIMD are all this kernel asks for: said explicitly, because the
//  compiler otherwise keeps to 128 registers and then issues the slot loads one at a time)
//
// FIN (early-exit form of the training call): the blocks behind the first `main_blocks` do the
// bookkeeping of the forward pass that came before (finish_block: loss, per-frame mean IoU, the
// metric for the host) instead -- it touches nothing this kernel reads or writes, and riding
// along saves that pass a launch of its own.
template <int C2, bool FIN>
__global__ void __launch_bounds__(256, 1)
k_conv3_bwd_mfma(const float* __restrict__ slots, const float* __restrict__ T,
                 const unsigned long long* __restrict__ n_valid, int CP, LossTiling lt,
                 const bf16* __restrict__ a2,
                 const bf16* __restrict__ W3T, bf16* __restrict__ da2, bf16* __restrict__ da2T,
                 float* __restrict__ part, Geo g, int PPT, int guard, int grp_blocks, int main_blocks, FinishArgs fin)
{
    if (FIN && (int)blockIdx.x >= main_blocks) {
        finish_block<true>(fin, (int)blockIdx.x - main_blocks, 0);
        return;
    }
    constexpr int BP = C3B_BP;
    constexpr int OT = C2 / 32;            // channel tiles
    constexpr int OH = OT / 2;             // da2 channel tiles per wavefront
    constexpr int DW = (OT + 3) / 4;       // dW3 channel tiles per wavefront
    constexpr int KS = BP / 16;            // K steps of the dW3 product
    constexpr int GP = BP + 8;             // pitch of g_cp rows (positions)
    constexpr int GC = 32 + 8;             // pitch of g_pc rows (classes)
    constexpr int OLD = C2 + 8;            // pitch of the output tile
    static_assert(OT % 2 == 0, "two wavefronts share the channel tiles of a position half");
    __shared__ __attribute__((aligned(16))) bf16 g_cp[32 * GP];     // [class][position]
    __shared__ __attribute__((aligned(16))) bf16 g_pc[BP * GC];     // [position][class]
    __shared__ __attribute__((aligned(16))) bf16 Os[BP * OLD];      // da2 tile [position][channel]
    __shared__ __attribute__((aligned(16))) bf16 A2s[BP * OLD];     // a2 tile [position][channel]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, lhi = lane >> 5;
    const int PP = g.padded_positions(), frame = g.Hp * g.Wp, hw = g.h * g.w;
    // several heads: blocks are counted per frame (grp_blocks each), so that no block mixes the
    // positions -- and with them W3 and the partial sums -- of two heads
    const int head = g.grouped ? blockIdx.x / grp_blocks : 0;
    const int m0 = g.grouped ? head * frame + (blockIdx.x - head * grp_blocks) * BP : blockIdx.x * BP;
    const int m_end = g.grouped ? (head + 1) * frame : PP;
    W3T += (size_t)head * C2 * 32;

    // ---- early loads: the block's a2 tile (position-major, 16 bytes per load) on its way to LDS.
    //      Both uses take it from there: the ReLU mask of the da2 part, and the dW3 part, whose
    //      reduction runs over the positions and therefore wants 8 consecutive positions of one
    //      channel per lane -- the transposing LDS read hands out exactly that, so the layer-2
    //      convolution need not leave a channel-major copy of a2 behind.
    const int pm = (wave & 1) * 32 + l32;          // position (inside the block) for the da2 part
    const int t0 = (wave >> 1) * OH;               // first channel tile of the da2 part
    constexpr int A2_CHUNKS = BP * (C2 / 8) / 256; // 16-byte chunks of the tile per thread
    u32x4 a2v[A2_CHUNKS];
#pragma unroll
    for (int k = 0; k < A2_CHUNKS; ++k) {
        const int q = tid + 256 * k, p = q / (C2 / 8), part8 = q - p * (C2 / 8);
        // (rows past the last position repeat it: d loss / d z is zero there)
        a2v[k] = *(const u32x4*)(a2 + (size_t)min(m0 + p, PP - 1) * C2 + part8 * 8);
    }
    // W3^T fragments of this wavefront's da2 tiles: rows = channels, k = 16 classes per step
    bf16x8 wfr[OH][2];
#pragma unroll
    for (int t = 0; t < OH; ++t)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) wfr[t][ks] = *(const bf16x8*)(W3T + ((size_t)(t0 + t) * 32 + l32) * 32 + ks * 16 + lhi * 8);
    // ---- stage g (both orientations) and W3^T
    {
        const int p = tid & (BP - 1), cq = tid / BP;     // this thread: one position, every fourth class
        constexpr int NQ = 256 / BP;
        const int mp = m0 + p;
        const int img = min(mp / frame, g.n - 1), rr = mp - img * frame, y = rr / g.Wp, x = rr - y * g.Wp;
        const bool inside = mp < m_end && y >= 1 && y <= g.h && x >= 1 && x <= g.w;
        const int cy = inside ? y - 1 : 0, cx = inside ? x - 1 : 0;
        const unsigned long long nv = n_valid[head];
        const float inv_n = (inside && nv) ? 1.0f / (float)nv : 0.f;
        // the tiles whose cell window contains (cy, cx): up to 3 tile rows x 2 tile columns
        const int ty_hi = min((cy + 1) / LOSS_TY, lt.tiles_y - 1), tx_hi = min((cx + 1) / LOSS_TX, lt.tiles_x - 1);
        // slot offset of class 0 and a 0/1 weight: tiles that do not exist or do not touch the
        // cell read slot element 0 with weight 0, so that every load is unconditional
        int off[3][2];
        float wgt[3][2];
#pragma unroll
        for (int a = 0; a < 3; ++a)
#pragma unroll
            for (int b = 0; b < 2; ++b) {
                const int ty = ty_hi - 2 + a, tx = tx_hi - 1 + b;
                const int r = cy - (ty * LOSS_TY - 1), lc = cx - (tx * LOSS_TX - 1);
                const bool ok = inside && ty >= 0 && tx >= 0 && r >= 0 && r < LOSS_CH && lc >= 0 && lc < LOSS_CW;
                off[a][b] = ok ? (((img * lt.tiles() + ty * lt.tiles_x + tx) * CP) * LOSS_CH + r) * LOSS_CW + lc : 0;
                wgt[a][b] = ok ? 1.f : 0.f;
            }
        const int cstride = LOSS_CH * LOSS_CW;
        const size_t tbase = (size_t)img * g.C * hw + cy * g.w + cx;
        // all loads of the gather first (their addresses do not depend on each other), then the sums
        float sv[32 / NQ][6], tv[32 / NQ];
#pragma unroll
        for (int k = 0; k < 32 / NQ; ++k) {
            const int c = min(cq + NQ * k, g.C - 1);     // classes beyond C re-read the last one, unused
#pragma unroll
            for (int a = 0; a < 3; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b) sv[k][a * 2 + b] = slots[(size_t)off[a][b] + (size_t)c * cstride];
            tv[k] = T[tbase + (size_t)c * hw];
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int k = 0; k < 32 / NQ; ++k) {
            const int cc = cq + NQ * k;
            float v = 0.f;
#pragma unroll
            for (int a = 0; a < 3; ++a)
#pragma unroll
                for (int b = 0; b < 2; ++b) v = __builtin_fmaf(wgt[a][b], sv[k][a * 2 + b], v);
            v = (v - tv[k]) * inv_n;
            const bf16 q = (cc < g.C) ? (bf16)v : (bf16)0.f;
            g_cp[cc * GP + p] = q;
            g_pc[p * GC + cc] = q;
        }
    }
#pragma unroll
    for (int k = 0; k < A2_CHUNKS; ++k) {
        const int q = tid + 256 * k, p = q / (C2 / 8), part8 = q - p * (C2 / 8);
        *(u32x4*)(A2s + p * OLD + part8 * 8) = a2v[k];
    }
    __syncthreads();

    // ReLU mask of this lane's position
    bf16x4 mk[OH][4];
#pragma unroll
    for (int t = 0; t < OH; ++t)
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) mk[t][rg] = *(const bf16x4*)(A2s + pm * OLD + (t0 + t) * 32 + rg * 8 + lhi * 4);

    // ---- da2: D[o][pos] = sum_c W3T[o][c] * g[c][pos], two K steps cover 32 classes
    {
        f32x16 acc[OH];
#pragma unroll
        for (int t = 0; t < OH; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
            const bf16x8 gf = *(const bf16x8*)(g_pc + pm * GC + ks * 16 + lhi * 8);
#pragma unroll
            for (int t = 0; t < OH; ++t) {
                acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wfr[t][ks], gf, acc[t], 0, 0, 0);
            }
        }
        // (a2 is zero on the border, and g is zero there too: border rows of da2 come out zero)
#pragma unroll
        for (int t = 0; t < OH; ++t)
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                bf16x4 ov;
#pragma unroll
                for (int e = 0; e < 4; ++e) ov[e] = (bf16)((float)mk[t][rg][e] > 0.f ? acc[t][rg * 4 + e] : 0.f);
                *(bf16x4*)(Os + pm * OLD + (t0 + t) * 32 + rg * 8 + lhi * 4) = ov;
            }
    }

    // ---- dW3: D[c][o] = sum_pos g[c][pos] * a2[pos][o] over this block's positions
    float* slot = part + (size_t)blockIdx.x * (32 * C2 + 32);
#pragma unroll
    for (int d = 0; d < DW; ++d) {
        const int t = wave + 4 * d;
        if (t < OT) {
            f32x16 acc;
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const bf16x8 gf = *(const bf16x8*)(g_cp + l32 * GP + ks * 16 + lhi * 8);
                // B fragment: lane = channel l32 of tile t, positions 16 ks + 8 lhi .. + 7.  In a
                // group of 16 lanes, lane r names the row (position r / 4, channels 4 (r % 4) .. + 3)
                // and lane i receives channel i of positions 0 .. 3 of the group's rows: two reads.
                const bf16* row = A2s + (ks * 16 + lhi * 8 + ((lane & 15) >> 2)) * OLD + t * 32 + (lane & 16) + 4 * (lane & 3);
                const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)row);
                const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((s16x4 __attribute__((address_space(3)))*)(row + 4 * OLD));
                const s16x8 xs = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gf, __builtin_bit_cast(bf16x8, xs), acc, 0, 0, 0);
            }
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int c = (r >> 2) * 8 + lhi * 4 + (r & 3);
                if (c < g.C) slot[c * C2 + t * 32 + l32] = acc[r];    // (rows beyond the classes are never read)
            }
        }
    }
    if (tid < 32) {
        float s = 0.f;
        for (int p = 0; p < BP; ++p) s += (float)g_cp[tid * GP + p];
        if (tid < g.C) slot[32 * C2 + tid] = s;
    }
    __syncthreads();

    // ---- write the da2 tile: position-major rows and channel-major 8-position groups
    for (int q = tid; q < BP * (C2 / 8); q += 256) {
        const int p = q / (C2 / 8), part8 = q % (C2 / 8);
        if (m0 + p < m_end)
            *(uint4*)(da2 + (size_t)(m0 + p) * C2 + part8 * 8) = *(const uint4*)(Os + p * OLD + part8 * 8);
    }
    for (int q = tid; q < (BP / 8) * C2; q += 256) {
        const int o = q % C2, pg = q / C2;
        if (m0 + pg * 8 >= m_end) continue;
        bf16x8 ov;
#pragma unroll
        for (int e = 0; e < 8; ++e) ov[e] = Os[(pg * 8 + e) * OLD + o];
        *(bf16x8*)(da2T + xt_index(o, guard + m0 + pg * 8, PPT / 8)) = ov;
    }
}

// blocks (and partial-sum slots) per head
int conv3_bwd_blocks(const Geo& g) { return cdiv(g.padded_positions() / g.heads(), C3B_BP); }
size_t conv3_bwd_slot_floats(const Geo& g) { return (size_t)32 * g.c2 + 32; }

void conv3_bwd_mfma(Ctx& c, const Plan& p, const float* slots, const float* T,
                    const unsigned long long* n_valid, const bf16* a2, const bf16* W3T,
                    bf16* da2, bf16* da2T, float* part, const FinishArgs* finish)
{
    const Geo& g = p.g;
    const int grp_blocks = conv3_bwd_blocks(g);
    const int main_blocks = g.heads() * grp_blocks;
    const int CP = (g.C + 3) / 4 * 4;   // class padding of the loss kernel's slots
    FinishArgs fin;
    memset(&fin, 0, sizeof(fin));
    if (finish) {
        if (g.grouped) { c.status = ST_ERR_ARG; return; }   // (the riding role serves one head)
        fin = *finish;
    }
    // with `finish`: one more block per frame and one for the loss
    const dim3 grid(main_blocks + (finish ? fin.fph + 1 : 0));
#define ST_C3B(C2)                                                                                             \
    do {                                                                                                       \
        if (finish)                                                                                            \
            ST_LAUNCH(c, "conv3_bwd_mfma+finish_pass", (k_conv3_bwd_mfma<C2, true>), grid, dim3(256), 0, slots, T,   \
                      n_valid, CP, p.lt, a2, W3T, da2, da2T, part, g, p.PPT, p.guard, grp_blocks, main_blocks, fin); \
        else                                                                                                   \
            ST_LAUNCH(c, "conv3_bwd_mfma", (k_conv3_bwd_mfma<C2, false>), grid, dim3(256), 0, slots, T, n_valid, CP, \
                      p.lt, a2, W3T, da2, da2T, part, g, p.PPT, p.guard, grp_blocks, main_blocks, fin);    \
    } while (0)
    switch (g.c2) {
    case 64: ST_C3B(64); break;
    case 128: ST_C3B(128); break;
    case 256: ST_C3B(256); break;
    default: c.status = ST_ERR_SHAPE;
    }
#undef ST_C3B
}

}  // namespace st

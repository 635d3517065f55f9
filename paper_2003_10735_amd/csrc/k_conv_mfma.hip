// 3x3 convolution (forward, and data-gradient as a forward with mirrored taps) as an implicit
// GEMM on the gfx950 matrix cores: bfloat16 operands, float32 accumulation
// (v_mfma_f32_32x32x16_bf16).
//
//   out[mp][n] = epi( sum_{kh,kw,c} X[mp + (kh-1)*Wp + (kw-1)][c] * W[n][kh*3+kw][c] )
//
// X is position-major on the zero-padded grid, so a tap is a constant row offset and the GEMM's
// M index can simply walk the padded positions mp = 0 .. PP-1 linearly (results at border
// positions are forced to zero, which keeps the border of the output zero as well).  Guard rows
// in front of and behind every activation buffer make all reads in-bounds without tests.
//
// Block = 512 threads = 8 wavefronts, tile = 128 positions x 64 output channels.  The LDS
// pipeline is the scarce resource of this kernel (a tile is small, so every byte staged is used
// only a few times), hence the two operands take different routes:
//   * the weights are the MFMA A operand (rows = output channels) and never touch LDS: they are
//     kept in memory in fragment order (wfrag_index), so a wavefront fetches the fragment it
//     needs with one coalesced 1 KB load straight into the operand registers, and no two
//     wavefronts of a block need the same fragment;
//   * the activations are the B operand (columns = positions) and go through LDS, because the
//     three taps kw = 0,1,2 of a kernel row read the same slab at row offsets 0,1,2.
// Wavefront (wn, kgrp): output channels 32 wn .. +31 of the tile, all 128 positions (four
// accumulator tiles), and of every 64-channel stage the 16 input channels 16 kgrp .. +15.  The
// four partial sums per output are exchanged once, through LDS, after the K loop: wavefront
// (wn, kgrp) ends up owning positions 32 kgrp .. +31 and adds the partials in ascending kgrp.
// K loop: stages of (one kernel row kh) x (64 input channels): 130 activation rows in LDS (the
// tile's rows shifted by kh, plus one on each side), rows padded by 16 bytes so that the 16-byte
// fragment reads of 32 consecutive rows spread over all banks.  Loads run two stages ahead of
// the matrix cores (global -> registers at stage s-2, registers -> LDS at stage s-1).
//
// A lane owns 4 consecutive output channels of one position per register group, which packs
// into one 8-byte LDS write in the epilogue.  The epilogue stages the tile in LDS and writes it
// twice with 16-byte stores: position-major (input of the next convolution) and channel-major
// (operand of the weight-gradient kernel).  For the layer that feeds the 1x1 classifier the
// staged tile is also multiplied with the classifier's weights (16 more MFMAs per block), which
// saves the classifier a launch and a pass over the activations.
#include "st_kernels.hpp"
#include "st_mfma.hpp"

namespace st {

constexpr int CV_BM = 128;
constexpr int CV_BN = 64;
constexpr int CV_BK = 64;
constexpr int CV_LDP = CV_BK + 8;   // LDS row pitch in elements (144 bytes)
constexpr int CV_XS_ROWS = CV_BM + 2;
constexpr int CV_OLD = CV_BN + 8;   // pitch of the staged output tile
// dynamic LDS: during the K loop two activation slabs; afterwards the exchanged partial sums
// (8 owners x 3 sources x 16 registers x 64 lanes, float32) followed by the staged output tile
constexpr size_t CV_RED_BYTES = (size_t)8 * 3 * 16 * 64 * sizeof(float);
constexpr size_t CV_SMEM_BYTES = CV_RED_BYTES + (size_t)CV_BM * CV_OLD * sizeof(bf16);
static_assert((size_t)2 * CV_XS_ROWS * CV_LDP * sizeof(bf16) <= CV_SMEM_BYTES, "K-loop buffers fit");

struct ConvArgs {
    const bf16* X;      // [PP][cin] position-major, guards before/after
    const bf16* Wq;     // fragment order, see wfrag_index(): rows = cout, K = cin
    const float* bias;  // EPI 0
    const bf16* mask;   // EPI 1: activation whose sign gates the gradient, [PP][cout]
    bf16* Y;            // [PP][cout] or nullptr
    bf16* YT;           // channel-major copy, blocked layout of xt_index(), or nullptr
    // EPI 2: the 1x1 classifier rides along.  Every block adds its 64 channels' share of the
    // logits of its 128 positions: zpart[n-tile][padded position][32 classes] float32; the
    // consumer adds the n_tiles shares and the bias.
    const bf16* W3q;    // [n_cls][cout] bfloat16
    float* zpart;
    int n_cls;
    // EPI 3: the plain sums go, as float32, straight to a dense [n][cout][h][w] tensor
    float* dense;
    int PP, Hp, Wp, h, w, cin, cout, PPT, guard;
    int m_tiles, n_tiles, tiles_per_xcd;
    // Several heads: positions [k * grp_pp, (k + 1) * grp_pp) use weight set k (Wq, bias and W3q
    // advance by wq_stride, bias_stride, w3_stride elements per set); position tiles are counted
    // per set (grp_tiles each) so that no tile mixes two sets.  One head: grp_pp = PP.
    int grp_pp, grp_tiles;
    size_t wq_stride, bias_stride, w3_stride;
};

// TAG only gives every call site (layer 1 forward, layer 2 forward, layer 2 data-gradient) a
// kernel symbol of its own, so that profiles list them separately.
template <int EPI, int TAG>
__global__ void __launch_bounds__(512) k_conv3x3_mfma(ConvArgs a)
{
    constexpr int NT = 512;                // threads per block
    // 16-byte chunks per stage: XS_FULL per thread and one more for the first XS_REST threads
    constexpr int XS_CHUNKS = CV_XS_ROWS * 8;
    constexpr int XS_FULL = XS_CHUNKS / NT, XS_REST = XS_CHUNKS % NT;
    constexpr int XS_PER_T = XS_FULL + 1;
    constexpr int XS_ELEMS = CV_XS_ROWS * CV_LDP;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    bf16* Xs = (bf16*)smem_raw;                       // [2][XS_ROWS][LDP]

    // XCD-aware tile order: consecutive blocks go to different XCDs, so give each XCD a
    // contiguous run of position tiles (neighbours share activation rows in that XCD's L2)
    const int xcd = blockIdx.x % 8, slot = blockIdx.x / 8;
    const int tile = xcd * a.tiles_per_xcd + slot;
    if (slot >= a.tiles_per_xcd || tile >= a.m_tiles * a.n_tiles) return;
    const int mt = tile / a.n_tiles, nt = tile % a.n_tiles;
    const int grp = mt / a.grp_tiles;
    const int m0 = grp * a.grp_pp + (mt - grp * a.grp_tiles) * CV_BM, n0 = nt * CV_BN;
    const int m_end = (grp + 1) * a.grp_pp;     // results from here on belong to another tile

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wn = wave & 1, kgrp = wave >> 1;
    const int l32 = lane & 31, lhi = lane >> 5;

    f32x16 acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;

    const int c_chunks = a.cin / CV_BK;
    const int n_stages = 3 * c_chunks;
    const int kfr = a.cin >> 4;                                   // 16-channel fragments per tap
    // this wavefront's block of 32 output channels (clamped: a half tile beyond cout computes
    // a copy of the last block and drops it in the epilogue)
    const int nb = min((n0 >> 5) + wn, (a.cout >> 5) - 1);
    const bf16* wbase = a.Wq + grp * a.wq_stride + ((size_t)nb * 9 * kfr + kgrp) * 512 + lane * 8;

    u32x4 xr[2][XS_PER_T];   // activations on their way to LDS
    u32x4 wr[2][3];          // weight fragments of the three taps of a stage

#define CV_LOAD_X1(SET, S, I)                                                                     \
    if ((I) < XS_FULL || tid < XS_REST) {                                                         \
        const int kh_ = (S) / c_chunks, c0_ = ((S) % c_chunks) * CV_BK;                           \
        const bf16* src_ = a.X + ((long long)m0 - 1 + (long long)(kh_ - 1) * a.Wp) * a.cin + c0_; \
        const int q = tid + (I) * NT;                                                             \
        xr[SET][I] = *(const u32x4*)(src_ + (long long)(q >> 3) * a.cin + (q & 7) * 8);           \
    }
#define CV_LOAD_X(SET, S) CV_LOAD_X1(SET, S, 0) CV_LOAD_X1(SET, S, 1) CV_LOAD_X1(SET, S, 2)
#define CV_LOAD_W(SET, S, KW)                                                                     \
    {                                                                                             \
        const int kh_ = (S) / c_chunks, kc_ = ((S) % c_chunks) * (CV_BK / 16);                    \
        wr[SET][KW] = *(const u32x4*)(wbase + ((size_t)(kh_ * 3 + (KW)) * kfr + kc_) * 512);      \
    }
#define CV_STORE1(SET, BUF, I)                                                                    \
    if ((I) < XS_FULL || tid < XS_REST) {                                                         \
        const int q = tid + (I) * NT;                                                             \
        *(u32x4*)(Xs + (BUF) * XS_ELEMS + (q >> 3) * CV_LDP + (q & 7) * 8) = xr[SET][I];          \
    }
#define CV_READ1(DST, J, BUF, KW)                                                                 \
    DST[J] = *(const bf16x8*)(Xs + (BUF) * XS_ELEMS + ((J) * 32 + l32 + (KW)) * CV_LDP + kgrp * 16 + lhi * 8);
#define CV_MMA1(SRC, J, SET, KW)                                                                  \
    acc[J] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wr[SET][KW]), SRC[J], acc[J], 0, 0, 0);
    // One stage S out of LDS buffer BUF and register set SET; meanwhile the activations of
    // stage S + 2 start their way into set SET, those of stage S + 1 (set 1 - SET) move to the
    // other buffer, and each weight register is refilled for stage S + 2 as soon as its tap is
    // done.  The issue order is pinned: the eight wavefronts run in step (a barrier per stage),
    // so a run of memory instructions would hit the LDS and vector-memory queues from all of
    // them at once while the matrix cores idle.  Instead every MFMA is followed by at most two
    // memory instructions, which issue while it executes; the activation fragments of a tap
    // (fragment sets xa, xb) are read while the tap before it is being multiplied.
    // (loads and LDS stores are unconditional, with the stage index clamped to the last stage:
    //  a load under a branch would force a wait for every outstanding load at the join; the
    //  redundant copies at the tail land where nobody reads any more)
#define CV_F __builtin_amdgcn_sched_barrier(0);
#define CV_STAGE(S, SET, BUF)                                                                     \
    {                                                                                             \
        const int s2_ = min((S) + 2, last);                                                       \
        CV_READ1(xa, 0, BUF, 0) CV_READ1(xa, 1, BUF, 0) CV_READ1(xa, 2, BUF, 0) CV_READ1(xa, 3, BUF, 0) \
        CV_READ1(xb, 0, BUF, 1) CV_F                                                              \
        CV_MMA1(xa, 0, SET, 0) CV_F CV_LOAD_X1(SET, s2_, 0) CV_READ1(xb, 1, BUF, 1) CV_F          \
        CV_MMA1(xa, 1, SET, 0) CV_F CV_LOAD_X1(SET, s2_, 1) CV_READ1(xb, 2, BUF, 1) CV_F          \
        CV_MMA1(xa, 2, SET, 0) CV_F CV_LOAD_X1(SET, s2_, 2) CV_READ1(xb, 3, BUF, 1) CV_F          \
        CV_MMA1(xa, 3, SET, 0) CV_F CV_LOAD_W(SET, s2_, 0) CV_F                                   \
        CV_MMA1(xb, 0, SET, 1) CV_F CV_READ1(xa, 0, BUF, 2) CV_F                                  \
        CV_MMA1(xb, 1, SET, 1) CV_F CV_READ1(xa, 1, BUF, 2) CV_F                                  \
        CV_MMA1(xb, 2, SET, 1) CV_F CV_READ1(xa, 2, BUF, 2) CV_F                                  \
        CV_MMA1(xb, 3, SET, 1) CV_F CV_READ1(xa, 3, BUF, 2) CV_LOAD_W(SET, s2_, 1) CV_F           \
        CV_MMA1(xa, 0, SET, 2) CV_F CV_STORE1(1 - (SET), 1 - (BUF), 0) CV_F                       \
        CV_MMA1(xa, 1, SET, 2) CV_F CV_STORE1(1 - (SET), 1 - (BUF), 1) CV_F                       \
        CV_MMA1(xa, 2, SET, 2) CV_F CV_STORE1(1 - (SET), 1 - (BUF), 2) CV_F                       \
        CV_MMA1(xa, 3, SET, 2) CV_F CV_LOAD_W(SET, s2_, 2)                                        \
        __syncthreads();                                                                          \
    }
    static_assert(XS_PER_T == 3, "the stage sequence places three activation stores");

    bf16x8 xa[4], xb[4];
    const int last = n_stages - 1;
    {
        const int s1 = min(1, last);
        CV_LOAD_X(0, 0)
        CV_LOAD_W(0, 0, 0) CV_LOAD_W(0, 0, 1) CV_LOAD_W(0, 0, 2)
        CV_LOAD_X(1, s1)
        CV_LOAD_W(1, s1, 0) CV_LOAD_W(1, s1, 1) CV_LOAD_W(1, s1, 2)
        CV_STORE1(0, 0, 0) CV_STORE1(0, 0, 1) CV_STORE1(0, 0, 2)
        __syncthreads();
    }
    // Two stages per trip, so that register sets and LDS buffers are compile-time choices; an
    // odd stage count runs its last stage after the loop.  (One loop with an exit in the middle
    // would do, but the accumulators then live across two different exits and get copied around
    // every stage.)
    for (int s = 0; s + 1 < n_stages; s += 2) {
        CV_STAGE(s, 0, 0)
        CV_STAGE(s + 1, 1, 1)
    }
    if (n_stages & 1) CV_STAGE(last, 0, 0)
#undef CV_STAGE
#undef CV_LOAD_X
#undef CV_LOAD_X1
#undef CV_LOAD_W
#undef CV_STORE1
#undef CV_READ1
#undef CV_MMA1
#undef CV_F

    // ---- exchange of the partial sums: accumulator tile j of every wavefront goes to the
    //      wavefront (wn, kgrp = j), which adds the four partials in ascending source order
    float* red = (float*)smem_raw;   // [owner = j * 2 + wn][source slot 0..2][16][64]
    // (all wavefronts are past the last barrier of the K loop: the slabs are free)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        if (j != kgrp) {
            const int src = kgrp - (kgrp > j ? 1 : 0);
            float* dst = red + ((size_t)((j * 2 + wn) * 3 + src) * 16) * 64 + lane;
#pragma unroll
            for (int r = 0; r < 16; ++r) dst[r * 64] = acc[j][r];
        }
    }
    f32x16 mine = kgrp == 0 ? acc[0] : kgrp == 1 ? acc[1] : kgrp == 2 ? acc[2] : acc[3];
    __syncthreads();
    {
        f32x16 sum;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            f32x16 term;
            if (k == kgrp) term = mine;
            else {
                const float* srcp = red + ((size_t)((kgrp * 2 + wn) * 3 + (k - (k > kgrp ? 1 : 0))) * 16) * 64 + lane;
#pragma unroll
                for (int r = 0; r < 16; ++r) term[r] = srcp[r * 64];
            }
            if (k == 0) sum = term;
            else
#pragma unroll
                for (int r = 0; r < 16; ++r) sum[r] += term[r];
        }
        mine = sum;
    }

    if (EPI == 3) {
        // a lane holds 16 channels of one position; for a fixed channel the 32 lanes of a half
        // wavefront are 32 consecutive positions, i.e. (inside one grid row) consecutive floats
        const int frame = a.Hp * a.Wp;
        const int mp = m0 + kgrp * 32 + l32;
        const int img = mp / frame, rr = mp - img * frame, y = rr / a.Wp, x = rr - y * a.Wp;
        if (mp < m_end && y >= 1 && y <= a.h && x >= 1 && x <= a.w) {
            float* dst = a.dense + ((size_t)img * a.cout * a.h + (y - 1)) * a.w + (x - 1);
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int ch = n0 + wn * 32 + (r >> 2) * 8 + lhi * 4 + (r & 3);
                if (ch < a.cout) dst[(size_t)ch * a.h * a.w] = mine[r];
            }
        }
        return;
    }

    // classifier fragments (A operand: rows = classes, k = 16 channels of this tile), fetched
    // now so that they arrive while the tile is being staged
    u32x4 w3f[4];
    if (EPI == 2) {
        const bf16* w3row = a.W3q + grp * a.w3_stride + (size_t)min(l32, a.n_cls - 1) * a.cout + n0 + lhi * 8;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const u32x4 v = *(const u32x4*)(w3row + ks * 16);
            w3f[ks] = l32 < a.n_cls ? v : u32x4{0u, 0u, 0u, 0u};
        }
    }

    // ---- epilogue: bias + ReLU (forward) or ReLU mask (data-gradient), zero outside the grid,
    //      round to bfloat16, stage the tile in LDS as [position][channel]
    bf16* Os = (bf16*)(smem_raw + CV_RED_BYTES);     // [CV_BM][CV_OLD], behind the partial sums
    {
        const int frame = a.Hp * a.Wp;
        const int p = kgrp * 32 + l32;
        const int mp = m0 + p;
        const int rr = mp % frame, y = rr / a.Wp, x = rr - y * a.Wp;
        const bool inside = mp < m_end && y >= 1 && y <= a.h && x >= 1 && x <= a.w;
        const float* bias = (EPI == 0 || EPI == 2) ? a.bias + grp * a.bias_stride : nullptr;
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
            const int c = wn * 32 + rg * 8 + lhi * 4;   // channel inside the tile
            const int cg = min(n0 + c, a.cout - 4);
            float v[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = mine[rg * 4 + e];
            if (EPI == 0 || EPI == 2) {
                const float4 b = *(const float4*)(bias + cg);
                v[0] = fmaxf(v[0] + b.x, 0.f); v[1] = fmaxf(v[1] + b.y, 0.f);
                v[2] = fmaxf(v[2] + b.z, 0.f); v[3] = fmaxf(v[3] + b.w, 0.f);
            } else {
                bf16x4 mk = {(bf16)0.f, (bf16)0.f, (bf16)0.f, (bf16)0.f};
                if (inside) mk = *(const bf16x4*)(a.mask + (size_t)mp * a.cout + cg);
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = (float)mk[e] > 0.f ? v[e] : 0.f;
            }
            bf16x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) o[e] = (bf16)(inside ? v[e] : 0.f);
            *(bf16x4*)(Os + p * CV_OLD + c) = o;
        }
    }
    __syncthreads();
    if (EPI == 2 && wave < 4) {
        // D[class][position] for positions 32 wave .. +31 over the tile's 64 channels
        f32x16 zacc;
#pragma unroll
        for (int r = 0; r < 16; ++r) zacc[r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            const bf16x8 xf = *(const bf16x8*)(Os + (wave * 32 + l32) * CV_OLD + ks * 16 + lhi * 8);
            zacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, w3f[ks]), xf, zacc, 0, 0, 0);
        }
        const int mp = m0 + wave * 32 + l32;
        if (mp < m_end) {
            float* zrow = a.zpart + ((size_t)nt * a.PP + mp) * 32 + lhi * 4;
#pragma unroll
            for (int gq = 0; gq < 4; ++gq)
                *(f32x4*)(zrow + gq * 8) = f32x4{zacc[gq * 4], zacc[gq * 4 + 1], zacc[gq * 4 + 2], zacc[gq * 4 + 3]};
        }
    }
    const int n_valid = min(CV_BN, a.cout - n0);
    if (a.Y) {
        // position-major: 16 bytes = 8 channels of one position
        for (int q = tid; q < CV_BM * (CV_BN / 8); q += NT) {
            const int p = q / (CV_BN / 8), part = q % (CV_BN / 8);
            if (m0 + p < m_end && part * 8 < n_valid)
                *(uint4*)(a.Y + (size_t)(m0 + p) * a.cout + n0 + part * 8) = *(const uint4*)(Os + p * CV_OLD + part * 8);
        }
    }
    if (a.YT) {
        // channel-major: 16 bytes = 8 consecutive positions of one channel
        for (int q = tid; q < (CV_BM / 8) * CV_BN; q += NT) {
            const int c = q % CV_BN, pg = q / CV_BN;
            if (c < n_valid && m0 + pg * 8 < m_end) {
                bf16x8 o;
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] = Os[(pg * 8 + e) * CV_OLD + c];
                *(bf16x8*)(a.YT + xt_index(n0 + c, a.guard + m0 + pg * 8, a.PPT / 8)) = o;
            }
        }
    }
}

bool conv3x3_mfma_supported(int cin, int cout) { return cin % CV_BK == 0 && cout % 32 == 0 && cout >= 32; }

// epi 0: Y = relu(conv + bias); epi 1: Y = conv * [mask > 0]; with W3q / zpart (epi 0, cout a
// multiple of 64) the block also leaves its share of the classifier's logits; epi 3: the plain
// sums as float32 to the dense tensor `dense` [n][cout][h][w]
void conv3x3_mfma(Ctx& c, const char* name, const Plan& p, const bf16* X, const bf16* Wq, const float* bias,
                  const bf16* mask, bf16* Y, bf16* YT, int cin, int cout, int epi, int layer, const bf16* W3q,
                  float* zpart, float* dense)
{
    const Geo& g = p.g;
    ConvArgs a;
    a.X = X; a.Wq = Wq; a.bias = bias; a.mask = mask; a.Y = Y; a.YT = YT;
    a.W3q = W3q; a.zpart = zpart; a.n_cls = p.g.C; a.dense = dense;
    a.PP = p.g.padded_positions(); a.Hp = p.g.Hp; a.Wp = p.g.Wp; a.h = p.g.h; a.w = p.g.w;
    a.cin = cin; a.cout = cout;
    a.PPT = p.PPT; a.guard = p.guard;
    // several heads: one weight set per frame (Wq holds them back to back, the biases sit
    // head_stride floats apart inside the parameter vectors, W3q back to back)
    a.grp_pp = g.grouped ? g.Hp * g.Wp : a.PP;
    a.grp_tiles = cdiv(a.grp_pp, CV_BM);
    a.wq_stride = (size_t)cin * cout * 9;
    a.bias_stride = p.head_stride;
    a.w3_stride = (size_t)g.C * cout;
    a.m_tiles = g.heads() * a.grp_tiles;
    a.n_tiles = cdiv(cout, CV_BN);
    const int tiles = a.m_tiles * a.n_tiles;
    a.tiles_per_xcd = cdiv(tiles, 8);
    const dim3 grid(a.tiles_per_xcd * 8);
    const size_t smem = CV_SMEM_BYTES;
    // tag 1: layer-1 forward, 2: layer-2 forward, 3: layer-2 data-gradient
    auto go = [&](auto kernel) {
        ensure_dynamic_lds((const void*)kernel, smem);
        ST_LAUNCH(c, name, kernel, grid, dim3(512), smem, a);
    };
    if (epi == 3) go(k_conv3x3_mfma<3, 4>);
    else if (epi == 1) go(k_conv3x3_mfma<1, 3>);
    else if (zpart) go(k_conv3x3_mfma<2, 2>);
    else if (layer == 1) go(k_conv3x3_mfma<0, 1>);
    else go(k_conv3x3_mfma<0, 2>);
}

}  // namespace st

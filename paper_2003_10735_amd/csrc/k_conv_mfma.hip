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
// Block = 512 threads = 8 wavefronts, tile = 128 positions x 64 output channels.  A tile is
// small (every byte staged is used only a few times), and the matrix cores, the LDS read path,
// the vector-memory path and plain instruction issue are all close to full in the K loop; so the
// two operands take different routes and the loop is written to issue as little as possible:
//   * the weights are the MFMA A operand (rows = output channels) and never touch LDS: they are
//     kept in memory in fragment order (wfrag_index), so a wavefront fetches the fragment it
//     needs with one coalesced 1 KB buffer load straight into the operand registers (buffer
//     descriptor + fixed lane offset + one scalar offset per stage: no address arithmetic), and
//     no two wavefronts of a block need the same fragment;
//   * the activations are the B operand (columns = positions) and go through LDS, because the
//     three taps kw = 0,1,2 of a kernel row read the same slab at row offsets 0,1,2.  They are
//     loaded from memory directly into LDS (no registers, no LDS store instructions).
// Wavefront (wn, kgrp): output channels 32 wn .. +31 of the tile, all 128 positions (four
// accumulator tiles), and of every 64-channel stage the 16 input channels 16 kgrp .. +15.  The
// four partial sums per output are exchanged once, through LDS, after the K loop: wavefront
// (wn, kgrp) ends up owning positions 32 kgrp .. +31 and adds the partials in ascending kgrp.
// K loop: stages of (one kernel row kh) x (64 input channels): 130 activation rows in LDS (the
// tile's rows shifted by kh, plus one on each side) of 128 bytes, their 16-byte chunks swizzled
// by the row number so that the fragment reads of 16 consecutive rows spread over all banks.  Three
// slabs and three sets of weight registers rotate: loads run two stages ahead of the matrix cores.
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
constexpr int CV_NBUF = 3;          // activation slabs in LDS: one in use, two on their way
constexpr int CV_XS_ROWS = CV_BM + 2;
constexpr int CV_OLD = CV_BN + 8;   // pitch of the staged output tile
// dynamic LDS: during the K loop the activation slabs; afterwards the exchanged partial sums
// (8 owners x 3 sources x 16 registers x 64 lanes, float32) followed by the staged output tile
constexpr size_t CV_RED_BYTES = (size_t)8 * 3 * 16 * 64 * sizeof(float);
constexpr size_t CV_SMEM_BYTES = CV_RED_BYTES + (size_t)CV_BM * CV_OLD * sizeof(bf16);
static_assert((size_t)CV_NBUF * CV_XS_ROWS * CV_BK * sizeof(bf16) <= CV_SMEM_BYTES, "K-loop buffers fit");

struct ConvArgs {
    const bf16* X;      // [PP][cin] position-major, guards before/after
    const bf16* Wq;     // fragment order, see wfrag_index(): rows = cout, K = cin
    const float* bias;  // EPI 0
    const bf16* mask;   // EPI 1: activation whose sign gates the gradient, [PP][cout]
    bf16* Y;            // [PP][cout] or nullptr
    bf16* YT;           // channel-major copy, blocked layout of xt_index(), or nullptr
    // EPI 2: the 1x1 classifier rides along.  Every block adds its 64 channels' share of the
    // logits of its 128 positions: zpart[n-tile][padded position][zpitch classes] float32 (zpitch =
    // the class count rounded up to a multiple of four); the consumer adds the n_tiles shares and
    // the bias.
    const bf16* W3q;    // [n_cls][cout] bfloat16
    float* zpart;
    int n_cls, zpitch;
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
    constexpr int XS_BYTES = CV_XS_ROWS * CV_BK * 2;   // one slab: 130 rows of 64 channels, unpadded
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    // smem_raw during the K loop: [CV_NBUF][XS_ROWS][128 bytes], chunks swizzled

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

    u32x4 wr[3][3];          // weight fragments of the three taps of a stage: in use, and two stages ahead

    // ---- activations: global memory -> LDS without passing through registers.  A wavefront-wide
    // 16-byte load puts lane l's bytes at (LDS base in M0) + 16 l, so one instruction fills eight
    // consecutive 128-byte rows (64 channels) of a slab.  Rows filled this way cannot be padded;
    // instead the 16-byte chunk c of row r is kept at chunk position c ^ ((r >> 1) & 7).  LDS
    // serves 16 lanes of a 16-byte read per cycle (64 banks): the 16 consecutive rows they read
    // are 8 even rows (banks 0-31) and 8 odd rows (banks 32-63), and within each group the eight
    // values of (r >> 1) & 7 differ, so the reads spread over all banks just as padded rows
    // would.  The lane that fills position pc of row r fetches chunk pc ^ ((r >> 1) & 7).
    // Wavefront w fills rows 8w .. 8w+7 and 64+8w .. 64+8w+7; wavefront 0 also rows 128, 129.
    // The loads are written in assembly: the compiler would order every barrier behind all
    // outstanding loads of this kind, while the pipeline below needs two stages in flight.
    // (M0 is a reserved register for this compiler: it never allocates a value to it, sets it
    //  right before each instruction of its own that reads it, and rejects it in an asm clobber
    //  list ("inline asm clobber list contains reserved registers: m0") -- so the statement
    //  below cannot declare the write and does not need to: nothing of the compiler's lives in M0
    //  across it, and each statement sets M0 itself before the one load that reads it.  One wait
    //  state separates the scalar write of M0 from that load.)
    const int lrow = lane >> 3, lpc = lane & 7;
    const int sw01 = (4 * wave + (lrow >> 1)) & 7, sw2 = lrow >> 1;          // (row >> 1) & 7 of the rows filled
    const int xo0 = ((wave * 8 + lrow) * a.cin + ((lpc ^ sw01) << 3)) * 2;   // byte offsets inside a slab
    const int xo1 = xo0 + 64 * a.cin * 2;
    const int xo2 = ((128 + lrow) * a.cin + ((lpc ^ sw2) << 3)) * 2;
    const bf16* xg = a.X + ((long long)m0 - 1 - a.Wp) * a.cin;               // first row of the kh = 0 slabs
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)smem_raw;
    const unsigned wave_lds = __builtin_amdgcn_readfirstlane(wave * 1024);   // a scalar: it goes to M0
    // fragment reads: row J*32 + l32 + KW, chunk kgrp*2 + lhi
    int rd[3];
#pragma unroll
    for (int kw = 0; kw < 3; ++kw) rd[kw] = (l32 + kw) * 128 + (((kgrp * 2 + lhi) ^ (((l32 + kw) >> 1) & 7)) << 4);

    // The stage being fetched runs two ahead of the one being multiplied.  Its operands are
    // addressed as (scalar base, advanced once per stage) + (per-lane byte offset, fixed), which
    // costs no vector instruction and two scalar ones per stage.
    const char* xsp = (const char*)xg;                                      // activations of the stage
    // (weights through a buffer descriptor: base in scalar registers, a fixed per-lane offset and
    //  a scalar offset per stage, so that a weight load needs no address arithmetic at all)
    const __amdgpu_buffer_rsrc_t wrsrc = __builtin_amdgcn_make_buffer_rsrc(
        (void*)(a.Wq + grp * a.wq_stride), 0, (int)(a.wq_stride * 2), 0x00020000);
    int w_soff = 0;                                                          // weights of the stage
    unsigned wv[3];
#pragma unroll
    for (int kw = 0; kw < 3; ++kw) wv[kw] = (unsigned)((((nb * 9 + kw) * kfr + kgrp) * 512 + lane * 8) * 2);
    const long long x_step = CV_BK * 2, x_row = ((long long)a.Wp * a.cin - (c_chunks - 1) * CV_BK) * 2;
    const int w_step = (CV_BK / 16) * 512 * 2, w_row = (2 * kfr + CV_BK / 16) * 512 * 2;
    int f_cc = 0;
#define CV_FETCH_NEXT                                                                             \
    if (++f_cc == c_chunks) { f_cc = 0; xsp += x_row; w_soff += w_row; } else { xsp += x_step; w_soff += w_step; }
#define CV_DMA(VOFF, LDSADDR)                                                                     \
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(VOFF), "s"(xsp), \
                 "s"(LDSADDR) : "memory");
#define CV_LOAD_X1(BUF, I)                                                                        \
    {                                                                                             \
        if ((I) == 0) CV_DMA(xo0, lds0 + (BUF) * XS_BYTES + wave_lds)                             \
        if ((I) == 1) CV_DMA(xo1, lds0 + (BUF) * XS_BYTES + 8192 + wave_lds)                      \
        if ((I) == 2 && wave == 0 && lane < 16) CV_DMA(xo2, lds0 + (BUF) * XS_BYTES + 16384)      \
    }
#define CV_LOAD_W(SET, KW) wr[SET][KW] = __builtin_amdgcn_raw_buffer_load_b128(wrsrc, wv[KW], w_soff, 0);
#define CV_READ1(DST, J, BUF, KW)                                                                 \
    DST[J] = *(const bf16x8*)(smem_raw + (BUF) * XS_BYTES + rd[KW] + (J) * 4096);
#define CV_MMA1(SRC, J, SET, KW)                                                                  \
    acc[J] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, wr[SET][KW]), SRC[J], acc[J], 0, 0, 0);
    // s_waitcnt vmcnt(N) alone (gfx9 encoding: vmcnt in bits 3:0 and 15:14, no wait on the others)
#define CV_VMCNT(N) __builtin_amdgcn_s_waitcnt(((N) & 15) | (((N) >> 4) << 14) | 0x0F70);
    // One stage out of LDS slab and weight register set B.  With FETCH, the activations and
    // weights of the stage two ahead start their way into slab / set (B + 2) % 3, which the stage
    // before this one used last; the loads are spread over the stage, one after every other
    // MFMA.  Before the barrier that ends the stage every wavefront waits until its own share of
    // the next stage's slab has landed: everything but the five (wavefront 0: six) loads issued
    // during this stage, or simply everything when the stage issued none.
#define CV_F __builtin_amdgcn_sched_barrier(0);
#define CV_STAGE(B, FETCH)                                                                        \
    {                                                                                             \
        constexpr int N_ = ((B) + 2) % 3;                                                         \
        CV_READ1(xa, 0, B, 0) CV_READ1(xa, 1, B, 0) CV_READ1(xa, 2, B, 0) CV_READ1(xa, 3, B, 0)   \
        CV_READ1(xb, 0, B, 1) CV_F                                                                \
        CV_MMA1(xa, 0, B, 0) CV_F if (FETCH) CV_LOAD_W(N_, 0) CV_READ1(xb, 1, B, 1) CV_F          \
        CV_MMA1(xa, 1, B, 0) CV_F if (FETCH) CV_LOAD_W(N_, 1) CV_READ1(xb, 2, B, 1) CV_F          \
        CV_MMA1(xa, 2, B, 0) CV_F if (FETCH) CV_LOAD_W(N_, 2) CV_READ1(xb, 3, B, 1) CV_F          \
        CV_MMA1(xa, 3, B, 0) CV_F                                                                 \
        CV_MMA1(xb, 0, B, 1) CV_F if (FETCH) CV_LOAD_X1(N_, 0) CV_READ1(xa, 0, B, 2) CV_F         \
        CV_MMA1(xb, 1, B, 1) CV_F CV_READ1(xa, 1, B, 2) CV_F                                      \
        CV_MMA1(xb, 2, B, 1) CV_F if (FETCH) CV_LOAD_X1(N_, 1) CV_READ1(xa, 2, B, 2) CV_F         \
        CV_MMA1(xb, 3, B, 1) CV_F CV_READ1(xa, 3, B, 2) CV_F                                      \
        CV_MMA1(xa, 0, B, 2) CV_F if (FETCH) CV_LOAD_X1(N_, 2) CV_F                               \
        CV_MMA1(xa, 1, B, 2) CV_F                                                                 \
        CV_MMA1(xa, 2, B, 2) CV_F                                                                 \
        CV_MMA1(xa, 3, B, 2) CV_F                                                                 \
        if (FETCH) { CV_FETCH_NEXT CV_VMCNT(5) } else { CV_VMCNT(0) }                             \
        __syncthreads();                                                                          \
    }

    bf16x8 xa[4], xb[4];
    {
        CV_LOAD_W(0, 0) CV_LOAD_W(0, 1) CV_LOAD_W(0, 2)
        CV_LOAD_X1(0, 0) CV_LOAD_X1(0, 1) CV_LOAD_X1(0, 2)
        CV_FETCH_NEXT
        CV_LOAD_W(1, 0) CV_LOAD_W(1, 1) CV_LOAD_W(1, 2)
        CV_LOAD_X1(1, 0) CV_LOAD_X1(1, 1) CV_LOAD_X1(1, 2)
        CV_FETCH_NEXT
        CV_F
        CV_VMCNT(5)
        __syncthreads();
    }
    // the number of stages is a multiple of three (three kernel rows): three stages per trip make
    // the LDS slab and the weight register set of every stage compile-time choices.  The last
    // three stages are written out: only the first of them still has something to fetch.
    for (int s = 0; s + 3 < n_stages; s += 3) {
        CV_STAGE(0, true)
        CV_STAGE(1, true)
        CV_STAGE(2, true)
    }
    CV_STAGE(0, true)
    CV_STAGE(1, false)
    CV_STAGE(2, false)
#undef CV_STAGE
#undef CV_FETCH_NEXT
#undef CV_LOAD_X1
#undef CV_LOAD_W
#undef CV_DMA
#undef CV_READ1
#undef CV_MMA1
#undef CV_VMCNT
#undef CV_F

    // ---- exchange of the partial sums: accumulator tile j of every wavefront goes to the
    //      wavefront (wn, kgrp = j), which adds the four partials in ascending source order
    float* red = (float*)smem_raw;   // [owner = j * 2 + wn][source slot 0..2][4 register groups][64 lanes][4]
    // (all wavefronts are past the last barrier of the K loop: the slabs are free)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        if (j != kgrp) {
            const int src = kgrp - (kgrp > j ? 1 : 0);
            float* dst = red + ((size_t)((j * 2 + wn) * 3 + src) * 16) * 64 + lane * 4;
#pragma unroll
            for (int rq = 0; rq < 4; ++rq)
                *(f32x4*)(dst + rq * 256) = f32x4{acc[j][rq * 4], acc[j][rq * 4 + 1], acc[j][rq * 4 + 2], acc[j][rq * 4 + 3]};
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
                const float* srcp = red + ((size_t)((kgrp * 2 + wn) * 3 + (k - (k > kgrp ? 1 : 0))) * 16) * 64 + lane * 4;
#pragma unroll
                for (int rq = 0; rq < 4; ++rq) {
                    const f32x4 v = *(const f32x4*)(srcp + rq * 256);
#pragma unroll
                    for (int e = 0; e < 4; ++e) term[rq * 4 + e] = v[e];
                }
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
            // (a lane holds classes 8 gq + 4 lhi .. + 3; the groups beyond the classes are padding)
            float* zrow = a.zpart + ((size_t)nt * a.PP + mp) * a.zpitch + lhi * 4;
#pragma unroll
            for (int gq = 0; gq < 4; ++gq)
                if (gq * 8 + lhi * 4 < a.zpitch)
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
    a.W3q = W3q; a.zpart = zpart; a.n_cls = p.g.C; a.zpitch = (p.g.C + 3) / 4 * 4; a.dense = dense;
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

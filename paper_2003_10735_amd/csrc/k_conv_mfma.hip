// 3x3 convolution (forward, and data-gradient as a forward with mirrored taps) as an implicit
// GEMM on the gfx950 matrix cores: bfloat16 operands, float32 accumulation
// (v_mfma_f32_32x32x16_bf16).
//
//   out[mp][n] = epi( sum_{kh,kw,c} X[mp + (kh-1)*Wp + (kw-1)][c] * Wq[n][kh*3+kw][c] )
//
// X is position-major on the zero-padded grid, so a tap is a constant row offset and the GEMM's
// M index can simply walk the padded positions mp = 0 .. PP-1 linearly (results at border
// positions are forced to zero, which keeps the border of the output zero as well).  Guard rows
// in front of and behind every activation buffer make all reads in-bounds without tests.
//
// Block = 512 threads = 8 wavefronts, tile = 128 positions x BN output channels.  Wavefronts
// 0-3 and 4-7 cover the same 2 x 2 arrangement of sub-tiles and split the K steps of every
// stage between them (two wavefronts per SIMD: while one waits for its LDS fragments the other
// one's MFMAs run); their accumulators are added through LDS once, before the epilogue.
// K loop: stages of (one kernel row kh) x (64 input channels).  A stage holds in LDS
//   Xs: 130 activation rows (the tile's rows shifted by kh, plus one on each side) -- the three
//       taps kw = 0,1,2 of that kernel row read the same slab at row offsets 0,1,2;
//   Ws: 3 x BN weight rows.
// Stages are pipelined three deep (global -> registers, registers -> LDS, LDS -> matrix cores),
// so the global loads of stage s+2 are in flight while the matrix cores work on stage s.  LDS rows are padded by 16 bytes so that the 16-byte fragment reads of
// 32 consecutive rows spread over all banks.
//
// The weights are the MFMA A operand (rows = output channels) and the activations the B operand
// (columns = positions): a lane then owns 4 consecutive output channels of one position per
// register group, which packs into one 8-byte LDS write in the epilogue.  The epilogue stages the
// tile in LDS and writes it twice with 16-byte stores: position-major (input of the next
// convolution) and channel-major (operand of the weight-gradient kernel).
#include "st_kernels.hpp"
#include "st_mfma.hpp"

namespace st {

constexpr int CV_BM = 128;
constexpr int CV_BK = 64;
constexpr int CV_LDP = CV_BK + 8;   // LDS row pitch in elements (144 bytes)

struct ConvArgs {
    const bf16* X;      // [PP][cin] position-major, guards before/after
    const bf16* Wq;     // [cout][9][cin]
    const float* bias;  // EPI 0
    const bf16* mask;   // EPI 1: activation whose sign gates the gradient, [PP][cout]
    bf16* Y;            // [PP][cout] or nullptr
    bf16* YT;           // channel-major copy, blocked layout of xt_index(), or nullptr
    int PP, Hp, Wp, h, w, cin, cout, PPT, guard;
    int m_tiles, n_tiles, tiles_per_xcd;
};

// TAG only gives every call site (layer 1 forward, layer 2 forward, layer 2 data-gradient) a
// kernel symbol of its own, so that profiles list them separately.
template <int BN, int EPI, int TAG>
__global__ void __launch_bounds__(512) k_conv3x3_mfma(ConvArgs a)
{
    constexpr int TA = BN / 64;          // 32-row weight fragments per wavefront
    constexpr int NT = 512;                // threads per block
    constexpr int XS_ROWS = CV_BM + 2;
    // 16-byte chunks per stage; every thread moves the same number without a bounds test: the
    // activation slots beyond the last chunk wrap around and re-copy a chunk (same bytes)
    constexpr int XS_CHUNKS = XS_ROWS * 8, WS_CHUNKS = 3 * BN * 8;
    constexpr int XS_PER_T = (XS_CHUNKS + NT - 1) / NT, WS_PER_T = WS_CHUNKS / NT;
    constexpr int XS_ELEMS = XS_ROWS * CV_LDP, WS_ELEMS = 3 * BN * CV_LDP;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    bf16* Xs = (bf16*)smem_raw;                       // [2][XS_ROWS][LDP]
    bf16* Ws = Xs + 2 * XS_ELEMS;                     // [2][3][BN][LDP]

    // XCD-aware tile order: consecutive blocks go to different XCDs, so give each XCD a
    // contiguous run of position tiles (neighbours share activation rows in that XCD's L2)
    const int xcd = blockIdx.x % 8, slot = blockIdx.x / 8;
    const int tile = xcd * a.tiles_per_xcd + slot;
    if (slot >= a.tiles_per_xcd || tile >= a.m_tiles * a.n_tiles) return;
    const int mt = tile / a.n_tiles, nt = tile % a.n_tiles;
    const int m0 = mt * CV_BM, n0 = nt * BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wn = wave & 1, wm = (wave >> 1) & 1, kgrp = wave >> 2;
    const int l32 = lane & 31, lhi = lane >> 5;

    f32x16 acc[TA][2];
#pragma unroll
    for (int i = 0; i < TA; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int c_chunks = a.cin / CV_BK;
    const int n_stages = 3 * c_chunks;
    // Three-deep pipeline: while the matrix cores work on stage s out of one LDS buffer, the
    // registers holding stage s+1 (loaded during stage s-1) are written to the other buffer and
    // the global loads of stage s+2 are issued into the second register set.  A load therefore
    // has a whole stage of matrix work to complete before anything waits for it.
    u32x4 xr[2][XS_PER_T], wr[2][WS_PER_T];

#define CV_LOAD(SET, S)                                                                           \
    {                                                                                             \
        const int kh_ = (S) / c_chunks, c0_ = ((S) % c_chunks) * CV_BK;                           \
        const long long row0_ = (long long)m0 - 1 + (long long)(kh_ - 1) * a.Wp;                  \
        _Pragma("unroll") for (int i = 0; i < XS_PER_T; ++i) {                                    \
            int q = tid + i * NT;                                                                 \
            q = q < XS_CHUNKS ? q : q - XS_CHUNKS;                                                \
            xr[SET][i] = *(const u32x4*)(a.X + (row0_ + (q >> 3)) * a.cin + c0_ + (q & 7) * 8);   \
        }                                                                                         \
        _Pragma("unroll") for (int i = 0; i < WS_PER_T; ++i) {                                    \
            const int q = tid + i * NT;                                                           \
            const int row = q >> 3;                                                               \
            const int n = min(n0 + row % BN, a.cout - 1);                                         \
            wr[SET][i] = *(const u32x4*)(a.Wq + ((size_t)n * 9 + kh_ * 3 + row / BN) * a.cin +    \
                                         c0_ + (q & 7) * 8);                                      \
        }                                                                                         \
    }
#define CV_STORE(SET, BUF)                                                                        \
    {                                                                                             \
        bf16* xs_ = Xs + (BUF) * XS_ELEMS;                                                        \
        bf16* ws_ = Ws + (BUF) * WS_ELEMS;                                                        \
        _Pragma("unroll") for (int i = 0; i < XS_PER_T; ++i) {                                    \
            int q = tid + i * NT;                                                                 \
            q = q < XS_CHUNKS ? q : q - XS_CHUNKS;                                                \
            *(u32x4*)(xs_ + (q >> 3) * CV_LDP + (q & 7) * 8) = xr[SET][i];                        \
        }                                                                                         \
        _Pragma("unroll") for (int i = 0; i < WS_PER_T; ++i) {                                    \
            const int q = tid + i * NT;                                                           \
            *(u32x4*)(ws_ + (q >> 3) * CV_LDP + (q & 7) * 8) = wr[SET][i];                        \
        }                                                                                         \
    }
#define CV_COMPUTE(BUF, KW)                                                                       \
    {                                                                                             \
        const bf16* xs = Xs + (BUF) * XS_ELEMS;                                                   \
        const bf16* ws = Ws + (BUF) * WS_ELEMS;                                                   \
        _Pragma("unroll") for (int k2 = 0; k2 < CV_BK / 32; ++k2) {                               \
            const int col = (k2 * 2 + kgrp) * 16 + lhi * 8;                                       \
            bf16x8 xf[2], wf[TA];                                                                 \
            _Pragma("unroll") for (int j = 0; j < 2; ++j)                                         \
                xf[j] = *(const bf16x8*)(xs + (wm * 64 + j * 32 + l32 + (KW)) * CV_LDP + col);    \
            _Pragma("unroll") for (int i = 0; i < TA; ++i)                                        \
                wf[i] = *(const bf16x8*)(ws + ((KW) * BN + wn * (BN / 2) + i * 32 + l32) * CV_LDP + col); \
            _Pragma("unroll") for (int i = 0; i < TA; ++i)                                        \
                _Pragma("unroll") for (int j = 0; j < 2; ++j)                                     \
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[i], xf[j], acc[i][j], 0, 0, 0); \
        }                                                                                         \
    }

    // (loads and LDS stores are unconditional, with the stage index clamped to the last stage:
    //  a load under a branch would force a wait for every outstanding load at the join; the
    //  redundant copies at the tail land in the buffer nobody reads any more)
    const int last = n_stages - 1;
    CV_LOAD(0, 0)
    CV_LOAD(1, min(1, last))
    CV_STORE(0, 0)
    __syncthreads();
    for (int s = 0; s < n_stages; s += 2) {
        // even stage s: LDS buffer 0; register set 1 holds stage s+1; set 0 is free
        CV_LOAD(0, min(s + 2, last))
        __builtin_amdgcn_sched_barrier(0);   // keep the loads first: the scheduler would sink them
        CV_COMPUTE(0, 0)
        __builtin_amdgcn_sched_barrier(0);
        CV_STORE(1, 1)
        __builtin_amdgcn_sched_barrier(0);
        CV_COMPUTE(0, 1)
        CV_COMPUTE(0, 2)
        __syncthreads();
        if (s + 1 >= n_stages) break;
        // odd stage s+1: LDS buffer 1; register set 0 holds stage s+2; set 1 is free
        CV_LOAD(1, min(s + 3, last))
        __builtin_amdgcn_sched_barrier(0);
        CV_COMPUTE(1, 0)
        __builtin_amdgcn_sched_barrier(0);
        CV_STORE(0, 0)
        __builtin_amdgcn_sched_barrier(0);
        CV_COMPUTE(1, 1)
        CV_COMPUTE(1, 2)
        __syncthreads();
    }
#undef CV_LOAD
#undef CV_STORE
#undef CV_COMPUTE

    // ---- epilogue: bias + ReLU (forward) or ReLU mask (data-gradient), zero outside the grid,
    //      round to bfloat16, stage the tile in LDS as [position][channel]
    // the second K group hands its accumulators to the first through LDS
    {
        float* red = (float*)smem_raw;   // [4 wavefronts][TA * 2 * 16][64]
        if (kgrp == 1) {
#pragma unroll
            for (int i = 0; i < TA; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        red[(((wave & 3) * TA * 2 + i * 2 + j) * 16 + r) * 64 + lane] = acc[i][j][r];
        }
        __syncthreads();
        if (kgrp == 0) {
#pragma unroll
            for (int i = 0; i < TA; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int r = 0; r < 16; ++r)
                        acc[i][j][r] += red[(((wave & 3) * TA * 2 + i * 2 + j) * 16 + r) * 64 + lane];
        }
        __syncthreads();
    }
    constexpr int OLD = BN + 8;
    bf16* Os = (bf16*)smem_raw;     // [CV_BM][OLD]; all waves are past the last barrier
    if (kgrp == 0) {
    const int frame = a.Hp * a.Wp;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int p = wm * 64 + j * 32 + l32;
        const int mp = m0 + p;
        const int rr = mp % frame, y = rr / a.Wp, x = rr - y * a.Wp;
        const bool inside = mp < a.PP && y >= 1 && y <= a.h && x >= 1 && x <= a.w;
#pragma unroll
        for (int i = 0; i < TA; ++i) {
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                const int c = wn * (BN / 2) + i * 32 + rg * 8 + lhi * 4;   // channel inside the tile
                const int cg = min(n0 + c, a.cout - 4);
                float v[4];
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = acc[i][j][rg * 4 + e];
                if (EPI == 0) {
                    const float4 b = *(const float4*)(a.bias + cg);
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
                *(bf16x4*)(Os + p * OLD + c) = o;
            }
        }
    }
    }
    __syncthreads();
    const int n_valid = min(BN, a.cout - n0);
    if (a.Y) {
        // position-major: 16 bytes = 8 channels of one position
        for (int q = tid; q < CV_BM * (BN / 8); q += NT) {
            const int p = q / (BN / 8), part = q % (BN / 8);
            if (m0 + p < a.PP && part * 8 < n_valid)
                *(uint4*)(a.Y + (size_t)(m0 + p) * a.cout + n0 + part * 8) = *(const uint4*)(Os + p * OLD + part * 8);
        }
    }
    if (a.YT) {
        // channel-major: 16 bytes = 8 consecutive positions of one channel
        for (int q = tid; q < (CV_BM / 8) * BN; q += NT) {
            const int c = q % BN, pg = q / BN;
            if (c < n_valid) {
                bf16x8 o;
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] = Os[(pg * 8 + e) * OLD + c];
                *(bf16x8*)(a.YT + xt_index(n0 + c, a.guard + m0 + pg * 8, a.PPT / 8)) = o;
            }
        }
    }
}

template <int BN>
static size_t conv_smem_bytes()
{
    return (size_t)2 * ((CV_BM + 2) * CV_LDP + 3 * BN * CV_LDP) * sizeof(bf16);
}

bool conv3x3_mfma_supported(int cin, int cout) { return cin % CV_BK == 0 && cout % 32 == 0 && cout >= 32; }

// epi 0: Y = relu(conv + bias); epi 1: Y = conv * [mask > 0]
void conv3x3_mfma(Ctx& c, const char* name, const Plan& p, const bf16* X, const bf16* Wq, const float* bias,
                  const bf16* mask, bf16* Y, bf16* YT, int cin, int cout, int epi, int layer)
{
    ConvArgs a;
    a.X = X; a.Wq = Wq; a.bias = bias; a.mask = mask; a.Y = Y; a.YT = YT;
    a.PP = p.g.padded_positions(); a.Hp = p.g.Hp; a.Wp = p.g.Wp; a.h = p.g.h; a.w = p.g.w;
    a.cin = cin; a.cout = cout;
    a.PPT = p.PPT; a.guard = p.guard;
    constexpr int BN = 64;
    a.m_tiles = cdiv(a.PP, CV_BM);
    a.n_tiles = cdiv(cout, BN);
    const int tiles = a.m_tiles * a.n_tiles;
    a.tiles_per_xcd = cdiv(tiles, 8);
    const dim3 grid(a.tiles_per_xcd * 8);
    const size_t smem = conv_smem_bytes<BN>();
    // tag 1: layer-1 forward, 2: layer-2 forward, 3: layer-2 data-gradient
    auto go = [&](auto kernel) {
        ensure_dynamic_lds((const void*)kernel, smem);
        ST_LAUNCH(c, name, kernel, grid, dim3(512), smem, a);
    };
    if (epi == 1) go(k_conv3x3_mfma<BN, 1, 3>);
    else if (layer == 1) go(k_conv3x3_mfma<BN, 0, 1>);
    else go(k_conv3x3_mfma<BN, 0, 2>);
}

}  // namespace st

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
// Block = 256 threads = 4 wavefronts, tile = 128 positions x BN output channels.
// K loop: stages of (one kernel row kh) x (64 input channels).  A stage holds in LDS
//   Xs: 130 activation rows (the tile's rows shifted by kh, plus one on each side) -- the three
//       taps kw = 0,1,2 of that kernel row read the same slab at row offsets 0,1,2;
//   Ws: 3 x BN weight rows.
// Stages are double-buffered: the global loads of stage s+1 are in flight while the matrix
// cores work on stage s.  LDS rows are padded by 16 bytes so that the 16-byte fragment reads of
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
    bf16* YT;           // [cout][PPT], position mp at column guard + mp, or nullptr
    int PP, Hp, Wp, cin, cout, PPT, guard;
    int m_tiles, n_tiles, tiles_per_xcd;
};

template <int BN, int EPI>
__global__ void __launch_bounds__(256) k_conv3x3_mfma(ConvArgs a)
{
    constexpr int TA = BN / 64;          // 32-row weight fragments per wavefront
    // 130 activation rows are needed; 160 are staged so that every thread moves the same
    // number of 16-byte chunks (5) without a bounds test -- the extra rows are never read back
    constexpr int XS_ROWS = 160;
    constexpr int XS_CHUNKS = XS_ROWS * 8, WS_CHUNKS = 3 * BN * 8;
    constexpr int XS_PER_T = XS_CHUNKS / 256, WS_PER_T = WS_CHUNKS / 256;
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
    const int wn = wave & 1, wm = wave >> 1;
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
    // prefetch registers of one stage (kept as plain unrolled register arrays)
    u32x4 xr[XS_PER_T], wr[WS_PER_T];

#define CV_LOAD_STAGE(S)                                                                          \
    {                                                                                             \
        const int kh_ = (S) / c_chunks, c0_ = ((S) % c_chunks) * CV_BK;                           \
        const long long row0_ = (long long)m0 - 1 + (long long)(kh_ - 1) * a.Wp;                  \
        _Pragma("unroll") for (int i = 0; i < XS_PER_T; ++i) {                                    \
            const int q = tid + i * 256;                                                          \
            xr[i] = *(const u32x4*)(a.X + (row0_ + (q >> 3)) * a.cin + c0_ + (q & 7) * 8);        \
        }                                                                                         \
        _Pragma("unroll") for (int i = 0; i < WS_PER_T; ++i) {                                    \
            const int q = tid + i * 256;                                                          \
            const int row = q >> 3;                                                               \
            const int n = min(n0 + row % BN, a.cout - 1);                                         \
            wr[i] = *(const u32x4*)(a.Wq + ((size_t)n * 9 + kh_ * 3 + row / BN) * a.cin + c0_ +   \
                                    (q & 7) * 8);                                                 \
        }                                                                                         \
    }
#define CV_STORE_STAGE(BUF)                                                                       \
    {                                                                                             \
        bf16* xs_ = Xs + (BUF) * XS_ELEMS;                                                        \
        bf16* ws_ = Ws + (BUF) * WS_ELEMS;                                                        \
        _Pragma("unroll") for (int i = 0; i < XS_PER_T; ++i) {                                    \
            const int q = tid + i * 256;                                                          \
            *(u32x4*)(xs_ + (q >> 3) * CV_LDP + (q & 7) * 8) = xr[i];                             \
        }                                                                                         \
        _Pragma("unroll") for (int i = 0; i < WS_PER_T; ++i) {                                    \
            const int q = tid + i * 256;                                                          \
            *(u32x4*)(ws_ + (q >> 3) * CV_LDP + (q & 7) * 8) = wr[i];                             \
        }                                                                                         \
    }

    CV_LOAD_STAGE(0)
    CV_STORE_STAGE(0)
    __syncthreads();
    for (int s = 0; s < n_stages; ++s) {
        const int buf = s & 1;
        if (s + 1 < n_stages) CV_LOAD_STAGE(s + 1)
        const bf16* xs = Xs + buf * XS_ELEMS;
        const bf16* ws = Ws + buf * WS_ELEMS;
#pragma unroll
        for (int kw = 0; kw < 3; ++kw) {
#pragma unroll
            for (int ks = 0; ks < CV_BK / 16; ++ks) {
                const int col = ks * 16 + lhi * 8;
                bf16x8 xf[2], wf[TA];
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    xf[j] = *(const bf16x8*)(xs + (wm * 64 + j * 32 + l32 + kw) * CV_LDP + col);
#pragma unroll
                for (int i = 0; i < TA; ++i)
                    wf[i] = *(const bf16x8*)(ws + (kw * BN + wn * (BN / 2) + i * 32 + l32) * CV_LDP + col);
#pragma unroll
                for (int i = 0; i < TA; ++i)
#pragma unroll
                    for (int j = 0; j < 2; ++j)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[i], xf[j], acc[i][j], 0, 0, 0);
            }
        }
        if (s + 1 < n_stages) CV_STORE_STAGE(buf ^ 1)
        __syncthreads();
    }
#undef CV_LOAD_STAGE
#undef CV_STORE_STAGE

    // ---- epilogue: bias + ReLU (forward) or ReLU mask (data-gradient), zero outside the grid,
    //      round to bfloat16, stage the tile in LDS as [position][channel]
    constexpr int OLD = BN + 8;
    bf16* Os = (bf16*)smem_raw;     // [CV_BM][OLD]; all waves are past the last barrier
    const int frame = a.Hp * a.Wp;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int p = wm * 64 + j * 32 + l32;
        const int mp = m0 + p;
        const int rr = mp % frame, y = rr / a.Wp, x = rr - y * a.Wp;
        const bool inside = mp < a.PP && y >= 1 && y <= a.Hp - 2 && x >= 1 && x <= a.Wp - 2;
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
    __syncthreads();
    const int n_valid = min(BN, a.cout - n0);
    if (a.Y) {
        // position-major: 16 bytes = 8 channels of one position
        for (int q = tid; q < CV_BM * (BN / 8); q += 256) {
            const int p = q / (BN / 8), part = q % (BN / 8);
            if (m0 + p < a.PP && part * 8 < n_valid)
                *(uint4*)(a.Y + (size_t)(m0 + p) * a.cout + n0 + part * 8) = *(const uint4*)(Os + p * OLD + part * 8);
        }
    }
    if (a.YT) {
        // channel-major: 16 bytes = 8 consecutive positions of one channel
        for (int q = tid; q < (CV_BM / 8) * BN; q += 256) {
            const int c = q % BN, pg = q / BN;
            if (c < n_valid) {
                bf16x8 o;
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] = Os[(pg * 8 + e) * OLD + c];
                *(bf16x8*)(a.YT + (size_t)(n0 + c) * a.PPT + a.guard + m0 + pg * 8) = o;
            }
        }
    }
}

template <int BN>
static size_t conv_smem_bytes()
{
    return (size_t)2 * (160 * CV_LDP + 3 * BN * CV_LDP) * sizeof(bf16);
}

bool conv3x3_mfma_supported(int cin, int cout) { return cin % CV_BK == 0 && cout % 32 == 0 && cout >= 32; }

// epi 0: Y = relu(conv + bias); epi 1: Y = conv * [mask > 0]
void conv3x3_mfma(Ctx& c, const char* name, const Plan& p, const bf16* X, const bf16* Wq, const float* bias,
                  const bf16* mask, bf16* Y, bf16* YT, int cin, int cout, int epi)
{
    ConvArgs a;
    a.X = X; a.Wq = Wq; a.bias = bias; a.mask = mask; a.Y = Y; a.YT = YT;
    a.PP = p.g.padded_positions(); a.Hp = p.g.Hp; a.Wp = p.g.Wp; a.cin = cin; a.cout = cout;
    a.PPT = p.PPT; a.guard = p.guard;
    constexpr int BN = 64;
    a.m_tiles = cdiv(a.PP, CV_BM);
    a.n_tiles = cdiv(cout, BN);
    const int tiles = a.m_tiles * a.n_tiles;
    a.tiles_per_xcd = cdiv(tiles, 8);
    const dim3 grid(a.tiles_per_xcd * 8);
    const size_t smem = conv_smem_bytes<BN>();
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute((const void*)k_conv3x3_mfma<BN, 0>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        (void)hipFuncSetAttribute((const void*)k_conv3x3_mfma<BN, 1>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        attr_set = true;
    }
    if (epi == 0) ST_LAUNCH(c, name, (k_conv3x3_mfma<BN, 0>), grid, dim3(256), smem, a);
    else ST_LAUNCH(c, name, (k_conv3x3_mfma<BN, 1>), grid, dim3(256), smem, a);
}

}  // namespace st

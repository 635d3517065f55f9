// Weight gradient of a 3x3 convolution on the matrix cores:
//
//   dW[o][tap][i] = sum_mp dY[o][mp] * X[i][mp + (kh-1)*Wp + (kw-1)]          (tap = kh*3 + kw)
//   db[o]         = sum_mp dY[o][mp]
//
// Both operands are read from their channel-major copies (positions contiguous), so that a
// lane's 8 reduction elements are 16 contiguous bytes and need no transposition.  dY is zero on
// the border of the padded grid, so the sum may run over all padded positions.
//
// One wavefront accumulates a 32 (o) x 32 (i) x 9 (taps) block (144 accumulator registers): per
// 16 positions it loads one dY fragment and, per kernel row kh, one 16-byte window of X (the
// row pitch of the padded grid is a multiple of 8, so all of them are aligned fragments of the
// blocked channel-major layout and every wavefront load is one contiguous kilobyte); the kw = 0
// and kw = 2 operands are the same window shifted by one element, built in registers
// (v_alignbyte + a cross-lane permute for the element that enters) instead of being loaded
// again.  9 MFMAs per 4 loads.  A bigger block would need fewer loads per MFMA but leaves too few blocks to fill the
// chip without multiplying the partial copies.
//
// The four wavefronts of a block own the same output block and a quarter each of the block's
// position range; they are added in LDS in a fixed order, and the grid's position splits are
// added by the optimiser kernel, also in a fixed order: no floating-point atomics.
#include "st_kernels.hpp"
#include "st_mfma.hpp"

namespace st {

struct WgradArgs {
    const bf16* dYT;   // channel-major copies in the blocked layout of xt_index()
    const bf16* XT;
    float* dW;         // [splits][stride] : this layer's weight block, [o][9][cin]
    float* db;         // [splits][stride] : this layer's bias block
    size_t split_stride;
    int cin, cout, PPT, guard, Wp;
    int units_per_wave;   // 16-position units per wavefront
    int n_units;          // total units
    int o_tiles, i_tiles;
};

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

__global__ void __launch_bounds__(256) k_wgrad3x3_mfma(WgradArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    float* red = (float*)smem_raw;    // [9][16][64] accumulators of one wavefront, then [64] bias sums

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, lhi = lane >> 5;
    const int tile = blockIdx.x % (a.o_tiles * a.i_tiles), split = blockIdx.x / (a.o_tiles * a.i_tiles);
    const int ot = tile / a.i_tiles, it = tile % a.i_tiles;
    const int o0 = ot * 32, i0 = it * 32;

    f32x16 acc[9];
#pragma unroll
    for (int t = 0; t < 9; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;
    float bsum = 0.f;

    const int unit0 = (split * 4 + wave) * a.units_per_wave;
    const int unit1 = min(unit0 + a.units_per_wave, a.n_units);
    // blocked layout: one 8-position group of 32 channels is 256 elements; lane (l32, lhi) reads
    // channel l32 of group 2u + lhi, so a wavefront's fragment load is one contiguous kilobyte
    const int NG = a.PPT >> 3;
    const bf16* ya = a.dYT + (((size_t)(o0 >> 5) * NG + (a.guard >> 3) + lhi) << 8) + l32 * 8;
    const bf16* xb = a.XT + (((size_t)(i0 >> 5) * NG + (a.guard >> 3) + lhi) << 8) + l32 * 8;
    const int row_groups = a.Wp >> 3;   // one kernel row = this many 8-position groups
    const bool want_bias = it == 0;
    const int swap_addr = (lane ^ 32) << 2;   // ds_bpermute address of the lane holding the other half

    // Operand ring: the loads of unit u + 3 are issued before the MFMAs of unit u, so that an L2
    // round trip is covered by matrix work of the same wavefront (there is only one wavefront
    // per SIMD: the accumulators take most of the register file).
    constexpr int DEPTH = 4;
    u32x4 ry[DEPTH], rx[DEPTH][3];
#define WG_LOAD(SLOT, U)                                                                        \
    {                                                                                           \
        const ptrdiff_t g_ = (ptrdiff_t)(U) * 2 * 256;                                          \
        ry[SLOT] = *(const u32x4*)(ya + g_);                                                    \
        _Pragma("unroll") for (int kh = 0; kh < 3; ++kh)                                        \
            rx[SLOT][kh] = *(const u32x4*)(xb + g_ + (ptrdiff_t)(kh - 1) * row_groups * 256);   \
    }
    // The kw = 0 / kw = 2 operands are the kw = 1 window moved by one position.  The element that
    // enters on the left is the last one of the previous 8-position group, the one on the right
    // the first of the next group: both sit in the *other half* of the wavefront (lane ^ 32), in
    // this unit's registers or in the neighbouring unit's, so they are fetched with a cross-lane
    // permute instead of being loaded again.
    unsigned int last_prev[3];   // for lhi = 0: dword 3 of the previous unit's upper half
    unsigned int first_cur[3];   // for lhi = 0: dword 0 of this unit's upper half (computed one unit ahead)
#define WG_COMPUTE(SLOT, NEXT)                                                                  \
    {                                                                                           \
        const bf16x8 y0 = as_bf16x8(ry[SLOT]);                                                  \
        if (want_bias) {                                                                        \
            _Pragma("unroll") for (int e = 0; e < 8; ++e) bsum += (float)y0[e];                 \
        }                                                                                       \
        _Pragma("unroll") for (int kh = 0; kh < 3; ++kh) {                                      \
            const u32x4 w_ = rx[SLOT][kh];                                                      \
            const unsigned int s3_ = __builtin_amdgcn_ds_bpermute(swap_addr, w_[3]);            \
            const unsigned int n0_ = __builtin_amdgcn_ds_bpermute(swap_addr, rx[NEXT][kh][0]);  \
            const unsigned int prev_ = lhi ? s3_ : last_prev[kh];                               \
            const unsigned int next_ = lhi ? n0_ : first_cur[kh];                               \
            last_prev[kh] = s3_;      /* lhi = 0 lanes: upper half of this unit, used next */   \
            first_cur[kh] = n0_;      /* lhi = 0 lanes: upper half of the next unit */          \
            u32x4 lft, rgt;                                                                     \
            lft[0] = __builtin_amdgcn_alignbyte(w_[0], prev_, 2);                               \
            lft[1] = __builtin_amdgcn_alignbyte(w_[1], w_[0], 2);                               \
            lft[2] = __builtin_amdgcn_alignbyte(w_[2], w_[1], 2);                               \
            lft[3] = __builtin_amdgcn_alignbyte(w_[3], w_[2], 2);                               \
            rgt[0] = lft[1]; rgt[1] = lft[2]; rgt[2] = lft[3];                                  \
            rgt[3] = __builtin_amdgcn_alignbyte(next_, w_[3], 2);                               \
            acc[kh * 3 + 0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(y0, as_bf16x8(lft), acc[kh * 3 + 0], 0, 0, 0); \
            acc[kh * 3 + 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(y0, as_bf16x8(w_), acc[kh * 3 + 1], 0, 0, 0);  \
            acc[kh * 3 + 2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(y0, as_bf16x8(rgt), acc[kh * 3 + 2], 0, 0, 0); \
        }                                                                                       \
    }

    if (unit0 < unit1) {
        // unit0 - 1 (guard columns make it readable) supplies the first left neighbours
        WG_LOAD(DEPTH - 1, unit0 - 1)
        WG_LOAD(0, unit0)
#pragma unroll
        for (int kh = 0; kh < 3; ++kh) {
            last_prev[kh] = __builtin_amdgcn_ds_bpermute(swap_addr, rx[DEPTH - 1][kh][3]);
            first_cur[kh] = __builtin_amdgcn_ds_bpermute(swap_addr, rx[0][kh][0]);
        }
#pragma unroll
        for (int d = 1; d < DEPTH - 1; ++d)
            if (unit0 + d <= unit1) WG_LOAD(d, unit0 + d)
        // unit1 itself is loaded too (readable: tail guard): it supplies the last right neighbours
        for (int u = unit0; u < unit1; u += DEPTH) {
#pragma unroll
            for (int d = 0; d < DEPTH; ++d) {
                if (u + d + DEPTH - 1 <= unit1) WG_LOAD((d + DEPTH - 1) % DEPTH, u + d + DEPTH - 1)
                if (u + d < unit1) WG_COMPUTE(d, (d + 1) % DEPTH)
            }
        }
    }
#undef WG_LOAD
#undef WG_COMPUTE

    // ---- add the four wavefronts in the order 3, 2, 1, 0 through LDS
    for (int w = 3; w >= 1; --w) {
        if (wave == w) {
#pragma unroll
            for (int t = 0; t < 9; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) red[(t * 16 + r) * 64 + lane] = acc[t][r];
            if (want_bias) red[9 * 16 * 64 + lane] = bsum;
        }
        __syncthreads();
        if (wave == w - 1) {
#pragma unroll
            for (int t = 0; t < 9; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[t][r] += red[(t * 16 + r) * 64 + lane];
            if (want_bias) bsum += red[9 * 16 * 64 + lane];
        }
        __syncthreads();
    }
    if (wave != 0) return;

    float* dW = a.dW + (size_t)split * a.split_stride;
#pragma unroll
    for (int t = 0; t < 9; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int o = o0 + (r >> 2) * 8 + lhi * 4 + (r & 3);
            dW[((size_t)o * 9 + t) * a.cin + i0 + l32] = acc[t][r];
        }
    if (want_bias) {
        // a lane pair (l, l + 32) holds the two halves of one output channel's sum
        float* db = a.db + (size_t)split * a.split_stride;
        const float other = __shfl(bsum, lane ^ 32, 64);
        if (lhi == 0) db[o0 + l32] = bsum + other;
    }
}

bool wgrad3x3_mfma_supported(int cin, int cout) { return cin % 32 == 0 && cout % 32 == 0; }

int wgrad_splits_for(const Geo& g, int cin, int cout)
{
    const int tiles = (cout / 32) * (cin / 32);
    int s = cdiv(256, tiles);
    const int n_units = cdiv(g.padded_positions(), 16);
    // keep at least 8 units (128 positions) per wavefront
    while (s > 1 && cdiv(n_units, s * 4) < 8) --s;
    return s < 1 ? 1 : (s > 16 ? 16 : s);
}

void wgrad3x3_mfma(Ctx& c, const char* name, const Plan& p, const bf16* dYT, const bf16* XT, float* dW,
                   float* db, int cin, int cout, int splits)
{
    WgradArgs a;
    a.dYT = dYT; a.XT = XT; a.dW = dW; a.db = db;
    a.split_stride = p.po.total;
    a.cin = cin; a.cout = cout; a.PPT = p.PPT; a.guard = p.guard; a.Wp = p.g.Wp;
    a.n_units = cdiv(p.g.padded_positions(), 16);
    a.units_per_wave = cdiv(a.n_units, splits * 4);
    a.o_tiles = cout / 32; a.i_tiles = cin / 32;
    const size_t smem = (size_t)(9 * 16 * 64 + 64) * sizeof(float);
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute((const void*)k_wgrad3x3_mfma, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        attr_set = true;
    }
    ST_LAUNCH(c, name, k_wgrad3x3_mfma, dim3(a.o_tiles * a.i_tiles * splits), dim3(256), smem, a);
}

}  // namespace st

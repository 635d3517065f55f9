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
// and kw = 2 products use the dY fragment shifted by one position, built in registers
// (v_alignbyte + a cross-lane permute for the element that enters) instead of loading shifted
// windows.  9 MFMAs per 4 loads.  A bigger block would need fewer loads per MFMA but leaves too few blocks to fill the
// chip without multiplying the partial copies.
//
// The four wavefronts of a block own the same output block and a quarter each of the block's
// position range; they are added through LDS in a fixed order, and the grid's position splits
// are added by the optimiser kernel, also in a fixed order: no floating-point atomics.  The
// bias gradient (sums of dY over the positions) comes from one extra MFMA against a fragment of
// ones in the blocks of the first input-channel tile.
#include <algorithm>
#include <vector>

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
    int n_units;          // units of one head's positions
    int o_tiles, i_tiles, splits, items_per_xcd;
    // Several heads: head k owns the positions from 8-position group k * head_groups8 on and
    // writes its partial copies head_out_stride floats after head k - 1.  (A head's last unit may
    // reach into the next frame's first row: dY is zero there, like on every border.)
    int heads, head_groups8;
    size_t head_out_stride;
};

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

// One launch serves both 3x3 layers: blocks [0, blocks1) work on the first argument set, the rest
// on the second.  Every block pays the same fixed cost (pipeline fill, the reduction through LDS,
// the partial-result store) whatever its share of positions, so one grid that covers the chip
// once, with the position splits of the two layers balanced against each other, is much cheaper
// than two grids that each cover it once.
__global__ void __launch_bounds__(256) k_wgrad3x3_mfma(WgradArgs a1, WgradArgs a2, int blocks1)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    const bool second = (int)blockIdx.x >= blocks1;
    const WgradArgs& a = second ? a2 : a1;
    const int bid = second ? blockIdx.x - blocks1 : blockIdx.x;

    // (the wavefront number through readfirstlane: the compiler then keeps everything derived
    //  from it -- the unit range, the loop counter, the load offsets -- in scalar registers)
    const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, lhi = lane >> 5;
    // XCD-aware order: consecutive blocks go to different XCDs; give each XCD a contiguous run
    // of work items in split-major order, so that one XCD's L2 only ever sees about 1/8 of the
    // positions (all channels) instead of every position of a few channels
    const int tiles = a.o_tiles * a.i_tiles;
    const int item = (bid % 8) * a.items_per_xcd + bid / 8;     // blocks1 is a multiple of 8
    if (bid / 8 >= a.items_per_xcd || item >= tiles * a.splits * a.heads) return;
    const int hsplit = item / tiles, tile = item % tiles;
    const int head = hsplit / a.splits, split = hsplit - head * a.splits;
    // output-channel tile fastest: the blocks that stream the same X rows (same split, same
    // input-channel tile) are neighbours in the order, run on one XCD and share them in its L2
    const int ot = tile % a.o_tiles, it = tile / a.o_tiles;
    const int o0 = ot * 32, i0 = it * 32;

    // acc[0..8]: the nine taps; acc[9]: row sums of dY (bias gradient), only in blocks with it == 0
    f32x16 acc[10];
#pragma unroll
    for (int t = 0; t < 10; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;

    const int unit0 = (split * 4 + wave) * a.units_per_wave;
    const int unit1 = min(unit0 + a.units_per_wave, a.n_units);
    // blocked layout: one 8-position group of 32 channels is 256 elements; lane (l32, lhi) reads
    // channel l32 of group 2u + lhi, so a wavefront's fragment load is one contiguous kilobyte.
    // The operands are read through buffer descriptors: the base (the unit before this
    // wavefront's first; for X one kernel row further up) sits in scalar registers, the lane
    // offset is fixed, and every load takes one scalar offset -- no address arithmetic at all
    // in the vector unit, which the K loop has no issue slots to spare for.
    const int NG = a.PPT >> 3;
    const int g0 = (a.guard >> 3) + head * a.head_groups8;     // this head's first 8-position group
    const int row_groups = a.Wp >> 3;   // one kernel row = this many 8-position groups
    const int row_bytes = row_groups * 512;
    const bf16* ybase = a.dYT + (((size_t)(o0 >> 5) * NG + g0) << 8) + (ptrdiff_t)(unit0 - 1) * 512;
    const bf16* xbase = a.XT + (((size_t)(i0 >> 5) * NG + g0) << 8) + (ptrdiff_t)(unit0 - 1) * 512 -
                        (ptrdiff_t)row_groups * 256;
    const int span = (max(unit1 - unit0, 0) + 2) * 1024;       // units unit0 - 1 .. unit1
    const __amdgpu_buffer_rsrc_t yrs = __builtin_amdgcn_make_buffer_rsrc((void*)ybase, 0, span, 0x00020000);
    const __amdgpu_buffer_rsrc_t xrs = __builtin_amdgcn_make_buffer_rsrc((void*)xbase, 0, span + 2 * row_bytes, 0x00020000);
    const unsigned lane_off = lhi * 512 + l32 * 16;
    const bool want_bias = it == 0;
    const int swap_addr = (lane ^ 32) << 2;   // ds_bpermute address of the lane holding the other half
    const bf16 one = (bf16)1.0f;
    const bf16x8 ones = {one, one, one, one, one, one, one, one};

    // Operand ring: the loads of unit u + DEPTH - 1 are issued before the MFMAs of unit u, so
    // that an L2 round trip is covered by matrix work of the same wavefront (there is only one
    // wavefront per SIMD: the accumulators take most of the register file).
#ifndef ST_WGRAD_DEPTH
#define ST_WGRAD_DEPTH 8
#endif
    constexpr int DEPTH = ST_WGRAD_DEPTH;
    u32x4 ry[DEPTH], rx[DEPTH][3];
#define WG_LOAD(SLOT, U)                                                                        \
    {                                                                                           \
        const int s_ = ((U) - unit0 + 1) * 1024;                                                \
        ry[SLOT] = __builtin_amdgcn_raw_buffer_load_b128(yrs, lane_off, s_, 0);                 \
        _Pragma("unroll") for (int kh = 0; kh < 3; ++kh)                                        \
            rx[SLOT][kh] = __builtin_amdgcn_raw_buffer_load_b128(xrs, lane_off, s_ + kh * row_bytes, 0); \
    }
    // The three taps of a kernel row differ by one position.  Moving the reduction index instead
    // of the window,
    //     dW[o][kh][kw][i] = sum_p dY[o][p - (kw - 1)] * X[i][p + (kh - 1) * Wp],
    // the kw = 0 / kw = 2 products use the same X fragment as kw = 1 and a dY fragment moved by
    // one position, which is built once per unit (not once per kernel row) in registers:
    // v_alignbyte over the lane's four dwords plus the one element that enters from the
    // neighbouring 8-position group.  That element sits in the *other half* of the wavefront
    // (lane ^ 32), in this unit's registers or in a neighbouring unit's, and is fetched with a
    // cross-lane permute, issued a unit before its result is picked up.
    //   up3_: dword 3 of lane^32 in the unit being prepared; dn0_: dword 0 of lane^32 in the unit
    //   after it.  For a lane of the lower half (lhi = 0) the element before its group is in the
    //   upper half of the *previous* unit (carry_prev) and the one after its group in the upper
    //   half of this unit (carry_next, fetched when the previous unit was prepared).
    // (dY is zero on the border of the padded grid and in the guard columns, so the terms the
    //  shift moves across the ends of the position range are zero.)
    unsigned int carry_prev, carry_next;
    unsigned int up3_, dn0_;              // permute results in flight
    u32x4 ymb[2], ypb[2];                 // dY at p - 1 / p + 1 of the unit in work and of the next one
#define WG_NEIGHBOURS_ISSUE(SLOT, NEXT)                                                         \
    {                                                                                           \
        up3_ = __builtin_amdgcn_ds_bpermute(swap_addr, ry[SLOT][3]);                            \
        dn0_ = __builtin_amdgcn_ds_bpermute(swap_addr, ry[NEXT][0]);                            \
    }
    // picks up the permutes issued for the unit in SLOT and builds its shifted fragments in BUF
#define WG_SHIFTED(SLOT, BUF)                                                                   \
    {                                                                                           \
        const unsigned int prev_ = lhi ? up3_ : carry_prev;                                     \
        const unsigned int next_ = lhi ? dn0_ : carry_next;                                     \
        carry_prev = up3_;                                                                      \
        carry_next = dn0_;                                                                      \
        const u32x4 w_ = ry[SLOT];                                                              \
        ymb[BUF][0] = __builtin_amdgcn_alignbyte(w_[0], prev_, 2);                              \
        ymb[BUF][1] = __builtin_amdgcn_alignbyte(w_[1], w_[0], 2);                              \
        ymb[BUF][2] = __builtin_amdgcn_alignbyte(w_[2], w_[1], 2);                              \
        ymb[BUF][3] = __builtin_amdgcn_alignbyte(w_[3], w_[2], 2);                              \
        ypb[BUF][0] = ymb[BUF][1]; ypb[BUF][1] = ymb[BUF][2]; ypb[BUF][2] = ymb[BUF][3];        \
        ypb[BUF][3] = __builtin_amdgcn_alignbyte(next_, w_[3], 2);                              \
    }
    // the same in two halves (the fragment at p - 1, then the one at p + 1), for the steady state:
    // five vector instructions each, which fit behind one MFMA; ten in a row do not
#define WG_SHIFTED_A(SLOT, BUF)                                                                 \
    {                                                                                           \
        const unsigned int prev_ = lhi ? up3_ : carry_prev;                                     \
        carry_prev = up3_;                                                                      \
        const u32x4 w_ = ry[SLOT];                                                              \
        ymb[BUF][0] = __builtin_amdgcn_alignbyte(w_[0], prev_, 2);                              \
        ymb[BUF][1] = __builtin_amdgcn_alignbyte(w_[1], w_[0], 2);                              \
        ymb[BUF][2] = __builtin_amdgcn_alignbyte(w_[2], w_[1], 2);                              \
        ymb[BUF][3] = __builtin_amdgcn_alignbyte(w_[3], w_[2], 2);                              \
    }
#define WG_SHIFTED_B(SLOT, BUF)                                                                 \
    {                                                                                           \
        const unsigned int next_ = lhi ? dn0_ : carry_next;                                     \
        carry_next = dn0_;                                                                      \
        ypb[BUF][0] = ymb[BUF][1]; ypb[BUF][1] = ymb[BUF][2]; ypb[BUF][2] = ymb[BUF][3];        \
        ypb[BUF][3] = __builtin_amdgcn_alignbyte(next_, ry[SLOT][3], 2);                        \
    }
#define WG_MMA(T, Y, KH, SLOT)                                                                  \
    acc[T] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(rx[SLOT][KH]), as_bf16x8(Y), acc[T], 0, 0, 0);
#define WG_F __builtin_amdgcn_sched_barrier(0);
    // One unit in slot D of the ring.  There is one wavefront per SIMD, so whatever this wavefront
    // issues between two MFMAs is all that can overlap them: the loads of unit + DEPTH - 1, the
    // pick-up of the permutes and the shifted fragments of unit + 1, and the permutes of unit + 2
    // are spread over the gaps between this unit's MFMAs, in a pinned order.
#define WG_UNIT(D, U, BIAS)                                                                     \
    {                                                                                           \
        const int L_ = ((D) + DEPTH - 1) % DEPTH, N1_ = ((D) + 1) % DEPTH;                      \
        const int N2_ = ((D) + 2) % DEPTH, N3_ = ((D) + 3) % DEPTH, B_ = (D) & 1;               \
        const int s_ = (min((U) + DEPTH - 1, unit1) - unit0 + 1) * 1024;                        \
        if (BIAS) acc[9] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ones, as_bf16x8(ry[D]), acc[9], 0, 0, 0); \
        WG_MMA(0, ypb[B_], 0, D) WG_F                                                           \
        ry[L_] = __builtin_amdgcn_raw_buffer_load_b128(yrs, lane_off, s_, 0); WG_F              \
        WG_MMA(1, ry[D], 0, D) WG_F                                                             \
        rx[L_][0] = __builtin_amdgcn_raw_buffer_load_b128(xrs, lane_off, s_, 0); WG_F           \
        WG_MMA(2, ymb[B_], 0, D) WG_F                                                           \
        rx[L_][1] = __builtin_amdgcn_raw_buffer_load_b128(xrs, lane_off, s_ + row_bytes, 0); WG_F \
        WG_MMA(3, ypb[B_], 1, D) WG_F                                                           \
        rx[L_][2] = __builtin_amdgcn_raw_buffer_load_b128(xrs, lane_off, s_ + 2 * row_bytes, 0); WG_F \
        WG_MMA(4, ry[D], 1, D) WG_F                                                             \
        WG_SHIFTED_A(N1_, 1 - B_) WG_F                                                          \
        WG_MMA(5, ymb[B_], 1, D) WG_F                                                           \
        WG_SHIFTED_B(N1_, 1 - B_) WG_F                                                          \
        WG_MMA(6, ypb[B_], 2, D) WG_F                                                           \
        WG_NEIGHBOURS_ISSUE(N2_, N3_) WG_F                                                      \
        WG_MMA(7, ry[D], 2, D)                                                                  \
        WG_MMA(8, ymb[B_], 2, D) WG_F                                                           \
    }
    // the same unit when it may lie beyond the end of the range (last, partial trip of the loop):
    // the bookkeeping runs as above, the MFMAs only for units inside the range
#define WG_UNIT_TAIL(D, U, BIAS)                                                                \
    {                                                                                           \
        const int L_ = ((D) + DEPTH - 1) % DEPTH, N1_ = ((D) + 1) % DEPTH;                      \
        const int N2_ = ((D) + 2) % DEPTH, N3_ = ((D) + 3) % DEPTH, B_ = (D) & 1;               \
        if ((U) < unit1) {                                                                      \
            if (BIAS) acc[9] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ones, as_bf16x8(ry[D]), acc[9], 0, 0, 0); \
            _Pragma("unroll") for (int kh = 0; kh < 3; ++kh) {                                  \
                WG_MMA(kh * 3 + 0, ypb[B_], kh, D)                                              \
                WG_MMA(kh * 3 + 1, ry[D], kh, D)                                                \
                WG_MMA(kh * 3 + 2, ymb[B_], kh, D)                                              \
            }                                                                                   \
        }                                                                                       \
        WG_F                                                                                    \
        WG_LOAD(L_, min((U) + DEPTH - 1, unit1))                                                \
        WG_SHIFTED(N1_, 1 - B_)                                                                 \
        WG_NEIGHBOURS_ISSUE(N2_, N3_) WG_F                                                      \
    }
#define WG_LOOPS(BIAS)                                                                          \
    {                                                                                           \
        int u = unit0;                                                                          \
        for (; u + DEPTH <= unit1; u += DEPTH) {                                                \
            _Pragma("unroll") for (int d = 0; d < DEPTH; ++d) WG_UNIT(d, u + d, BIAS)           \
        }                                                                                       \
        if (u < unit1) {                                                                        \
            _Pragma("unroll") for (int d = 0; d < DEPTH; ++d) WG_UNIT_TAIL(d, u + d, BIAS)      \
        }                                                                                       \
    }

    static_assert(DEPTH % 2 == 0 && DEPTH >= 4, "two fragment buffers alternate; permutes look three units ahead");
    if (unit0 < unit1) {
        // unit0 - 1 (guard columns make it readable) supplies the first left neighbours and
        // unit1 (tail guard) the last right neighbours
        // (all loads are unconditional, with the unit index clamped to unit1: a load under a
        //  branch would force the compiler to wait for every outstanding load at the join;
        //  past the end of the range the slots hold clamped re-loads, finite and unused)
        WG_LOAD(DEPTH - 1, unit0 - 1)
#pragma unroll
        for (int d = 0; d < DEPTH - 1; ++d) WG_LOAD(d, min(unit0 + d, unit1))
        carry_prev = __builtin_amdgcn_ds_bpermute(swap_addr, ry[DEPTH - 1][3]);
        carry_next = __builtin_amdgcn_ds_bpermute(swap_addr, ry[0][0]);
        WG_NEIGHBOURS_ISSUE(0, 1)
        WG_SHIFTED(0, 0)
        WG_NEIGHBOURS_ISSUE(1, 2)
        if (want_bias) WG_LOOPS(true) else WG_LOOPS(false)
    }
#undef WG_LOAD
#undef WG_NEIGHBOURS_ISSUE
#undef WG_SHIFTED
#undef WG_SHIFTED_A
#undef WG_SHIFTED_B
#undef WG_MMA
#undef WG_F
#undef WG_UNIT
#undef WG_UNIT_TAIL
#undef WG_LOOPS

    // ---- every wavefront leaves its block in LDS as [tap][o][i]; then all 256 threads add the
    //      four copies in the order ((w0 + w1) + w2) + w3 and write the result with 16-byte stores.
    //      The X fragment is the MFMA's A operand, so a lane holds four consecutive input channels
    //      i of one output channel o per register group: one 16-byte LDS write.  Rows are 128
    //      bytes; the 16-byte chunk c of row o is stored at chunk c ^ ((o >> 1) & 7), which spreads
    //      the 16 lanes of a write (and of a read) over all banks.
    float* red = (float*)smem_raw;                 // [4][9 * 32 rows][32]
    float* redb = red + 4 * 9 * 32 * 32;           // [4][32] sums of dY over the positions
    {
        const int sw = (l32 >> 1) & 7;
#pragma unroll
        for (int t = 0; t < 9; ++t)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const f32x4 v = {acc[t][gq * 4], acc[t][gq * 4 + 1], acc[t][gq * 4 + 2], acc[t][gq * 4 + 3]};
                *(f32x4*)(red + ((wave * 9 + t) * 32 + l32) * 32 + (((gq * 2 + lhi) ^ sw) << 2)) = v;
            }
    }
    // every row of acc[9] holds the sums over the positions: row 0 lives in lanes 0 .. 31
    if (want_bias && lhi == 0) redb[wave * 32 + l32] = acc[9][0];
    __syncthreads();
    float* dW = a.dW + head * a.head_out_stride + (size_t)split * a.split_stride;
    for (int q = tid; q < 9 * 32 * 8; q += 256) {
        const int row = q >> 3, part = q & 7;
        const int t = row >> 5, ol = row & 31;
        const int chunk = (part ^ ((ol >> 1) & 7)) << 2;
        const f32x4 v0 = *(const f32x4*)(red + ((0 * 9 * 32 + row) * 32 + chunk));
        const f32x4 v1 = *(const f32x4*)(red + ((1 * 9 * 32 + row) * 32 + chunk));
        const f32x4 v2 = *(const f32x4*)(red + ((2 * 9 * 32 + row) * 32 + chunk));
        const f32x4 v3 = *(const f32x4*)(red + ((3 * 9 * 32 + row) * 32 + chunk));
        const f32x4 sum = ((v0 + v1) + v2) + v3;
        *(f32x4*)(dW + ((size_t)(o0 + ol) * 9 + t) * a.cin + i0 + part * 4) = sum;
    }
    if (want_bias && tid < 32) {
        float* db = a.db + head * a.head_out_stride + (size_t)split * a.split_stride;
        db[o0 + tid] = ((redb[tid] + redb[32 + tid]) + redb[64 + tid]) + redb[96 + tid];
    }
}

bool wgrad3x3_mfma_supported(int cin, int cout) { return cin % 32 == 0 && cout % 32 == 0; }

// Position splits of the two layers for the shared launch.  Every block pays a fixed cost (ring
// fill, the reduction through LDS, the partial-result store: about 22 units' worth) on top of its
// units, blocks start in launch order on whichever compute unit is free, and every partial copy
// is read once more by the optimiser kernel.  The search simulates exactly that for every pair of
// split counts and keeps the shortest; among equals, fewer partial copies.
void wgrad_splits_for(const Geo& g, int* s1_out, int* s2_out)
{
    constexpr int n_cu = 256, fixed_units = 22, reread_units_per_chip = 13;
    const int tiles1 = g.heads() * (g.c1 / 32) * (g.c_in / 32), tiles2 = g.heads() * (g.c2 / 32) * (g.c1 / 32);
    const int n_units = cdiv(g.padded_positions() / g.heads(), 16);
    int best1 = 1, best2 = 1;
    long best_cost = -1;
    // compute units with the same free time form a group: (time, how many)
    struct Group { long t; long n; };
    auto run = [](std::vector<Group>& gs, long blocks, long d) {
        long makespan = 0;
        while (blocks > 0) {
            size_t e = 0;
            for (size_t i = 1; i < gs.size(); ++i)
                if (gs[i].t < gs[e].t) e = i;
            const long k = std::min(gs[e].n, blocks), t = gs[e].t + d;
            gs[e].n -= k;
            if (gs[e].n == 0) gs.erase(gs.begin() + e);
            size_t j = 0;
            for (; j < gs.size(); ++j)
                if (gs[j].t == t) break;
            if (j < gs.size()) gs[j].n += k; else gs.push_back(Group{t, k});
            makespan = std::max(makespan, t);
            blocks -= k;
        }
        return makespan;
    };
    std::vector<Group> gs;
    for (int s1 = 1; s1 <= 16; ++s1) {
        // keep at least 8 units (128 positions) per wavefront
        if (s1 > 1 && cdiv(n_units, s1 * 4) < 8) break;
        for (int s2 = 1; s2 <= 16; ++s2) {
            if (s2 > 1 && cdiv(n_units, s2 * 4) < 8) break;
            const long d1 = cdiv(n_units, s1 * 4) + fixed_units, d2 = cdiv(n_units, s2 * 4) + fixed_units;
            const long n1 = (long)tiles1 * s1, n2 = (long)tiles2 * s2;
            // list scheduling on n_cu units, layer 1 first
            gs.assign(1, Group{0, n_cu});
            long makespan = run(gs, n1, d1);
            makespan = std::max(makespan, run(gs, n2, d2));
            const long cost = (makespan * n_cu + reread_units_per_chip * (n1 + n2)) * 64 + s1 + s2;
            if (best_cost < 0 || cost < best_cost) { best_cost = cost; best1 = s1; best2 = s2; }
        }
    }
    *s1_out = best1; *s2_out = best2;
}

static WgradArgs wgrad_args(const Plan& p, const bf16* dYT, const bf16* XT, float* dW, float* db, int cin,
                            int cout, int splits)
{
    WgradArgs a;
    a.dYT = dYT; a.XT = XT; a.dW = dW; a.db = db;
    a.split_stride = p.grad_stride;
    a.cin = cin; a.cout = cout; a.PPT = p.PPT; a.guard = p.guard; a.Wp = p.g.Wp;
    a.heads = p.g.heads();
    a.n_units = cdiv(p.g.padded_positions() / a.heads, 16);
    a.head_groups8 = p.g.Hp * p.g.Wp / 8;
    a.head_out_stride = p.grad_stride * p.grad_copies;
    a.units_per_wave = cdiv(a.n_units, splits * 4);
    a.o_tiles = cout / 32; a.i_tiles = cin / 32;
    a.splits = splits;
    a.items_per_xcd = cdiv(a.o_tiles * a.i_tiles * splits * a.heads, 8);
    return a;
}

// weight and bias gradients of layer 1 (dY = da1, X = features) and layer 2 (dY = da2, X = a1)
void wgrad3x3_mfma(Ctx& c, const Plan& p, const bf16* da1T, const bf16* featT, const bf16* da2T,
                   const bf16* a1T, float* grad)
{
    const Geo& g = p.g;
    const WgradArgs a1 = wgrad_args(p, da1T, featT, grad + p.po.W1, grad + p.po.b1, g.c_in, g.c1, p.splits1);
    const WgradArgs a2 = wgrad_args(p, da2T, a1T, grad + p.po.W2, grad + p.po.b2, g.c1, g.c2, p.splits2);
    const int blocks1 = a1.items_per_xcd * 8, blocks2 = a2.items_per_xcd * 8;
    const size_t smem = (size_t)(4 * 9 * 32 * 32 + 4 * 32) * sizeof(float);
    ensure_dynamic_lds((const void*)k_wgrad3x3_mfma, smem);
    ST_LAUNCH(c, "conv12_wgrad_mfma", k_wgrad3x3_mfma, dim3(blocks1 + blocks2), dim3(256), smem, a1, a2, blocks1);
}

}  // namespace st

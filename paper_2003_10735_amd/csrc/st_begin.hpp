// Work that opens a call -- packing the features, the label-dependent half of the gradient --
// written as per-block device functions, so that it can run either as kernels of its own or as
// roles of the one launch that opens a call (k_call_begin, next to the optimiser kernel).
#pragma once
#include "st_kernels.hpp"
#include "st_mfma.hpp"

namespace st {

// features [n, c_in, h, w] (or [n, h, w, c_in]: Geo::nhwc) (Tin) -> padded position-major
// [n, Hp, Wp, c_in] (E) and, when
// outT != nullptr, a channel-major copy in the blocked layout of xt_index() for the
// weight-gradient kernel.
// One block (256 threads) transposes a 32-channel x 32-column tile of one row through LDS so that
// both the read (along x) and the write (along c) are contiguous.  Block coordinates: column
// tile bx, channel tile by, row bz = img * h + y.  `tile` is 32 x 33 floats of LDS.
template <class Tin, class E>
__device__ __forceinline__ void pack_features_block(const Tin* __restrict__ f, E* __restrict__ out,
                                                    E* __restrict__ outT, const Geo& g, int PPT, int guard,
                                                    int bx, int by, int bz, float (*tile)[33])
{
    const int x0 = bx * 32, c0 = by * 32;
    const int img = bz / g.h, y = bz % g.h;
    const int tx = threadIdx.x % 32, ty = threadIdx.x / 32;  // 32 x 8
    if (g.nhwc) {
        // channels are already the fast index: the position-major copy is a straight (padded)
        // copy, and only the channel-major one goes through the tile
        for (int k = ty; k < 32; k += 8) {
            const int x = x0 + k, c = c0 + tx;
            float v = 0.f;
            if (c < g.c_in && x < g.w) {
                v = to_f32(f[(((size_t)img * g.h + y) * g.w + x) * g.c_in + c]);
                out[(((size_t)img * g.Hp + y + 1) * g.Wp + x + 1) * g.c_in + c] = from_f32<E>(v);
            }
            tile[tx][k] = v;
        }
        if (!outT) return;
        __syncthreads();
        for (int k = ty; k < 32; k += 8) {
            const int c = c0 + k, x = x0 + tx;
            if (c < g.c_in && x < g.w)
                outT[xt_index(c, guard + (img * g.Hp + y + 1) * g.Wp + x + 1, PPT / 8)] = from_f32<E>(tile[k][tx]);
        }
        return;
    }
    for (int k = ty; k < 32; k += 8) {
        const int c = c0 + k, x = x0 + tx;
        float v = 0.f;
        if (c < g.c_in && x < g.w) v = to_f32(f[(((size_t)img * g.c_in + c) * g.h + y) * g.w + x]);
        tile[k][tx] = v;
        if (outT && c < g.c_in && x < g.w)
            outT[xt_index(c, guard + (img * g.Hp + y + 1) * g.Wp + x + 1, PPT / 8)] = from_f32<E>(v);
    }
    __syncthreads();
    for (int k = ty; k < 32; k += 8) {
        const int x = x0 + k, c = c0 + tx;
        if (c < g.c_in && x < g.w)
            out[(((size_t)img * g.Hp + y + 1) * g.Wp + x + 1) * g.c_in + c] = from_f32<E>(tile[tx][k]);
    }
}

// The same for bfloat16 in and out on the matrix-core path, with 16-byte accesses and covering the
// whole padded grid (zeros on the border), so that nothing of the two feature buffers but their
// guards needs clearing beforehand.  One block (256 threads): one padded row yp (bz = img * Hp + yp),
// 64 channels (by), 64 padded columns xp0 .. xp0 + 63 (bx).  Needs w % 8 == 0, c_in % 64 == 0 and a
// 16-byte aligned source.  `tile` is 64 rows of PACKV_PITCH bfloat16 in LDS.
constexpr int PACKV_PITCH = 64 + 8;
__device__ __forceinline__ void pack_features_vec_block(const bf16* __restrict__ f, bf16* __restrict__ out,
                                                        bf16* __restrict__ outT, const Geo& g, int PPT, int guard,
                                                        int bx, int by, int bz, bf16* tile)
{
    const int xp0 = bx * 64, c0 = by * 64;
    const int img = bz / g.Hp, yp = bz % g.Hp;
    const bool row_in = yp >= 1 && yp <= g.h;
    const int tid = threadIdx.x;
    // source chunks of 8 columns x = 8q .. 8q + 7 land at padded columns x + 1; the tile's first
    // padded column (a border or an x = 8k - 1) comes from the chunk before
    bf16x8 v[2];
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const int i = tid + r * 256, ch = i >> 3, q = i & 7;
        const int x = xp0 + 8 * q;                         // first column of the chunk
        v[r] = bf16x8{(bf16)0.f, (bf16)0.f, (bf16)0.f, (bf16)0.f, (bf16)0.f, (bf16)0.f, (bf16)0.f, (bf16)0.f};
        if (row_in && x < g.w) v[r] = *(const bf16x8*)(f + (((size_t)img * g.c_in + c0 + ch) * g.h + (yp - 1)) * g.w + x);
    }
    bf16 first = (bf16)0.f;                                // column xp0 - 1 of channel tid (threads 0 .. 63)
    if (tid < 64 && row_in && xp0 >= 1 && xp0 - 1 < g.w)
        first = f[(((size_t)img * g.c_in + c0 + tid) * g.h + (yp - 1)) * g.w + xp0 - 1];
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const int i = tid + r * 256, ch = i >> 3, q = i & 7;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int xl = 8 * q + e + 1;                  // padded column inside the tile
            if (xl < 64) tile[ch * PACKV_PITCH + xl] = v[r][e];
        }
    }
    if (tid < 64) tile[tid * PACKV_PITCH] = first;
    __syncthreads();
    const size_t prow = ((size_t)img * g.Hp + yp) * g.Wp;  // padded position of column 0 of this row
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const int i = tid + r * 256;
        {   // position-major: 8 channels of one position
            const int xl = i >> 3, cq = i & 7;
            if (xp0 + xl < g.Wp) {
                bf16x8 o;
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] = tile[(cq * 8 + e) * PACKV_PITCH + xl];
                *(bf16x8*)(out + (prow + xp0 + xl) * g.c_in + c0 + cq * 8) = o;
            }
        }
        {   // channel-major: 8 positions of one channel
            const int ch = i >> 3, g8 = i & 7;
            if (xp0 + 8 * g8 < g.Wp)
                *(bf16x8*)(outT + xt_index(c0 + ch, guard + (int)prow + xp0 + 8 * g8, PPT / 8)) =
                    *(const bf16x8*)(tile + ch * PACKV_PITCH + 8 * g8);
        }
    }
}

// weight with which frame index X (0 .. 8*len-1) contributes to cell `cell` of a line of `len`
// cells: the tent (1, 3, .. 15, 15, .. 3, 1)/16 around the cell, plus, for the first and last
// cell, the weight that edge replication folds back onto them
__device__ __forceinline__ float tap_weight(int X, int cell, int len)
{
    const int t = X - 8 * cell + 4;   // 0 .. 15 inside the tent
    float wgt = 0.f;
    if (t >= 0 && t < 16) wgt = (t < 8 ? 2 * t + 1 : 31 - 2 * t) * 0.0625f;
    if (cell == 0 && X < 4) wgt = 1.f;
    if (cell == len - 1 && X >= 8 * len - 4) wgt = 1.f;
    return wgt;
}

// T[img][c][cy][cx] = sum over valid pixels p with label c of wy(p, cy) * wx(p, cx).
// One block (256 threads) per cell row and run of 32 cells.  First every pixel column that can
// reach those cells (256 + 2 x 4 columns) adds its 16 rows' y-weights into a per-column table in
// LDS (the class index is data, so the table cannot live in registers); then one thread per
// (class, cell) applies the x-weights of the 16 columns under the cell.  All terms are
// multiples of 1/256 and the sums stay below 2^8 -- below 2^16 with 8-bit pixel weights -- so the
// result is exact in float32 and does not depend on the order of additions.
// colsum: CP x (LABEL_NCOL + 1) floats of LDS, CP >= number of classes; cnt_part: 4 words.
constexpr int LABEL_TX = 32;                 // 8-pixel column groups per block of this role
constexpr int LABEL_NCOL = LABEL_TX * 8 + 8;
__device__ __forceinline__ void label_adjoint_block(const int32_t* __restrict__ labels,
                                                    const uint8_t* __restrict__ wmap, float* __restrict__ T,
                                                    unsigned long long* __restrict__ n_valid, const Geo& g,
                                                    int block, float* colsum, unsigned int* cnt_part, int CP,
                                                    uint8_t* __restrict__ lab8)
{
    constexpr int NCOL = LABEL_NCOL, PITCH = LABEL_NCOL + 1;
    const int tid = threadIdx.x;
    const int tiles_x = (g.w + LABEL_TX - 1) / LABEL_TX;
    const int tx = block % tiles_x, cy = (block / tiles_x) % g.h, img = block / (tiles_x * g.h);
    const int hw = g.h * g.w;
    const int32_t* lab = labels + (size_t)img * g.H * g.W;
    const uint8_t* wm = wmap ? wmap + (size_t)img * g.H * g.W : nullptr;
    for (int i = tid; i < CP * PITCH; i += 256) colsum[i] = 0.f;
    __syncthreads();
    const int X0 = tx * LABEL_TX * 8 - 4;                  // frame column of table column 0
    const int Yt = 8 * cy - 4;                             // frame row of tent position 0
    unsigned int cnt = 0;     // valid labels (their weights) of this block's own 8 x 256 pixels
    // A thread takes table column tid and, the first NCOL - 256 threads, column tid + 256 as
    // well.  The loads of both columns are issued before either is worked on: one trip to memory
    // for the block instead of two.
    static_assert(NCOL > 256 && NCOL <= 512, "one or two columns per thread");
    const bool second = tid < NCOL - 256;
    int ys[2][16];
    unsigned int ws[2][16];
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        if (k == 1 && !second) break;
        const int Xc = min(max(X0 + tid + 256 * k, 0), g.W - 1);
        // the 16 rows under the tent (clamped, so that no load depends on a branch of its own)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const size_t at = (size_t)min(max(Yt + r, 0), g.H - 1) * g.W + Xc;
            ys[k][r] = lab[at];
            ws[k][r] = wm ? wm[at] : 1u;
        }
    }
#pragma unroll
    for (int k = 0; k < 2; ++k) {
        if (k == 1 && !second) break;
        const int col = tid + 256 * k;
        const int X = X0 + col;
        const bool xin = X >= 0 && X < g.W;
        const bool own_col = col >= 4 && col < NCOL - 4;
        // label maps are piecewise constant: rows with the same label are added up in a register
        // and reach the table once per run (all terms are multiples of 1/256, so any grouping of
        // the additions gives the same float32 sum)
        int run_y = -1;
        float run = 0.f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int Y = Yt + r, y = ys[k][r];
            const bool ok = xin && Y >= 0 && Y < g.H && y != g.ignore_index && y >= 0 && y < g.C;
            const int yy = ok ? y : -1;
            if (yy != run_y) {
                if (run_y >= 0) colsum[run_y * PITCH + col] += run;
                run_y = yy;
                run = 0.f;
            }
            if (ok) {
                run += (float)ws[k][r] * tap_weight(Y, cy, g.h);
                if (own_col && r >= 4 && r < 12) cnt += ws[k][r];
            }
            // the block's own 8 x 256 pixels as bytes for the loss kernel, which reads them in every
            // pass: the class, or 255 where the pixel does not count (a quarter of the bytes)
            if (lab8 && xin && own_col && r >= 4 && r < 12)
                lab8[(size_t)img * g.H * g.W + (size_t)Y * g.W + X] = ok ? (uint8_t)y : (uint8_t)255;
        }
        if (run_y >= 0) colsum[run_y * PITCH + col] += run;
    }
    if (n_valid) {
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) cnt += __shfl_down(cnt, off, 64);
        if ((tid & 63) == 0) cnt_part[tid >> 6] = cnt;
    }
    __syncthreads();
    if (n_valid && tid == 0)
        atomicAdd(n_valid + g.head_of(img), (unsigned long long)(cnt_part[0] + cnt_part[1] + cnt_part[2] + cnt_part[3]));
    for (int i = tid; i < g.C * LABEL_TX; i += 256) {
        const int lc = i % LABEL_TX, c = i / LABEL_TX;
        const int cx = tx * LABEL_TX + lc;
        if (cx >= g.w) continue;
        float acc = 0.f;
#pragma unroll
        for (int t = 0; t < 16; ++t) {
            const int X = 8 * cx - 4 + t;                  // table column 8 * lc + t
            if (X >= 0 && X < g.W) acc += tap_weight(X, cx, g.w) * colsum[c * PITCH + 8 * lc + t];
        }
        T[((size_t)img * g.C + c) * hw + cy * g.w + cx] = acc;
    }
}

}  // namespace st

// Bookkeeping of a forward pass (role (3) of the step-closing kernel): per-frame mean IoU from the
// confusion counts, the tile losses added in a fixed order.  A header of its own because the role
// also rides on other launches (the classifier's backward kernel in the early-exit form).
#pragma once
#include "st_common.hpp"

namespace st {

struct FinishArgs {
    const float* loss_part; int n_part; const unsigned long long* n_valid; unsigned long long* conf;
    int n, C; float* loss_out; double* miou_a; double* miou_b; long long* conf_out;
    // per head (blockIdx.y): fph frames and pph tile losses; one head owns all of them
    int fph, pph;
    // early-exit form only: host memory that also receives the per-frame metric, each value followed by
    // the pass's token in token_c (or null)
    double* miou_c; unsigned long long* token_c; unsigned long long token;
};

// (EE: the early-exit form's extra -- the host copy of the metric -- is compiled in)
template <bool EE>
__device__ void finish_block(const FinishArgs& f, int block, int head)
{
    __shared__ double part[256];
    __shared__ unsigned long long cl[32 * 32];
    __shared__ double iou[32];
    __shared__ int present[32];
    const int tid = threadIdx.x;
    if (block == f.fph) {
        double acc = 0.0;
        const int per = (f.pph + 255) / 256;
        const float* lp = f.loss_part + (size_t)head * f.pph;
        for (int i = tid * per; i < min(f.pph, (tid + 1) * per); ++i) acc += (double)lp[i];
        part[tid] = acc;
        __syncthreads();
        for (int s = 128; s > 0; s >>= 1) {
            if (tid < s) part[tid] += part[tid + s];
            __syncthreads();
        }
        if (tid == 0 && f.loss_out) {
            const unsigned long long nv = f.n_valid[head];
            f.loss_out[head] = nv ? (float)(part[0] / (double)nv) : 0.f;
        }
        return;
    }
    block += head * f.fph;      // the frame
    const int C = f.C;
    unsigned long long* cf = f.conf + (size_t)block * C * C;
    for (int i = tid; i < C * C; i += 256) {
        const unsigned long long v = cf[i];
        cl[i] = v;
        if (f.conf_out) f.conf_out[(size_t)block * C * C + i] = (long long)v;
        cf[i] = 0ull;
    }
    __syncthreads();
    // IoU_c = conf[c][c] / (row_c + col_c - conf[c][c]) for classes with row_c > 0, added in
    // ascending c in float64, divided by their number; 0 when no class is present
    if (tid < C) {
        unsigned long long row = 0, col = 0;
        for (int k = 0; k < C; ++k) { row += cl[tid * C + k]; col += cl[k * C + tid]; }
        const unsigned long long inter = cl[tid * C + tid];
        present[tid] = row != 0;
        iou[tid] = row ? (double)inter / (double)(row + col - inter) : 0.0;
    }
    __syncthreads();
    if (tid == 0) {
        double sum = 0.0;
        int cnt = 0;
        for (int c = 0; c < C; ++c)
            if (present[c]) { sum += iou[c]; ++cnt; }
        const double m = cnt ? sum / cnt : 0.0;
        if (f.miou_a) f.miou_a[block] = m;
        if (f.miou_b) f.miou_b[block] = m;
        if (EE && f.miou_c) {
            // host memory: the value, then the pass's token as a release at system scope, so a host
            // that sees the token also sees the value
            f.miou_c[block] = m;
            if (f.token_c) __hip_atomic_store(&f.token_c[block], f.token, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_SYSTEM);
        }
    }
}

}  // namespace st

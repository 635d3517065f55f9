// Layout kernels: zero fill and the permutation between the caller's parameter order (OIHW) and
// the internal one ([o][kh][kw][i]).
#include "st_kernels.hpp"
#include "st_mfma.hpp"

namespace st {

// Clears a list of regions in one launch: region r owns blocks [first[r], first[r + 1]), each
// block a fixed run of ZERO_PER_BLOCK 16-byte words.
constexpr int ZERO_PER_BLOCK = 256 * 8;

__global__ void __launch_bounds__(256) k_zero_regions(ZeroList z)
{
    int r = 0;
    while (r + 1 < z.n && (int)blockIdx.x >= z.first[r + 1]) ++r;     // block-uniform, n is small
    uint4* p = (uint4*)z.ptr[r];
    const size_t base = (size_t)((int)blockIdx.x - z.first[r]) * ZERO_PER_BLOCK;
    const uint4 zero = make_uint4(0, 0, 0, 0);
#pragma unroll
    for (int k = 0; k < ZERO_PER_BLOCK / 256; ++k) {
        const size_t i = base + (size_t)k * 256 + threadIdx.x;
        if (i < z.n16[r]) p[i] = zero;
    }
}

void ZeroList::add(void* p, size_t bytes)
{
    if (bytes == 0 || n >= MAX) { overflow = overflow || (bytes != 0); return; }
    ptr[n] = p;
    n16[n] = (bytes + 15) / 16;
    first[n + 1] = first[n] + (int)((n16[n] + ZERO_PER_BLOCK - 1) / ZERO_PER_BLOCK);
    ++n;
}

// all workspace regions are 16-byte aligned and padded to 16 bytes
void zero_regions(Ctx& c, const ZeroList& z)
{
    if (z.overflow) { c.status = ST_ERR_SHAPE; return; }
    if (z.n == 0) return;
    ST_LAUNCH(c, "zero_fill", k_zero_regions, dim3(z.first[z.n]), dim3(256), 0, z);
}

__global__ void __launch_bounds__(256) k_zero8(unsigned long long* p, size_t n)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = 0ull;
}

void zero_u64(Ctx& c, unsigned long long* p, size_t n)
{
    if (n == 0) return;
    int blocks = (int)((n + 255) / 256);
    if (blocks > 1024) blocks = 1024;
    ST_LAUNCH(c, "zero_fill", k_zero8, dim3(blocks), dim3(256), 0, p, n);
}

// Parameter permutation.  dir = 0: external (OIHW) -> internal; dir = 1: internal -> external.
// Thread j walks the internal index; inside a 3x3 weight block
//   internal (o*9 + tap)*ci + i   <->   external (o*ci + i)*9 + tap.
__global__ void __launch_bounds__(256)
k_permute_params(const float* __restrict__ src, float* __restrict__ dst, ParamOffsets po,
                 int ci1, int ci2, int dir, size_t head_stride)
{
    const size_t j = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= po.total) return;
    // one head per blockIdx.y: internal blocks head_stride floats apart, external ones back to back
    src += blockIdx.y * (dir == 0 ? po.total : head_stride);
    dst += blockIdx.y * (dir == 0 ? head_stride : po.total);
    size_t e = j;
    if (j < po.b1) {
        const size_t r = j - po.W1;
        const size_t i = r % ci1, tap = (r / ci1) % 9, o = r / ((size_t)ci1 * 9);
        e = po.W1 + (o * ci1 + i) * 9 + tap;
    } else if (j >= po.W2 && j < po.b2) {
        const size_t r = j - po.W2;
        const size_t i = r % ci2, tap = (r / ci2) % 9, o = r / ((size_t)ci2 * 9);
        e = po.W2 + (o * ci2 + i) * 9 + tap;
    }
    if (dir == 0) dst[j] = src[e];
    else dst[e] = src[j];
}

void permute_params(Ctx& c, const Plan& p, const float* src, float* dst, int dir)
{
    ST_LAUNCH(c, dir == 0 ? "params_to_internal" : "params_from_internal", k_permute_params,
              dim3(cdiv(p.po.total, 256), p.g.heads()), dim3(256), 0, src, dst, p.po, p.g.c_in, p.g.c1, dir,
              p.head_stride);
}

}  // namespace st

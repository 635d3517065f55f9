// Loss weights from the teacher's label map (Section 5.2: the cross-entropy of pixels near and
// within non-background objects is scaled by a factor; "near" = within `radius` pixels along x
// and along y).  One launch, one pass over the labels: 4 bytes read and 1 byte written per pixel.
//
// A block owns a tile of OW_TH rows x 256 columns.  The object mask lives in LDS as a bit matrix,
// one 64-bit word per 64 consecutive pixels of a row: a wavefront loads 64 consecutive labels (one
// coalesced 256-byte read) and a single ballot turns them into a word.  The tile's mask is taken
// with `radius` more rows above and below and one more word on either side, then spread along x
// with shifts (bits cross word boundaries through the neighbouring words; radius <= 32 < 64, so
// one neighbour per side is enough), then along y by OR-ing 2 radius + 1 rows.  Pixels outside
// the frame hold no object.  Each thread finally writes four pixels of the result.
#include "st_common.hpp"
#include "st_kernels.hpp"

namespace st {

constexpr int OW_TH = 16;                    // rows of a tile
constexpr int OW_WORDS = 4;                  // 64-pixel words of a tile row
constexpr int OW_TW = 64 * OW_WORDS;         // columns of a tile
constexpr int OW_THREADS = 1024;
constexpr int OW_BATCH = 12;                 // label loads a wavefront keeps in flight
constexpr int OW_ROWS = OW_TH + 2 * ST_OBJECT_WEIGHTS_MAX_RADIUS;   // most mask rows a tile looks at
static_assert(OW_THREADS * 4 == OW_TH * OW_TW, "four result pixels per thread");
static_assert(ST_OBJECT_WEIGHTS_MAX_RADIUS < 64, "one neighbouring word per side");

__global__ void __launch_bounds__(OW_THREADS)
k_object_weights(const int32_t* __restrict__ labels, int H, int W, int C, int background, int ignore, int radius,
                 int factor, uint8_t* __restrict__ out)
{
    __shared__ unsigned long long obj[OW_ROWS * (OW_WORDS + 2)];   // object bits, one halo word per side
    __shared__ unsigned long long hor[OW_ROWS * OW_WORDS];         // spread along x
    __shared__ unsigned long long ver[OW_TH * OW_WORDS];           // and along y
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int x0 = blockIdx.x * OW_TW, y0 = blockIdx.y * OW_TH;
    const size_t frame = (size_t)blockIdx.z * H * W;
    const int rows = OW_TH + 2 * radius;

    // object bits of rows y0 - radius .. y0 + OW_TH + radius - 1, columns x0 - 64 .. x0 + OW_TW + 63;
    // OW_BATCH loads of a wavefront are in flight before the first ballot needs its labels (with
    // a radius of up to 8 that is all a wavefront has to load: one round trip to memory)
    constexpr int WAVES = OW_THREADS / 64;
    const int items = rows * (OW_WORDS + 2);
    for (int i0 = wave; i0 < items; i0 += OW_BATCH * WAVES) {
        int v[OW_BATCH];
#pragma unroll
        for (int k = 0; k < OW_BATCH; ++k) {
            const int i = i0 + k * WAVES;
            const int row = i / (OW_WORDS + 2), word = i - row * (OW_WORDS + 2);
            const int y = y0 - radius + row, x = x0 - 64 + 64 * word + lane;
            v[k] = -1;                                  // no class: outside the frame or the tile's mask
            if (i < items && y >= 0 && y < H && x >= 0 && x < W) v[k] = labels[frame + (size_t)y * W + x];
        }
#pragma unroll
        for (int k = 0; k < OW_BATCH; ++k) {
            const int i = i0 + k * WAVES;               // the same for all lanes of a wavefront
            if (i < items) {
                const unsigned long long m = __ballot(v[k] >= 0 && v[k] < C && v[k] != background && v[k] != ignore);
                if (lane == 0) obj[i] = m;
            }
        }
    }
    __syncthreads();

    // bit x of the result = OR of bits x - radius .. x + radius
    for (int j = threadIdx.x; j < rows * OW_WORDS; j += OW_THREADS) {
        const int row = j / OW_WORDS, word = j - row * OW_WORDS;
        const unsigned long long* o = obj + row * (OW_WORDS + 2) + word;
        const unsigned long long left = o[0], mid = o[1], right = o[2];
        unsigned long long h = mid;
        for (int s = 1; s <= radius; ++s)
            h |= (mid >> s) | (right << (64 - s)) | (mid << s) | (left >> (64 - s));
        hor[j] = h;
    }
    __syncthreads();

    if (threadIdx.x < OW_TH * OW_WORDS) {
        const int row = threadIdx.x / OW_WORDS, word = threadIdx.x - row * OW_WORDS;
        unsigned long long v = 0;
        for (int d = 0; d <= 2 * radius; ++d) v |= hor[(row + d) * OW_WORDS + word];
        ver[threadIdx.x] = v;
    }
    __syncthreads();

    // four consecutive pixels per thread: one 4-byte store where the address allows it
    const int row = threadIdx.x / (OW_TW / 4), quad = threadIdx.x - row * (OW_TW / 4);
    const int y = y0 + row, x = x0 + 4 * quad;
    if (y < H && x < W) {
        const unsigned int bits = (unsigned int)(ver[row * OW_WORDS + (quad >> 4)] >> (4 * (quad & 15))) & 15u;
        uint8_t* dst = out + frame + (size_t)y * W + x;
        unsigned int packed = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) packed |= (unsigned int)(((bits >> i) & 1u) ? factor : 1) << (8 * i);
        if (x + 4 <= W && ((uintptr_t)dst & 3) == 0) {
            *(unsigned int*)dst = packed;
        } else {
            for (int i = 0; i < 4 && x + i < W; ++i) dst[i] = (uint8_t)(packed >> (8 * i));
        }
    }
}

void object_weights(Ctx& c, const int32_t* labels, int n, int H, int W, int C, int background, int ignore, int radius,
                    int factor, uint8_t* out)
{
    ST_LAUNCH(c, "object_weights", k_object_weights, dim3(cdiv(W, OW_TW), cdiv(H, OW_TH), n), dim3(OW_THREADS), 0,
              labels, H, W, C, background, ignore, radius, factor, out);
}

}  // namespace st

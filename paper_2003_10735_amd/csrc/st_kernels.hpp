// Host-side launchers of the kernels, one group per source file.
#pragma once
#include "st_common.hpp"

namespace st {

struct FinishArgs;   // st_finish.hpp: arguments of the bookkeeping role

// k_layout.hip
// regions to clear, each 16-byte aligned and padded to 16 bytes; one launch clears them all
struct ZeroList {
    static constexpr int MAX = 96;
    void* ptr[MAX]; size_t n16[MAX]; int first[MAX + 1]; int n = 0; bool overflow = false;
    ZeroList() { first[0] = 0; }
    void add(void* p, size_t bytes);
};
void zero_regions(Ctx& c, const ZeroList& z);
void zero_u64(Ctx& c, unsigned long long* p, size_t n);
void permute_params(Ctx& c, const Plan& p, const float* src, float* dst, int dir);

// k_conv_generic.hip -- plain tiled kernels (float32 path; bfloat16 shapes the MFMA kernels skip)
void generic_forward(Ctx& c, const Plan& p, char* ws, float* z);
void generic_backward(Ctx& c, const Plan& p, char* ws);
void generic_feature_grad(Ctx& c, const Plan& p, char* ws, float* dfeat);

// k_conv_mfma.hip, k_wgrad_mfma.hip, k_conv3_mfma.hip -- matrix-core kernels of the bfloat16 path
bool conv3x3_mfma_supported(int cin, int cout);
void conv3x3_mfma(Ctx& c, const char* name, const Plan& p, const bf16* X, const bf16* Wq, const float* bias,
                  const bf16* mask, bf16* Y, bf16* YT, int cin, int cout, int epi, int layer,
                  const bf16* W3q = nullptr, float* zpart = nullptr, float* dense = nullptr);
bool wgrad3x3_mfma_supported(int cin, int cout);
void wgrad_splits_for(const Geo& g, int* splits1, int* splits2);
void generic_wgrad_splits(const Geo& g, int* splits1, int* splits2, int* splits3);
void wgrad3x3_mfma(Ctx& c, const Plan& p, const bf16* da1T, const bf16* featT, const bf16* da2T,
                   const bf16* a1T, float* grad);
bool conv3_mfma_supported(int c2, int C);
int conv3_bwd_blocks(const Geo& g);
size_t conv3_bwd_slot_floats(const Geo& g);
// finish: the bookkeeping of the pass that precedes this backward pass rides on the launch (a few more blocks)
void conv3_bwd_mfma(Ctx& c, const Plan& p, const float* slots, const float* T,
                    const unsigned long long* n_valid, const bf16* a2, const bf16* W3T,
                    bf16* da2, bf16* da2T, float* part,
                    const FinishArgs* finish = nullptr);

// k_loss.hip
size_t loss_slot_floats(const Geo& g);
int loss_blocks(const Geo& g);
// Where the loss kernel finds the low-resolution logits: either the planar tensor [n, C, h, w], or
// the shares the classifier-fused convolution left behind, [n_parts][padded position][classes rounded up to a multiple of four],
// to be added in ascending order together with the bias b3; in that case the kernel also writes
// the sums to the planar tensor z_out (each tile its own cells), if given.
struct ZSrc {
    const float* planar;
    const float* parts; int n_parts; const float* b3; float* z_out;
    size_t b3_stride;     // floats between the biases of two heads (one head per frame)
};
// labels8: the labels as bytes (class, or 255 where the pixel does not count), or null: no loss, prediction only
void loss_pass(Ctx& c, const Geo& g, const ZSrc& zs, const uint8_t* labels8, const uint8_t* pixel_weights,
               const float* T, uint8_t* pred,
               float* slots, float* gz, float* loss_part, unsigned long long* conf,
               const unsigned long long* n_valid, bool grad, bool assemble);

// k_update.hip
// (every per-head quantity below -- parameters, optimiser state, partial gradients, weight copies,
//  the caller's vectors -- holds Geo::heads() blocks; the kernels take the head from blockIdx.y)
// One Adam step's constants, prepared on the host in double precision:
//   theta <- theta - step_scale * m / (sqrt(v) * inv_sqrt_bc2 + eps),
//   step_scale = lr / (1 - beta1^t),  inv_sqrt_bc2 = 1 / sqrt(1 - beta2^t).
struct AdamStep { float beta1, beta2, one_minus_beta1, one_minus_beta2, eps, step_scale, inv_sqrt_bc2; };
bool pack_covers_borders(const Plan& p, const void* features, int feat_dtype);
void call_begin(Ctx& c, const Plan& p, char* ws, const void* features, int feat_dtype, const float* head_params,
                bool w1t, const int32_t* labels, const uint8_t* pixel_weights);
void step_end(Ctx& c, const Plan& p, char* ws, float lr, float mu, const AdamStep* adam, bool do_step, bool finish, float* loss_out,
              double* miou_out, long long* conf_out, const float* ext_in = nullptr,
              bool w1t = false, float* save_old = nullptr);
// arguments of the bookkeeping role; miou_host / token_host / token as for finish_pass
FinishArgs finish_args(const Plan& p, char* ws, float* loss_out, double* miou_out, long long* conf_out,
                       double* miou_host = nullptr, unsigned long long* token_host = nullptr,
                       unsigned long long token = 0);
// miou_host: host memory the device can write (or null) that also receives the per-frame metric,
// each value followed by `token` in token_host (a release store at system scope)
void finish_pass(Ctx& c, const Plan& p, char* ws, float* loss_out, double* miou_out, long long* conf_out,
                 float* ext_out = nullptr, double* miou_host = nullptr, unsigned long long* token_host = nullptr,
                 unsigned long long token = 0);
void confusion_and_miou(Ctx& c, const uint8_t* pred, const int32_t* labels, long long P, int C, int ignore,
                        long long* conf, double* miou);

// k_weights.hip
void object_weights(Ctx& c, const int32_t* labels, int n, int H, int W, int C, int background, int ignore, int radius,
                    int factor, uint8_t* out);

}  // namespace st

// Shared by the CNN gradient translation units: bf16 helpers, layer descriptors, dispatch.
#pragma once

#include <vector>

#include "dpsgd_internal.h"

namespace dpsgd {

typedef unsigned short bf16_t;

__device__ __forceinline__ bf16_t f2bf(float f)
{   // round to nearest, ties to even
    unsigned u = __float_as_uint(f);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (bf16_t)(u >> 16);
}
__device__ __forceinline__ float bf2f(bf16_t h) { return __uint_as_float((unsigned)h << 16); }
__device__ __forceinline__ bool bf16_positive(bf16_t h) { return (h & 0x7fffu) != 0 && (h & 0x8000u) == 0; }

// One 3x3 convolution (zero padding 1): input Ci x H x W, output Co x Ho x Wo, weights at w_off
// ([Co][Ci][3][3] fp32) and one scalar bias at b_off inside a worker's parameter vector.
struct ConvDesc {
    int Ci, Co, H, W, Ho, Wo, stride;
    long long w_off, b_off;
};

struct ResnetPlan {
    std::vector<ConvDesc> convs;   // [0] stem, then conv1, conv2 of each block
    long long fcw_off = 0, fcb_off = 0;
    int classes = 0, C_last = 0, H_last = 0, W_last = 0, nblocks = 0;
};

ResnetPlan make_resnet_plan(const dpsgd_model_desc &m);

// out = round(ReLU(conv(in) + bias + shortcut)); in/out NHWC bf16 [n][B][H][W][C].  sc (may be null):
// the block input, added at (y*scS, x*scS) for the first scC output channels.
dpsgd_status conv_forward(dpsgd_ctx *ctx, const ConvDesc &c, int B, const bf16_t *in, const float *X, const bf16_t *sc,
                          int scC, int scH, int scW, int scS, bf16_t *out);
// din = round([act > 0] * (conv^T(dout) + shortcut delta)); scd (may be null): delta of the block output.
dpsgd_status conv_data_grad(dpsgd_ctx *ctx, const ConvDesc &c, int B, const bf16_t *dout, const float *X,
                            const bf16_t *scd, int scC, int scH, int scW, int scS, const bf16_t *act, bf16_t *din);
// G[w_off..] = dout (*) in, G[b_off] = sum(dout).
dpsgd_status conv_weight_grad(dpsgd_ctx *ctx, const ConvDesc &c, int B, const bf16_t *in, const bf16_t *dout, float *G);

dpsgd_status conv_forward_generic(dpsgd_ctx *ctx, const ConvDesc &c, int B, const bf16_t *in, const float *X,
                                  const bf16_t *sc, int scC, int scH, int scW, int scS, bf16_t *out);
dpsgd_status conv_data_grad_generic(dpsgd_ctx *ctx, const ConvDesc &c, int B, const bf16_t *dout, const float *X,
                                    const bf16_t *scd, int scC, int scH, int scW, int scS, const bf16_t *act,
                                    bf16_t *din);
dpsgd_status conv_weight_grad_generic(dpsgd_ctx *ctx, const ConvDesc &c, int B, const bf16_t *in, const bf16_t *dout,
                                      float *G);

}  // namespace dpsgd

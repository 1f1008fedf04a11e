// Shared by the CNN gradient translation units: bf16 helpers, layer descriptors, dispatch.
#pragma once

#include <vector>

#include "dpsgd_internal.h"

namespace dpsgd {

typedef unsigned short bf16_t;

__device__ __forceinline__ bf16_t f2bf(float f)
{   // round to nearest, ties to even (v_cvt_pk_bf16_f32)
    const __bf16 h = (__bf16)f;
    return __builtin_bit_cast(unsigned short, h);
}
__device__ __forceinline__ unsigned f2bf_pack(float lo, float hi)
{
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    const f32x2_t v = {lo, hi};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2_t));
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

// An activation or delta tensor: bf16, channel-major [n][B][C][H][W].  The weight gradient contracts
// over pixels and reads them contiguously; forward and data gradient contract over channels and
// transpose their source rows on the way into LDS; epilogues read and write 4 consecutive pixels
// of one channel.
// `sign` (may be null): one bit per element of an activation, stored per band of 8 rows:
// [n][B][H / 8][C][8 rows][W / 8] bytes, bit i of a byte = pixel 8 k + i of that row is positive.  The MFMA forward kernel writes it next to the activation and the MFMA data gradient reads
// it as its ReLU mask instead of the 16 times larger activation.
struct Tensor {
    bf16_t *t = nullptr;
    unsigned char *sign = nullptr;
};
// Forward: the block input added to the block output at (y*S, x*S) for the first C channels.
// Backward: the delta of the block output added to the block input's delta at multiples of S.
struct ShortcutRef {
    const bf16_t *t;
    int C, H, W, S;
};

// out = round(ReLU(conv(in) + bias + shortcut)).  wpack: this conv's packed bf16 weights (see conv_pack_weights).
// For the stem on MFMA (conv_stem_uses_mfma) `in` is the image padded to 8 channels, pixel-major.
dpsgd_status conv_forward(dpsgd_ctx *ctx, const ConvDesc &c, int B, Tensor in, const float *X, const bf16_t *wpack,
                          ShortcutRef sc, Tensor out);
// A residual block that keeps the resolution, both convolutions in one launch: u = conv_forward(c1, in),
// out = conv_forward(c2, u, shortcut = in), the same bits, without reading u back from memory.  _ok: whether the
// shapes allow it (stride 1; 16 channels on images of 16 or 32 pixels by a multiple of 8 rows, 32 channels on images of
// 16 x 16 pixels, 64 channels on images of 8 x 8 pixels; "conv_block" option on).
bool conv_block_forward_ok(const dpsgd_ctx *ctx, const ConvDesc &c1, const ConvDesc &c2);
dpsgd_status conv_block_forward(dpsgd_ctx *ctx, const ConvDesc &c1, const ConvDesc &c2, int B, Tensor in, const float *X,
                                const bf16_t *wpack1, const bf16_t *wpack2, Tensor u, Tensor out);
// din = round([act > 0] * (conv^T(dout) + shortcut delta)).
dpsgd_status conv_data_grad(dpsgd_ctx *ctx, const ConvDesc &c, int B, Tensor dout, const float *X, const bf16_t *wpack_d,
                            ShortcutRef scd, Tensor act, Tensor din);
// The weight-gradient kernels of the MFMA path leave partial sums (several workgroups per worker); what turns them
// into G is collected here and done for all convolutions of the network by ONE launch, conv_weight_grad_finish.
struct WgradReduceList {
    alignas(8) unsigned char table[2560];   // the job table the reduction kernel takes as its argument
    int njobs = 0, blocks = 0;
};
// G[w_off..] = dout (*) in, G[b_off] = sum(dout).  partials: this conv's own scratch of conv_wgrad_partial_bytes(c, B) * n
// bytes, which must stay untouched until conv_weight_grad_finish(pending) has run on the same stream; G holds the
// result only after that call.  Without partials or pending (or for shapes the MFMA kernel does not take) G is
// written directly.
dpsgd_status conv_weight_grad(dpsgd_ctx *ctx, const ConvDesc &c, int B, Tensor in, Tensor dout, float *G, float *partials,
                              WgradReduceList *pending);
dpsgd_status conv_weight_grad_finish(dpsgd_ctx *ctx, WgradReduceList *pending, float *G);

// Bytes per worker of the packed weights of one conv (forward operand, or data-gradient operand).
size_t conv_pack_bytes(const ConvDesc &c, bool dgrad);
size_t conv_wgrad_partial_bytes(const ConvDesc &c, int B);
// Rounds the fp32 weights of every conv and worker to bf16 in MFMA operand order (forward and data-gradient
// operands, wpack_f[q] / wpack_d[q] for convs[q]; nothing is written for convs the MFMA kernels do not take).
dpsgd_status conv_pack_weights(dpsgd_ctx *ctx, const std::vector<ConvDesc> &convs, const float *X,
                               const std::vector<bf16_t *> &wpack_f, const std::vector<bf16_t *> &wpack_d);

// Stem support: whether the first conv runs on MFMA, and the image copies it then needs: a bf16
// channel-major copy (only made from fp32 images; may be null) and the image padded to 8 channels (NHWC8).
bool conv_stem_uses_mfma(const ConvDesc &c);
// Whether conv_forward fills out.sign for this conv (the stem counts only when it runs on MFMA).
bool conv_forward_writes_sign(const ConvDesc &c, bool is_stem);
dpsgd_status conv_prep_image(dpsgd_ctx *ctx, const ConvDesc &c, int B, const void *image, bool image_is_bf16,
                             bf16_t *chw_bf16, bf16_t *nhwc8);

dpsgd_status conv_forward_generic(dpsgd_ctx *ctx, const ConvDesc &c, int B, Tensor in, const float *X, ShortcutRef sc,
                                  Tensor out);
dpsgd_status conv_data_grad_generic(dpsgd_ctx *ctx, const ConvDesc &c, int B, Tensor dout, const float *X,
                                    ShortcutRef scd, Tensor act, Tensor din);
dpsgd_status conv_weight_grad_generic(dpsgd_ctx *ctx, const ConvDesc &c, int B, Tensor in, Tensor dout, float *G);

}  // namespace dpsgd

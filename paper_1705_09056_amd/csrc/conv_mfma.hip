// Dispatch of the CNN's convolutions: MFMA kernels for the benchmark's channel counts, the
// shape-generic kernels otherwise.
#include "resnet_common.h"

namespace dpsgd {

dpsgd_status conv_forward(dpsgd_ctx *ctx, const ConvDesc &c, int B, const bf16_t *in, const float *X, const bf16_t *sc,
                          int scC, int scH, int scW, int scS, bf16_t *out)
{
    return conv_forward_generic(ctx, c, B, in, X, sc, scC, scH, scW, scS, out);
}

dpsgd_status conv_data_grad(dpsgd_ctx *ctx, const ConvDesc &c, int B, const bf16_t *dout, const float *X,
                            const bf16_t *scd, int scC, int scH, int scW, int scS, const bf16_t *act, bf16_t *din)
{
    return conv_data_grad_generic(ctx, c, B, dout, X, scd, scC, scH, scW, scS, act, din);
}

dpsgd_status conv_weight_grad(dpsgd_ctx *ctx, const ConvDesc &c, int B, const bf16_t *in, const bf16_t *dout, float *G)
{
    return conv_weight_grad_generic(ctx, c, B, in, dout, G);
}

}  // namespace dpsgd

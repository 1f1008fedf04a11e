// Declarations shared by the gradient translation units.
#pragma once

#include "dpsgd_internal.h"

namespace dpsgd {

// logits [n][B][C] -> dz = (softmax - onehot)/B and loss[w] (may be null); grid n, block 256.
// Labels outside [0, C) are clamped into range.  With G set, also the bias gradient of the class layer:
// G[w * ld + boff + c] = sum_b dz[w][b][c].
__global__ void softmax_xent_kernel(const float *__restrict__ z, const int *__restrict__ labels, int B, int C,
                                    float *__restrict__ dz, float *__restrict__ loss, float *__restrict__ G,
                                    long long ld, long long boff);

size_t f32_workspace_bytes(const dpsgd_ctx *ctx, const dpsgd_model_desc &m);
dpsgd_status launch_grad_f32(dpsgd_ctx *ctx, const dpsgd_model_desc &m, const float *X, const void *inputs,
                             const void *targets, float *G, float *loss);

size_t mlp_bf16_workspace_bytes(const dpsgd_ctx *ctx, const dpsgd_model_desc &m);
dpsgd_status launch_grad_mlp_bf16(dpsgd_ctx *ctx, const dpsgd_model_desc &m, const float *X, const void *inputs,
                                  const void *targets, float *G, float *loss);

// One whole iteration in place for bf16 MLPs on a ring: weight gradients of the large layers are formed inside
// the mix kernel and never written to G.
dpsgd_status launch_step_mlp_bf16(dpsgd_ctx *ctx, const dpsgd_model_desc &m, float *X, const void *inputs,
                                  const void *targets, float *G, float *loss, float *consensus);

size_t resnet_workspace_bytes(const dpsgd_ctx *ctx, const dpsgd_model_desc &m);
dpsgd_status launch_grad_resnet(dpsgd_ctx *ctx, const dpsgd_model_desc &m, const float *X, const void *inputs,
                                const void *targets, float *G, float *loss);

}  // namespace dpsgd

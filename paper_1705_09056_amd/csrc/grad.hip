// Dispatch of dpsgd_grad to the kernels of each workload model and arithmetic.
#include "grad_common.h"

namespace dpsgd {

static bool is_dense(const dpsgd_model_desc &m) { return m.kind == DPSGD_MODEL_SOFTMAX || m.kind == DPSGD_MODEL_MLP; }

size_t grad_workspace_bytes(const dpsgd_ctx *ctx, const dpsgd_model_desc &m)
{
    if (m.kind == DPSGD_MODEL_RESNET20) return resnet_workspace_bytes(ctx, m);
    if (is_dense(m) && m.compute_bf16) return mlp_bf16_workspace_bytes(ctx, m);
    return f32_workspace_bytes(ctx, m);
}

dpsgd_status launch_grad(dpsgd_ctx *ctx, const dpsgd_model_desc &m, const float *X, const void *inputs,
                         const void *targets, float *G, float *loss)
{
    if (m.kind == DPSGD_MODEL_RESNET20) return launch_grad_resnet(ctx, m, X, inputs, targets, G, loss);
    if (is_dense(m) && m.compute_bf16) return launch_grad_mlp_bf16(ctx, m, X, inputs, targets, G, loss);
    return launch_grad_f32(ctx, m, X, inputs, targets, G, loss);
}

dpsgd_status launch_step(dpsgd_ctx *ctx, const dpsgd_model_desc &m, float *X, const void *inputs, const void *targets,
                         float *G, float *loss, float *consensus)
{
    // the bf16 MLP path fuses the weight gradient of its large layers into the mix where a kernel exists for W: the
    // ring, a torus of at most 8 columns, or any W of at most 64 workers
    const bool any_w = ctx->opt_fused_slab && ctx->n <= 64 && ctx->d_rowptr;
    if (is_dense(m) && m.compute_bf16 && (ctx->ring_uniform || ctx->torus_uniform || any_w) && !ctx->opt_mix_force_csr)
        return launch_step_mlp_bf16(ctx, m, X, inputs, targets, G, loss, consensus);
    // everything else: the two calls of the boundary, back to back, in place.  X changes without the fused kernels
    // seeing it, so a bf16 weight copy they left for this X is stale from here on.
    ctx->shadow_valid = false;
    dpsgd_status st = launch_grad(ctx, m, X, inputs, targets, G, loss);
    if (st != DPSGD_OK) return st;
    return launch_mix(ctx, X, G, X, consensus, false);
}

}  // namespace dpsgd

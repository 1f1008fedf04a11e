// Internal declarations shared by the host API and the kernel translation units.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "dpsgd.h"

struct dpsgd_model_desc {
    int32_t kind = -1;
    int32_t compute_bf16 = 0;
    std::vector<int32_t> widths;
    int32_t batch = 0;
    int32_t input_is_bf16 = 0;
    bool operator==(const dpsgd_model_desc &o) const
    {
        return kind == o.kind && compute_bf16 == o.compute_bf16 && widths == o.widths && batch == o.batch &&
               input_is_bf16 == o.input_is_bf16;
    }
};

struct dpsgd_ctx {
    int32_t n = 0;
    int64_t d = 0, ld = 0;
    float gamma = 0.f;
    hipStream_t stream = nullptr;

    // W, host and device copies (CSR, ascending columns)
    int32_t topo_kind = 0, dim0 = 0, dim1 = 0;
    std::vector<int32_t> rowptr, colidx;
    std::vector<float> vals;
    int32_t *d_rowptr = nullptr, *d_colidx = nullptr;
    float *d_vals = nullptr;
    bool ring_uniform = false;   // Theorem 3's ring with n >= 3: three equal weights per row
    float ring_w = 0.f;
    bool torus_uniform = false;  // 2-D torus with both dimensions >= 3: five equal weights per row
    float torus_w = 0.f;

    // per-workgroup partial sums of the consensus distance
    double *d_partials = nullptr;
    int64_t partials_cap = 0;

    // launch-shape options (0 = auto)
    int32_t opt_mix_bands = 0, opt_mix_vec = 0, opt_mix_force_csr = 0;
    int32_t opt_mix_narrow = 0;     // ring mix of a wide matrix: one float4 per lane instead of the fat-lane kernel
    int32_t opt_ring_rows = 1;      // dpsgd_step on the ring, minibatch <= 32: the [16 rows][1 KB] kernel where the layer's shape allows

    // measurement aid: HIP events around the fused wgrad+mix launches of dpsgd_step ("time_fused")
    int32_t opt_ring_chunks = 1;    // the [16 rows][1 KB] kernel at K = 4096 or 8192: waves own 512-byte pieces 32 KB apart
    int32_t opt_fused_lds = 1;      // dpsgd_step on the ring, minibatch > 32: operands of the fused kernel through LDS
    int32_t opt_time_fused = 0;
    int32_t opt_conv_block = 1;     // CNN forward: the two convolutions of a resolution-keeping residual block in one launch
    int32_t opt_fused_slab = 1;     // dpsgd_step, bf16 MLP, W without a walk kernel, n <= 64: every worker's tile in LDS (2: also for the torus)
    int32_t opt_class_bwd = 1;      // bf16 MLP: backward of a class layer of at most 16 outputs in one launch
    int32_t opt_conv_band_rows = 0; // output rows per workgroup of the MFMA convolutions: 8, 16, or 0 = chosen per convolution
    std::vector<hipEvent_t> ev;   // pairs (start, stop)
    int64_t ev_pairs = 0, ev_launches = 0;

    // "bf16_shadow": dpsgd_step's fused kernel also leaves the bf16 rounding of the new hidden-layer weights here,
    // and the next dpsgd_step on the same X reads them (2 B instead of 4 B per weight in the forward and the data
    // gradient).  Valid only from one dpsgd_step to the next on the same X and model; everything else clears it.
    int32_t opt_bf16_shadow = 0;
    void *shadow = nullptr;
    size_t shadow_bytes = 0;
    bool shadow_valid = false;
    const float *shadow_X = nullptr;
    dpsgd_model_desc shadow_model;
    std::vector<int64_t> shadow_off;   // per layer: element offset of its [n][O][K] block, or -1
    std::vector<char> shadow_strips;   // per layer: the block is in [16][256] tiles (written by the ring kernel with 1 KB rows), not 32 x 32

    // gradient workspace (activations, bf16 operand copies), owned by the context
    void *ws = nullptr;
    size_t ws_bytes = 0;
    dpsgd_model_desc ws_model;
};

namespace dpsgd {

// ---- mix.hip
// Vel != NULL: heavy-ball variant (Vel <- mu Vel + G is the step direction); not with swapped.
dpsgd_status launch_mix(dpsgd_ctx *ctx, const float *Xin, const float *G, float *Xout, float *consensus,
                        bool swapped, float *Vel = nullptr, float mu = 0.f);
dpsgd_status launch_mean(dpsgd_ctx *ctx, const float *X, float *xbar);
int64_t mix_partials_needed(const dpsgd_ctx *ctx);
dpsgd_status launch_mix_range(dpsgd_ctx *ctx, const float *Xin, const float *G, float *Xout, int64_t col0,
                              int64_t ncols, bool cons, int64_t *nparts);
dpsgd_status launch_consensus_finalize(dpsgd_ctx *ctx, int64_t count, float *consensus);

// ---- grad_*.hip : each returns the workspace it needs and runs on ctx->stream
size_t grad_workspace_bytes(const dpsgd_ctx *ctx, const dpsgd_model_desc &m);
dpsgd_status launch_grad(dpsgd_ctx *ctx, const dpsgd_model_desc &m, const float *X, const void *inputs,
                         const void *targets, float *G, float *loss);
// One whole iteration in place (X <- W X - gamma grad(X)); G is scratch.  Fuses what it can.
dpsgd_status launch_step(dpsgd_ctx *ctx, const dpsgd_model_desc &m, float *X, const void *inputs, const void *targets,
                         float *G, float *loss, float *consensus);

inline dpsgd_status hip_status(hipError_t e) { return e == hipSuccess ? DPSGD_OK : DPSGD_EDEVICE; }

}  // namespace dpsgd

#define DPSGD_HIP_TRY(expr)                                   \
    do {                                                      \
        hipError_t _e = (expr);                               \
        if (_e != hipSuccess) return DPSGD_EDEVICE;           \
    } while (0)

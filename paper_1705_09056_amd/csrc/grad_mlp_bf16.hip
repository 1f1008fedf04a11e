#include "grad_common.h"
namespace dpsgd {
size_t mlp_bf16_workspace_bytes(const dpsgd_ctx *, const dpsgd_model_desc &) { return 256; }
dpsgd_status launch_grad_mlp_bf16(dpsgd_ctx *, const dpsgd_model_desc &, const float *, const void *, const void *,
                                  float *, float *) { return DPSGD_EUNSUPPORTED; }
}

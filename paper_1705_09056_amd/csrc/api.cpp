// Host side of the C-ABI: argument and topology validation, context life cycle.
// Everything that can be rejected is rejected here, before any device call.
#include <cmath>
#include <cstring>
#include <map>
#include <new>
#include <string>

#include "dpsgd_internal.h"

namespace {

struct HostCsr {
    std::vector<int32_t> rowptr, colidx;
    std::vector<float> vals;
};

// Accumulate (column, weight) pairs of one row, merging coinciding columns, ascending order.
void push_row(HostCsr &csr, std::map<int32_t, float> &row)
{
    for (auto &kv : row) {
        csr.colidx.push_back(kv.first);
        csr.vals.push_back(kv.second);
    }
    csr.rowptr.push_back((int32_t)csr.colidx.size());
    row.clear();
}

// Section 3: W_ij in [0,1], W symmetric, every row sums to one (hence every column).
dpsgd_status validate_csr(int32_t n, const int32_t *rowptr, const int32_t *colidx, const float *vals)
{
    if (rowptr[0] != 0) return DPSGD_ETOPOLOGY;
    for (int32_t i = 0; i < n; ++i) {
        if (rowptr[i + 1] < rowptr[i]) return DPSGD_ETOPOLOGY;
        if ((int64_t)rowptr[i + 1] - rowptr[i] > n) return DPSGD_ETOPOLOGY;
    }
    for (int32_t i = 0; i < n; ++i) {
        double sum = 0.0;
        for (int32_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
            if (colidx[p] < 0 || colidx[p] >= n) return DPSGD_ETOPOLOGY;
            if (p > rowptr[i] && colidx[p] <= colidx[p - 1]) return DPSGD_ETOPOLOGY;
            if (!(vals[p] >= 0.f && vals[p] <= 1.f)) return DPSGD_ETOPOLOGY;
            sum += (double)vals[p];
        }
        if (!(std::fabs(sum - 1.0) <= 1e-6)) return DPSGD_ETOPOLOGY;
    }
    for (int32_t i = 0; i < n; ++i)
        for (int32_t p = rowptr[i]; p < rowptr[i + 1]; ++p) {
            int32_t j = colidx[p];
            // binary search for column i in row j
            int32_t lo = rowptr[j], hi = rowptr[j + 1];
            while (lo < hi) {
                int32_t mid = lo + (hi - lo) / 2;
                if (colidx[mid] < i) lo = mid + 1; else hi = mid;
            }
            if (lo >= rowptr[j + 1] || colidx[lo] != i) return DPSGD_ETOPOLOGY;
            if (std::memcmp(&vals[lo], &vals[p], sizeof(float)) != 0) return DPSGD_ETOPOLOGY;
        }
    return DPSGD_OK;
}

dpsgd_status build_host_csr(int32_t n, const dpsgd_topology *W, HostCsr &csr)
{
    if (n < 1 || !W) return DPSGD_EINVAL;
    csr.rowptr.assign(1, 0);
    csr.colidx.clear();
    csr.vals.clear();
    std::map<int32_t, float> row;
    switch (W->kind) {
    case DPSGD_TOPO_RING: {
        const float w = (float)(1.0 / 3.0);
        for (int32_t i = 0; i < n; ++i) {
            row[(i + n - 1) % n] += w;
            row[i] += w;
            row[(i + 1) % n] += w;
            push_row(csr, row);
        }
        break;
    }
    case DPSGD_TOPO_RING_CHORD: {
        if (n < 4 || (n % 2) != 0) return DPSGD_EINVAL;
        for (int32_t i = 0; i < n; ++i) {
            row[(i + n - 1) % n] += 0.25f;
            row[i] += 0.25f;
            row[(i + 1) % n] += 0.25f;
            row[(i + n / 2) % n] += 0.25f;
            push_row(csr, row);
        }
        break;
    }
    case DPSGD_TOPO_TORUS2D: {
        if (W->dim0 < 1 || W->dim1 < 1 || (int64_t)W->dim0 * W->dim1 != n) return DPSGD_EINVAL;
        const float w = (float)(1.0 / 5.0);
        const int32_t R = W->dim0, C = W->dim1;
        for (int32_t r = 0; r < R; ++r)
            for (int32_t c = 0; c < C; ++c) {
                row[r * C + c] += w;
                row[((r + 1) % R) * C + c] += w;
                row[((r + R - 1) % R) * C + c] += w;
                row[r * C + (c + 1) % C] += w;
                row[r * C + (c + C - 1) % C] += w;
                push_row(csr, row);
            }
        break;
    }
    case DPSGD_TOPO_COMPLETE: {
        if ((int64_t)n * n > (int64_t)1 << 30) return DPSGD_EINVAL;
        const float w = (float)(1.0 / (double)n);
        for (int32_t i = 0; i < n; ++i) {
            for (int32_t j = 0; j < n; ++j) row[j] = w;
            push_row(csr, row);
        }
        break;
    }
    case DPSGD_TOPO_CSR: {
        if (!W->rowptr || !W->colidx || !W->vals) return DPSGD_EINVAL;
        // structure first, so that nothing is read out of bounds
        if (W->rowptr[0] != 0) return DPSGD_ETOPOLOGY;
        for (int32_t i = 0; i < n; ++i)
            if (W->rowptr[i + 1] < W->rowptr[i] || (int64_t)W->rowptr[i + 1] - W->rowptr[i] > n)
                return DPSGD_ETOPOLOGY;
        dpsgd_status st = validate_csr(n, W->rowptr, W->colidx, W->vals);
        if (st != DPSGD_OK) return st;
        csr.rowptr.assign(W->rowptr, W->rowptr + n + 1);
        csr.colidx.assign(W->colidx, W->colidx + W->rowptr[n]);
        csr.vals.assign(W->vals, W->vals + W->rowptr[n]);
        return DPSGD_OK;
    }
    default: return DPSGD_EINVAL;
    }
    // tags are correct by construction; run the same validation as a self-check
    return validate_csr(n, csr.rowptr.data(), csr.colidx.data(), csr.vals.data());
}

dpsgd_status copy_out_csr(const std::vector<int32_t> &rowptr, const std::vector<int32_t> &colidx,
                          const std::vector<float> &vals, int32_t *rp, int32_t *ci, float *va, int64_t *nnz_inout)
{
    if (!nnz_inout) return DPSGD_EINVAL;
    const int64_t nnz = (int64_t)colidx.size();
    const int64_t cap = *nnz_inout;
    *nnz_inout = nnz;
    if (rp) std::memcpy(rp, rowptr.data(), rowptr.size() * sizeof(int32_t));
    if (ci || va) {
        if (cap < nnz) return DPSGD_EINVAL;
        if (ci) std::memcpy(ci, colidx.data(), (size_t)nnz * sizeof(int32_t));
        if (va) std::memcpy(va, vals.data(), (size_t)nnz * sizeof(float));
    }
    return DPSGD_OK;
}

bool model_ok(const dpsgd_model *m)
{
    if (!m || !m->widths || m->n_widths < 1) return false;
    for (int32_t i = 0; i < m->n_widths; ++i)
        if (m->widths[i] < 1) return false;
    switch (m->kind) {
    case DPSGD_MODEL_LSQ: return m->n_widths == 1;
    case DPSGD_MODEL_SOFTMAX: return m->n_widths == 2;
    case DPSGD_MODEL_MLP: return m->n_widths >= 2 && m->n_widths <= 16;
    case DPSGD_MODEL_RESNET20: return m->n_widths == 6 && m->widths[3] <= 1024 && m->widths[4] <= 64;
    default: return false;
    }
}

}  // namespace

extern "C" {

dpsgd_status dpsgd_topology_build(int32_t n, const dpsgd_topology *W, int32_t *rowptr_out, int32_t *colidx_out,
                                  float *vals_out, int64_t *nnz_inout)
{
    if (n < 1 || !W || !nnz_inout) return DPSGD_EINVAL;
    HostCsr csr;
    try {
        dpsgd_status st = build_host_csr(n, W, csr);
        if (st != DPSGD_OK) return st;
    } catch (const std::bad_alloc &) {
        return DPSGD_ENOMEM;
    }
    return copy_out_csr(csr.rowptr, csr.colidx, csr.vals, rowptr_out, colidx_out, vals_out, nnz_inout);
}

int64_t dpsgd_model_dim(const dpsgd_model *m)
{
    if (!model_ok(m)) return -1;
    const int32_t *w = m->widths;
    switch (m->kind) {
    case DPSGD_MODEL_LSQ: return w[0];
    case DPSGD_MODEL_SOFTMAX:
    case DPSGD_MODEL_MLP: {
        int64_t d = 0;
        for (int32_t l = 0; l + 1 < m->n_widths; ++l) d += (int64_t)w[l + 1] * w[l] + w[l + 1];
        return d;
    }
    case DPSGD_MODEL_RESNET20: {
        const int64_t cin = w[0], base = w[3], blocks = w[4], classes = w[5];
        int64_t d = base * cin * 9 + 1, cprev = base;
        for (int s = 0; s < 3; ++s) {
            const int64_t c = base << s;
            for (int64_t j = 0; j < blocks; ++j) {
                d += c * cprev * 9 + 1 + c * c * 9 + 1;
                cprev = c;
            }
        }
        return d + classes * cprev + classes;
    }
    }
    return -1;
}

int64_t dpsgd_recommended_ld(int64_t d, const dpsgd_topology *W)
{
    if (d < 1 || !W || d > ((int64_t)1 << 60)) return -1;
    if (W->kind == DPSGD_TOPO_TORUS2D) {
        int64_t ld = (d + 63) / 64 * 64;
        if (ld % 256 == 0) ld += 64;
        return ld;
    }
    return (d + 255) / 256 * 256;
}

dpsgd_status dpsgd_create(dpsgd_ctx **out, int32_t n, int64_t d, int64_t ld, const dpsgd_topology *W, float gamma,
                          void *hip_stream)
{
    if (!out) return DPSGD_EINVAL;
    *out = nullptr;
    if (n < 1 || d < 1 || !W || !std::isfinite(gamma)) return DPSGD_EINVAL;
    if (ld == 0) ld = d;
    if (ld < d) return DPSGD_EINVAL;
    if ((double)n * (double)ld > 9.0e18 / 4.0) return DPSGD_EINVAL;
    HostCsr csr;
    dpsgd_ctx *ctx = nullptr;
    try {
        dpsgd_status st = build_host_csr(n, W, csr);
        if (st != DPSGD_OK) return st;
        ctx = new dpsgd_ctx();
    } catch (const std::bad_alloc &) {
        return DPSGD_ENOMEM;
    }
    ctx->n = n;
    ctx->d = d;
    ctx->ld = ld;
    ctx->gamma = gamma;
    ctx->stream = (hipStream_t)hip_stream;
    ctx->topo_kind = W->kind;
    ctx->dim0 = W->dim0;
    ctx->dim1 = W->dim1;
    ctx->rowptr.swap(csr.rowptr);
    ctx->colidx.swap(csr.colidx);
    ctx->vals.swap(csr.vals);
    if (W->kind == DPSGD_TOPO_RING && n >= 3) {
        ctx->ring_uniform = true;
        ctx->ring_w = ctx->vals[0];
    }
    if (W->kind == DPSGD_TOPO_TORUS2D && W->dim0 >= 3 && W->dim1 >= 3) {
        ctx->torus_uniform = true;
        ctx->torus_w = ctx->vals[0];
    }

    // ---- device side
    const size_t nnz = ctx->colidx.size();
    hipError_t e = hipMalloc((void **)&ctx->d_rowptr, (size_t)(n + 1) * sizeof(int32_t));
    if (e == hipSuccess) e = hipMalloc((void **)&ctx->d_colidx, nnz * sizeof(int32_t));
    if (e == hipSuccess) e = hipMalloc((void **)&ctx->d_vals, nnz * sizeof(float));
    if (e == hipSuccess)
        e = hipMemcpy(ctx->d_rowptr, ctx->rowptr.data(), (size_t)(n + 1) * sizeof(int32_t), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(ctx->d_colidx, ctx->colidx.data(), nnz * sizeof(int32_t), hipMemcpyHostToDevice);
    if (e == hipSuccess) e = hipMemcpy(ctx->d_vals, ctx->vals.data(), nnz * sizeof(float), hipMemcpyHostToDevice);
    if (e == hipSuccess) {
        ctx->partials_cap = dpsgd::mix_partials_needed(ctx);
        e = hipMalloc((void **)&ctx->d_partials, (size_t)ctx->partials_cap * sizeof(double));
    }
    if (e != hipSuccess) {
        const dpsgd_status st = (e == hipErrorOutOfMemory) ? DPSGD_ENOMEM : DPSGD_EDEVICE;
        (void)hipGetLastError();
        if (ctx->d_rowptr) (void)hipFree(ctx->d_rowptr);
        if (ctx->d_colidx) (void)hipFree(ctx->d_colidx);
        if (ctx->d_vals) (void)hipFree(ctx->d_vals);
        if (ctx->d_partials) (void)hipFree(ctx->d_partials);
        delete ctx;
        return st;
    }
    *out = ctx;
    return DPSGD_OK;
}

dpsgd_status dpsgd_destroy(dpsgd_ctx *ctx)
{
    if (!ctx) return DPSGD_OK;
    hipError_t e = hipStreamSynchronize(ctx->stream);
    (void)hipFree(ctx->d_rowptr);
    (void)hipFree(ctx->d_colidx);
    (void)hipFree(ctx->d_vals);
    (void)hipFree(ctx->d_partials);
    if (ctx->ws) (void)hipFree(ctx->ws);
    if (ctx->shadow) (void)hipFree(ctx->shadow);
    for (hipEvent_t e2 : ctx->ev) (void)hipEventDestroy(e2);
    delete ctx;
    return dpsgd::hip_status(e);
}

dpsgd_status dpsgd_set_gamma(dpsgd_ctx *ctx, float gamma)
{
    if (!ctx || !std::isfinite(gamma)) return DPSGD_EINVAL;
    ctx->gamma = gamma;
    return DPSGD_OK;
}

dpsgd_status dpsgd_set_option(dpsgd_ctx *ctx, const char *key, int64_t value)
{
    if (!ctx || !key) return DPSGD_EINVAL;
    const std::string k(key);
    // a bf16 weight copy was written by the kernels the old options selected: none survives a change of options
    ctx->shadow_valid = false;
    if (k == "mix_bands") {
        if (value < 0 || value > 16) return DPSGD_EINVAL;
        ctx->opt_mix_bands = (int32_t)value;
    } else if (k == "mix_vec") {
        if (!(value == 0 || value == 1 || value == 2 || value == 4)) return DPSGD_EINVAL;
        ctx->opt_mix_vec = (int32_t)value;
    } else if (k == "mix_narrow") {
        ctx->opt_mix_narrow = value ? 1 : 0;
    } else if (k == "mix_force_csr") {
        ctx->opt_mix_force_csr = value ? 1 : 0;
    } else if (k == "ring_rows") {
        ctx->opt_ring_rows = value ? 1 : 0;
    } else if (k == "bf16_shadow") {
        ctx->opt_bf16_shadow = value ? 1 : 0;
        ctx->shadow_valid = false;
    } else if (k == "conv_band_rows") {
        if (!(value == 0 || value == 8 || value == 16)) return DPSGD_EINVAL;
        ctx->opt_conv_band_rows = (int32_t)value;
    } else if (k == "ring_chunks") {
        ctx->opt_ring_chunks = value ? 1 : 0;
    } else if (k == "fused_lds") {
        ctx->opt_fused_lds = value ? 1 : 0;
    } else if (k == "class_bwd") {
        ctx->opt_class_bwd = value ? 1 : 0;
    } else if (k == "fused_slab") {
        if (value < 0 || value > 2) return DPSGD_EINVAL;
        ctx->opt_fused_slab = (int32_t)value;
    } else if (k == "conv_block") {
        ctx->opt_conv_block = value ? 1 : 0;
    } else if (k == "time_fused") {
        ctx->opt_time_fused = value ? 1 : 0;
    } else {
        return DPSGD_EINVAL;
    }
    return DPSGD_OK;
}

dpsgd_status dpsgd_topology_export(const dpsgd_ctx *ctx, int32_t *rowptr_out, int32_t *colidx_out, float *vals_out,
                                   int64_t *nnz_inout)
{
    if (!ctx) return DPSGD_EINVAL;
    return copy_out_csr(ctx->rowptr, ctx->colidx, ctx->vals, rowptr_out, colidx_out, vals_out, nnz_inout);
}

static bool overlaps(const void *a, const void *b, size_t bytes)
{
    const char *pa = (const char *)a, *pb = (const char *)b;
    return pa < pb + bytes && pb < pa + bytes;
}

static dpsgd_status mix_common(dpsgd_ctx *ctx, const float *X_in, const float *G, float *X_out, float *consensus,
                               bool swapped)
{
    if (!ctx || !X_in || !G || !X_out) return DPSGD_EINVAL;
    const size_t bytes = (size_t)ctx->n * (size_t)ctx->ld * sizeof(float);
    // G must be distinct from the output; X_out is either X_in itself or a disjoint buffer
    if (overlaps(G, X_out, bytes)) return DPSGD_EINVAL;
    if (X_out != X_in && overlaps(X_in, X_out, bytes)) return DPSGD_EINVAL;
    ctx->shadow_valid = false;   // X_out may be the matrix the bf16 copy belongs to
    return dpsgd::launch_mix(ctx, X_in, G, X_out, consensus, swapped);
}

dpsgd_status dpsgd_mix_step(dpsgd_ctx *ctx, const float *X_in, const float *G, float *X_out, float *consensus)
{
    return mix_common(ctx, X_in, G, X_out, consensus, false);
}

dpsgd_status dpsgd_mix_step_swapped(dpsgd_ctx *ctx, const float *X_in, const float *G, float *X_out,
                                    float *consensus)
{
    return mix_common(ctx, X_in, G, X_out, consensus, true);
}

dpsgd_status dpsgd_mix_step_momentum(dpsgd_ctx *ctx, const float *X_in, const float *G, float *V, float mu, float *X_out,
                                     float *consensus)
{
    if (!ctx || !X_in || !G || !V || !X_out) return DPSGD_EINVAL;
    if (!(mu >= 0.f && mu < 1.f)) return DPSGD_EINVAL;
    const size_t bytes = (size_t)ctx->n * (size_t)ctx->ld * sizeof(float);
    if (overlaps(G, X_out, bytes) || overlaps(V, X_out, bytes) || overlaps(V, X_in, bytes) || overlaps(V, G, bytes))
        return DPSGD_EINVAL;
    if (X_out != X_in && overlaps(X_in, X_out, bytes)) return DPSGD_EINVAL;
    ctx->shadow_valid = false;   // X_out may be the matrix the bf16 copy belongs to
    return dpsgd::launch_mix(ctx, X_in, G, X_out, consensus, false, V, mu);
}

dpsgd_status dpsgd_mean(dpsgd_ctx *ctx, const float *X, float *xbar)
{
    if (!ctx || !X || !xbar) return DPSGD_EINVAL;
    return dpsgd::launch_mean(ctx, X, xbar);
}

static dpsgd_status grad_or_step(dpsgd_ctx *ctx, const dpsgd_model *model, const float *X, const dpsgd_batch *batch,
                                 float *G, float *loss, bool step, float *consensus);

dpsgd_status dpsgd_grad(dpsgd_ctx *ctx, const dpsgd_model *model, const float *X, const dpsgd_batch *batch, float *G,
                        float *loss)
{
    return grad_or_step(ctx, model, X, batch, G, loss, false, nullptr);
}

dpsgd_status dpsgd_step(dpsgd_ctx *ctx, const dpsgd_model *model, float *X, const dpsgd_batch *batch, float *G_scratch,
                        float *loss, float *consensus)
{
    return grad_or_step(ctx, model, X, batch, G_scratch, loss, true, consensus);
}

static dpsgd_status grad_or_step(dpsgd_ctx *ctx, const dpsgd_model *model, const float *X, const dpsgd_batch *batch,
                                 float *G, float *loss, bool step, float *consensus)
{
    if (!ctx || !model || !X || !batch || !G) return DPSGD_EINVAL;
    if (!batch->inputs || !batch->targets || batch->batch < 1 || batch->batch > (1 << 20)) return DPSGD_EINVAL;
    if (dpsgd_model_dim(model) != ctx->d) return DPSGD_EINVAL;
    if (overlaps(X, G, (size_t)ctx->n * (size_t)ctx->ld * sizeof(float))) return DPSGD_EINVAL;
    dpsgd_model_desc m;
    m.kind = model->kind;
    m.compute_bf16 = model->compute_bf16 ? 1 : 0;
    m.widths.assign(model->widths, model->widths + model->n_widths);
    m.batch = batch->batch;
    m.input_is_bf16 = batch->input_is_bf16 ? 1 : 0;
    if (m.input_is_bf16 && m.kind == DPSGD_MODEL_LSQ) return DPSGD_EUNSUPPORTED;
    if (!(m == ctx->ws_model)) {
        const size_t need = dpsgd::grad_workspace_bytes(ctx, m);
        if (need > ctx->ws_bytes) {
            DPSGD_HIP_TRY(hipStreamSynchronize(ctx->stream));
            if (ctx->ws) (void)hipFree(ctx->ws);
            ctx->ws = nullptr;
            ctx->ws_bytes = 0;
            if (hipMalloc(&ctx->ws, need) != hipSuccess) {
                (void)hipGetLastError();
                return DPSGD_ENOMEM;
            }
            ctx->ws_bytes = need;
        }
        ctx->ws_model = m;
    }
    if (step) return dpsgd::launch_step(ctx, m, const_cast<float *>(X), batch->inputs, batch->targets, G, loss, consensus);
    return dpsgd::launch_grad(ctx, m, X, batch->inputs, batch->targets, G, loss);
}

dpsgd_status dpsgd_read_timing(dpsgd_ctx *ctx, double *total_ms, int64_t *launches)
{
    if (!ctx || !total_ms || !launches) return DPSGD_EINVAL;
    DPSGD_HIP_TRY(hipStreamSynchronize(ctx->stream));
    double sum = 0.0;
    for (int64_t i = 0; i < ctx->ev_pairs; ++i) {
        float ms = 0.f;
        DPSGD_HIP_TRY(hipEventElapsedTime(&ms, ctx->ev[2 * i], ctx->ev[2 * i + 1]));
        sum += (double)ms;
    }
    *total_ms = sum;
    *launches = ctx->ev_launches;
    ctx->ev_pairs = 0;
    ctx->ev_launches = 0;
    return DPSGD_OK;
}

const char *dpsgd_strerror(dpsgd_status s)
{
    switch (s) {
    case DPSGD_OK: return "ok";
    case DPSGD_EINVAL: return "invalid argument";
    case DPSGD_ETOPOLOGY: return "weight matrix is not a valid symmetric doubly stochastic CSR";
    case DPSGD_ENOMEM: return "out of memory";
    case DPSGD_EDEVICE: return "HIP call failed";
    case DPSGD_EUNSUPPORTED: return "unsupported configuration";
    }
    return "unknown status";
}

}  // extern "C"

/*
 * dpsgd.h - C-ABI of the MI355X-native D-PSGD hot path.
 *
 * One synchronous iteration of decentralized parallel SGD (Algorithm 1) over n simulated
 * workers whose iterates are the rows of an n x d fp32 matrix X resident in one GPU's HBM:
 *
 *     G[i]      = minibatch gradient of F at X[i] on worker i's batch     (Algorithm 1 step 3, footnote [a])
 *     X_next[i] = sum_j W_ij X[j] - gamma * G[i]                          (Algorithm 1 steps 4-5;
 *                                                                          global form of Section 3)
 *     xbar      = (1/n) sum_i X[i]                                        (Algorithm 1 step 7)
 *
 * Conventions shared by every call
 *   - Rows are workers: X and G are n x d fp32, row-major with a row stride of `ld` floats
 *     (ld >= d).  This is the transpose of Section 3's X_k (columns = nodes); the two agree
 *     because W is symmetric.  Vectorised kernels are used when ld is a multiple of 4 and the
 *     base pointers are 16-byte aligned; any other ld still works (scalar path).
 *   - "device" pointers are HIP device memory owned by the caller; "host" pointers are
 *     ordinary host memory.  The library owns only the context (device copy of W and its
 *     workspace) and frees it in dpsgd_destroy.
 *   - All device work is enqueued on the hipStream_t given to dpsgd_create; no call
 *     synchronises the host with the device except dpsgd_create, dpsgd_destroy,
 *     dpsgd_read_timing, and a dpsgd_grad / dpsgd_step call that has to allocate or grow the
 *     gradient workspace (the first call for a model, or one with a larger minibatch).
 *     Device outputs (G, X_out, loss, consensus, xbar) are valid in stream order.
 *   - HIP graphs: once a dpsgd_grad / dpsgd_step call for a model and minibatch size has run, later calls for it
 *     (and every mix, mean and consensus call) only enqueue kernels: no allocation, no memset, no host wait.  A caller
 *     may record them into a HIP graph on the context's stream.  Scalars are kernel arguments: a recorded call keeps the
 *     gamma, mu and pointers it was recorded with.  The "time_fused" option records events and must be off.
 *   - Every call returns a dpsgd_status.  Arguments and the topology are validated on the
 *     host before anything touches the device.
 *   - One context must not be used from two threads at once; calls that share a context and a
 *     workspace must be ordered on its stream.
 */
#ifndef DPSGD_H
#define DPSGD_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct dpsgd_ctx dpsgd_ctx;

typedef enum {
    DPSGD_OK = 0,
    DPSGD_EINVAL = 1,       /* null pointer, size out of range, model/dimension mismatch */
    DPSGD_ETOPOLOGY = 2,    /* W violates Section 3's requirements or the CSR is malformed */
    DPSGD_ENOMEM = 3,       /* host or device allocation failed */
    DPSGD_EDEVICE = 4,      /* a HIP call failed (no device, launch error) */
    DPSGD_EUNSUPPORTED = 5  /* valid request this build has no kernel for */
} dpsgd_status;

/* ---- topology: the weight matrix W of Section 3 (symmetric, doubly stochastic, W_ij in [0,1],
 *      W_ij = 0 when i and j are not connected). */
typedef enum {
    DPSGD_TOPO_CSR = 0,      /* caller-supplied CSR (host arrays) */
    DPSGD_TOPO_RING = 1,     /* Theorem 3's matrix: W_ii = W_i,i+-1 = 1/3 (indices mod n) */
    DPSGD_TOPO_TORUS2D = 2,  /* worker i = r*dim1 + c; itself and (r+-1,c), (r,c+-1) at 1/5 */
    DPSGD_TOPO_COMPLETE = 3, /* W = (1/n) 1 1^T, the centralized special case */
    DPSGD_TOPO_RING_CHORD = 4 /* ring plus a link to the node farthest away on it, i + n/2 (the 16-machine runs
                                 of the supplement's scalability experiment); itself, i+-1 and i+n/2 at 1/4 each;
                                 n even and >= 4, else DPSGD_EINVAL */
} dpsgd_topo_kind;

typedef struct {
    int32_t kind;            /* dpsgd_topo_kind */
    int32_t dim0, dim1;      /* TORUS2D only: dim0*dim1 == n */
    const int32_t *rowptr;   /* CSR only, host, n+1 entries, rowptr[0] == 0, non-decreasing */
    const int32_t *colidx;   /* CSR only, host, nnz entries, strictly ascending inside a row */
    const float *vals;       /* CSR only, host, nnz entries in [0,1] */
} dpsgd_topology;

/* Builds (tags) or validates (CSR) W on the host and writes its CSR form; touches no device.
 * Tags with coinciding neighbours (ring with n < 3, torus with a dimension < 3) accumulate the
 * duplicate weights, so the result always satisfies Section 3.  Tag values are (float)(1.0/3.0),
 * (float)(1.0/5.0), (float)(1.0/n), 0.25f.
 * Validation (DPSGD_ETOPOLOGY on failure): rowptr monotone from 0; column indices in [0,n),
 * strictly ascending per row; values in [0,1]; |row sum - 1| <= 1e-6; W_ij == W_ji bitwise.
 * rowptr_out (n+1), colidx_out, vals_out (capacity *nnz_inout entries) are host arrays; any of the
 * three may be NULL to query only the size.  On return *nnz_inout is the number of non-zeros;
 * DPSGD_EINVAL if the capacity passed in was too small. */
dpsgd_status dpsgd_topology_build(int32_t n, const dpsgd_topology *W, int32_t *rowptr_out,
                                  int32_t *colidx_out, float *vals_out, int64_t *nnz_inout);

/* ---- workload model: fixes F of Section 3's problem statement (F_i = F for all i), the length d
 *      of a worker's parameter vector and the order of the parameters inside it.
 *
 * Flattening order: layer by layer, weight (out x in [x 3 x 3], row-major) then its bias.
 *   LSQ       widths = {features}.  F = (1/(2B)) ||A x - y||^2 over the minibatch rows.
 *   SOFTMAX   widths = {features, classes}.  Linear layer + softmax cross-entropy (natural log,
 *             mean over the minibatch).
 *   MLP       widths = {features, hidden..., classes}.  ReLU hidden layers (ReLU'(0) = 0),
 *             softmax cross-entropy.
 *   RESNET20  widths = {in_ch, height, width, base_ch, blocks_per_stage, classes}.  3x3 stem conv,
 *             3 stages of basic blocks with base, 2*base, 4*base channels (first conv of stages
 *             2 and 3 has stride 2), no batch-norm, ONE scalar bias per conv added before the
 *             ReLU, parameter-free shortcuts (identity; on a stage change every second pixel and
 *             zero-padded channels), global average pool, fully connected layer with bias,
 *             softmax cross-entropy.  Inputs are [B][in_ch][height][width].
 * The minibatch gradient is the MEAN of the B sample gradients (footnote [a]). */
typedef enum { DPSGD_MODEL_LSQ = 0, DPSGD_MODEL_SOFTMAX = 1, DPSGD_MODEL_MLP = 2, DPSGD_MODEL_RESNET20 = 3 } dpsgd_model_kind;

typedef struct {
    int32_t kind;            /* dpsgd_model_kind */
    int32_t n_widths;        /* entries in widths */
    const int32_t *widths;   /* host */
    int32_t compute_bf16;    /* 0: fp32 arithmetic.  1: bf16 MFMA operands (weights and activations
                                rounded to bf16, ties to even), fp32 accumulation, fp32 G */
} dpsgd_model;

/* Length d the model implies, or -1 if the description is invalid.  Host only. */
int64_t dpsgd_model_dim(const dpsgd_model *model);

/* A row stride ld >= d (in floats) for the n x d replica matrix that the kernels stream well; dpsgd_create accepts
 * any ld >= d, this is a recommendation for the caller's allocation.  -1 if d < 1 or W is NULL.  Host only.
 * Ring and every other topology: d rounded up to a multiple of 256 floats, so that the 1 KB row pieces the ring
 * kernels move are 1 KB-aligned for every worker.  2-D torus: a multiple of 64 floats that is not a multiple of
 * 256, so that the tiles of a grid row's workers, which the fused torus kernel touches together, start 256 bytes
 * apart inside their 1 KB granules instead of on top of each other.  (A layout decision for this GPU's memory; the
 * paper, whose replicas live on different machines, has no counterpart.) */
int64_t dpsgd_recommended_ld(int64_t d, const dpsgd_topology *W);

/* One minibatch per worker (Algorithm 1 step 2 has already happened in the caller). */
typedef struct {
    const void *inputs;      /* device, [n][batch][features]; fp32, or bf16 if input_is_bf16 */
    const void *targets;     /* device, [n][batch]; fp32 y for LSQ, int32 class labels otherwise */
    int32_t batch;           /* B >= 1, samples per worker */
    int32_t input_is_bf16;   /* 0 or 1 */
} dpsgd_batch;

/* ---- context */

/* Creates a context for n workers with d parameters each (row stride ld floats, ld >= d; pass 0
 * for ld == d), the weight matrix W (copied; the caller's arrays may be freed afterwards), the
 * step length gamma (finite) and a hipStream_t (NULL = the default stream).
 * Uses the current HIP device.  DPSGD_EINVAL / DPSGD_ETOPOLOGY are decided before any device call. */
dpsgd_status dpsgd_create(dpsgd_ctx **out, int32_t n, int64_t d, int64_t ld, const dpsgd_topology *W,
                          float gamma, void *hip_stream);

/* Waits for the context's stream, then frees the context and everything it owns.  NULL is accepted. */
dpsgd_status dpsgd_destroy(dpsgd_ctx *ctx);

/* Changes the step length gamma of Algorithm 1 step 5 for every later call that applies the update: dpsgd_mix_step,
 * dpsgd_mix_step_swapped, dpsgd_mix_step_momentum and dpsgd_step (learning-rate schedules, Section 5.3).  Calls already
 * enqueued, or recorded into a HIP graph, keep the value they were issued with. */
dpsgd_status dpsgd_set_gamma(dpsgd_ctx *ctx, float gamma);

/* Launch-shape knobs for measurements and comparisons (no passage of the paper: they select between kernels that
 * compute the same iteration); unknown keys give DPSGD_EINVAL.  Defaults are chosen from (n, d) and are what the
 * benchmark runs.  Changing any option drops a bf16 weight copy ("bf16_shadow").  Keys: "mix_bands" (row bands per workgroup of the ring kernel, 0 = auto),
 * "mix_vec" (floats per lane: 0 = auto, 1, 2 or 4), "mix_force_csr" (1: run the generic CSR
 * kernel even for ring / torus tags), "mix_narrow" (1: the ring kernel with one float4 per lane also for wide
 * matrices, where the default gives a lane eight), "ring_rows" (default 1: dpsgd_step on the ring, bf16 MLP, minibatch of at most 32 rows: layers whose input width is
 * a multiple of 256 use the kernel whose workgroups own [16 rows][1 KB] of the weight matrix, each wave whole 1 KB
 * row pieces; 0: the kernel with 32 x 32 tiles per wave for every layer.  The two add up the minibatch in a different
 * order inside the matrix instructions, so their results agree to fp32 rounding, not bit for bit),
 * "bf16_shadow" (1: dpsgd_step on the ring also leaves the bf16 rounding of the new hidden-layer weights of a bf16 MLP
 * in a buffer of the context, and the next dpsgd_step on the same X and model reads them instead of the fp32
 * weights in its forward and data-gradient kernels: the same values, half the bytes.  The caller promises that
 * between two dpsgd_step calls nobody else writes X; every dpsgd_mix_step* call, a change of this option, another
 * X or model, and calls recorded under stream capture drop the copy.  Costs 2 bytes per hidden-layer weight and
 * worker of device memory.  The iterates are bit for bit those of the same "ring_rows" setting without the copy),
 * "ring_chunks" (default 1: in that [16 rows][1 KB] kernel, for layers whose number of inputs is a multiple of 1024, a
 * wave owns pieces of rows a multiple of 32 KB apart instead of four consecutive rows; 0: consecutive rows.  Same bits),
 * "fused_lds" (default 1: dpsgd_step on the ring, bf16 MLP, minibatch of more than 32 rows: the operands of the fused
 * weight-gradient + mix kernel travel from L2 into LDS asynchronously, one worker ahead; 0: they are fetched into
 * registers two steps at a time.  Same bits),
 * "class_bwd" (default 1: bf16 MLP whose last layer has at most 16 outputs, minibatch of at most 256 rows: the weight,
 * bias and data gradient of that layer and the bias gradient of the layer below come from one launch in which a thread
 * walks the samples of one column of the activations; 0: the tiled kernels of the other layers, three launches.  The
 * two add up the same products in a different order: results agree to fp32 rounding of the sums),
 * "fused_slab" (default 1: dpsgd_step, bf16 MLP, a W of at most 64 workers that is neither Theorem 3's ring nor a torus
 * of 3 to 16 columns: the weight gradient of the large layers is formed inside a mix kernel that holds every worker's tile
 * in LDS; 0: such a W runs dpsgd_grad and dpsgd_mix_step back to back; 2: that kernel also takes the tori the torus
 * kernel would take.  Results agree to fp32 rounding),
 * "conv_block" (default 1: CNN forward, residual blocks that keep the resolution (16 channels, 32 on 16 x 16 or 64 on 8 x 8
 * pixels): both convolutions of
 * the block in one launch, the activation between them kept in LDS for the second one; 0: two launches.  Same bits),
 * "conv_band_rows" (output rows of an image per workgroup of the CNN's 3 x 3 convolution kernels: 8, 16, or 0 = chosen
 * per convolution, the default; every setting gives the same bits),
 * "time_fused" (see dpsgd_read_timing). */
dpsgd_status dpsgd_set_option(dpsgd_ctx *ctx, const char *key, int64_t value);

/* CSR of the context's W (host arrays as in dpsgd_topology_build). */
dpsgd_status dpsgd_topology_export(const dpsgd_ctx *ctx, int32_t *rowptr_out, int32_t *colidx_out,
                                   float *vals_out, int64_t *nnz_inout);

/* ---- the iteration */

/* Algorithm 1 step 3 for all workers: G[i] = (1/B) sum_b grad_x F(X[i]; sample b of worker i),
 * evaluated at the worker's own iterate X[i].
 *   X      device, n x d (stride ld), read only
 *   G      device, n x d (stride ld), overwritten (padding columns d..ld-1 are left untouched)
 *   loss   device, n floats: each worker's minibatch loss; may be NULL
 * dpsgd_model_dim(model) must equal the context's d (else DPSGD_EINVAL).  Activations live in a
 * workspace owned by the context, (re)allocated when the model or batch size changes. */
dpsgd_status dpsgd_grad(dpsgd_ctx *ctx, const dpsgd_model *model, const float *X, const dpsgd_batch *batch,
                        float *G, float *loss);

/* Algorithm 1 steps 4 and 5 fused: X_out[i] = sum_j W_ij X_in[j] - gamma * G[i].
 *   X_in, G  device, n x d (stride ld), read only
 *   X_out    device, n x d (stride ld); may be the same buffer as X_in (in place): every workgroup
 *            owns whole columns and reads all of them before it writes
 *   consensus device, 1 float, may be NULL: M = (1/n) sum_i || xbar - X_out[i] ||^2 of the OUTPUT
 *            iterates (the consensus distance of Theorem 4 / eq. 13), reduced in a fixed order.
 * Each X and G element is read once from HBM and each X_out element written once.
 * Limits.  Theorem 3's ring (DPSGD_TOPO_RING, n >= 3) walks the rows with three of them in registers: any n, in place or
 * not.  Every other W stages the n rows of a column slab in 64 KB of LDS, which holds n <= 256 workers (n <= 64 with 16-byte
 * accesses, n <= 128 with 8-byte ones; beyond that narrower accesses are used).  For n > 256 such a W is mixed by a gather
 * kernel that cannot work in place: X_out == X_in then returns DPSGD_EUNSUPPORTED and nothing is launched; out of place
 * it takes up to 65535 workers (more: DPSGD_EUNSUPPORTED). */
dpsgd_status dpsgd_mix_step(dpsgd_ctx *ctx, const float *X_in, const float *G, float *X_out, float *consensus);

/* Footnote [c]'s admissible reordering: update first, then average,
 *   X_out[i] = sum_j W_ij (X_in[j] - gamma G[j]).  Same arguments as dpsgd_mix_step. */
dpsgd_status dpsgd_mix_step_swapped(dpsgd_ctx *ctx, const float *X_in, const float *G, float *X_out,
                                    float *consensus);

/* Heavy-ball variant of steps 4 and 5.  Section 5.3 runs D-PSGD with learning rate 0.1 and momentum 0.9 without
 * saying where the momentum enters; the reading taken is the plain momentum update of the local gradient, the
 * averaging untouched:
 *   V[i]     <- mu * V[i] + G[i]                      (in place)
 *   X_out[i]  = sum_j W_ij X_in[j] - gamma * V[i]
 *   V        device, n x d (stride ld), read and written once; must not overlap X_in, X_out or G
 *   mu       in [0, 1); mu = 0 gives dpsgd_mix_step (and V = G)
 * Other arguments, in-place rule and consensus as in dpsgd_mix_step.  20 bytes per (worker, parameter).
 * DPSGD_EINVAL for a mu outside [0, 1) or overlapping buffers. */
dpsgd_status dpsgd_mix_step_momentum(dpsgd_ctx *ctx, const float *X_in, const float *G, float *V, float mu,
                                     float *X_out, float *consensus);

/* One whole iteration of Algorithm 1 in place: X <- W X - gamma * grad(X), i.e. the result of dpsgd_grad(X -> G)
 * followed by dpsgd_mix_step(X, G -> X), up to the order of floating-point sums.  Footnote [b] observes that steps 3
 * and 4 are independent; here they share one pass over X wherever a kernel exists for it.
 * Fused (the weight gradient of a layer is formed inside the mix kernel and never written to memory): model MLP or
 * SOFTMAX with compute_bf16 = 1, on DPSGD_TOPO_RING with n >= 3 (a walk around the ring with three rows in
 * registers), on DPSGD_TOPO_TORUS2D with dim0 >= 3 and 3 <= dim1 <= 16 (a walk down the grid columns), and on every
 * other W of at most 64 workers - DPSGD_TOPO_RING_CHORD, DPSGD_TOPO_COMPLETE, DPSGD_TOPO_CSR, the remaining rings and
 * tori - through a kernel that holds every worker's tile in LDS; for every layer with at least 2^20 weights whose
 * outputs are a multiple of 32 and whose inputs are a multiple of 128 (ring) or of 32 (any other W; also 8-byte
 * aligned rows); the remaining parameters of such a model (small layers, biases) take the ordinary gradient kernels
 * and the mix kernels on their column ranges inside the same call.
 * Not fused - the call runs dpsgd_grad and an in-place dpsgd_mix_step back to back, same results: a W other than
 * those two walks with more than 64 workers, fp32 arithmetic (compute_bf16 = 0), LSQ and RESNET20 models, and the
 * "mix_force_csr" option.
 *   X          device, n x d (stride ld), overwritten by the next iterate
 *   G_scratch  device, n x d (stride ld), must not overlap X; on return it holds the gradient only of those
 *              parameters whose update was not fused (contents otherwise unspecified)
 *   loss, consensus  as in dpsgd_grad and dpsgd_mix_step; either may be NULL
 * The update is in place, so the in-place limit of dpsgd_mix_step applies: a W other than Theorem 3's ring with n > 256
 * workers returns DPSGD_EUNSUPPORTED (after the gradient has been written to G_scratch; X is untouched). */
dpsgd_status dpsgd_step(dpsgd_ctx *ctx, const dpsgd_model *model, float *X, const dpsgd_batch *batch, float *G_scratch,
                        float *loss, float *consensus);

/* dpsgd_mix_step for callers that cannot allocate device memory: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  It needs no context and calls no hipMalloc / hipFree (nor any other allocating
 * routine): what dpsgd_mix_step keeps in buffers of its context - the per-workgroup partial sums of the consensus
 * distance, the device CSR of a torus - lives in one fixed array of 4 MiB + 64 KiB of device memory inside the library,
 * which every GPU the library runs on holds from the first use until the process ends.
 *   n, d, ld, gamma, X_in, G, X_out, consensus   as in dpsgd_create / dpsgd_mix_step (ld == 0 means ld == d); X_out may
 *            be X_in; the caller still owns and passes every input and output
 *   W        a tag only: DPSGD_TOPO_RING with n >= 3, or DPSGD_TOPO_TORUS2D with both dimensions >= 3 and n <= 256
 *   hip_stream  the hipStream_t the kernels are enqueued on (NULL = the default stream)
 * Same kernels, same results, bit for bit, as dpsgd_mix_step on a context created with the same arguments.
 * Limits: d <= 33 554 432 (2^25) parameters per worker; anything larger, any other W (CSR, complete graph, ring with
 * a far link, rings and tori with coinciding neighbours) and a torus with n > 256 return DPSGD_EUNSUPPORTED before
 * anything is launched; argument errors return DPSGD_EINVAL as in dpsgd_mix_step.
 * All calls on one GPU share that GPU's array: the kernels overwrite every part of it they later read (nothing has to
 * start at zero), so consecutive calls on one stream are independent of each other, but two calls that overlap in
 * time on the same GPU (different streams or threads) race on it.  The first call on a device looks up the array's
 * address and must not be made under stream capture; later ones only enqueue kernels. */
dpsgd_status dpsgd_mix_step_static(int32_t n, int64_t d, int64_t ld, const dpsgd_topology *W, float gamma,
                                   const float *X_in, const float *G, float *X_out, float *consensus, void *hip_stream);

/* Algorithm 1 step 7: xbar = (1/n) sum_i X[i].  X device n x d (stride ld); xbar device, d floats. */
dpsgd_status dpsgd_mean(dpsgd_ctx *ctx, const float *X, float *xbar);

/* Measurement aid.  With dpsgd_set_option(ctx, "time_fused", 1), dpsgd_step brackets its fused weight-gradient +
 * mix kernel launches with HIP events on the context's stream.  This call waits for the stream and returns the summed
 * duration (ms) and the number of bracketed kernel launches since the previous call (at most 8192 steps are kept). */
dpsgd_status dpsgd_read_timing(dpsgd_ctx *ctx, double *total_ms, int64_t *launches);

/* Static, never NULL. */
const char *dpsgd_strerror(dpsgd_status status);

#ifdef __cplusplus
}
#endif
#endif /* DPSGD_H */

/*
 * CPU oracle for one synchronous D-PSGD iteration (TEST INFRASTRUCTURE).
 *
 * Plain, slow, fp64 loops written from the paper; it shares no code with the
 * HIP library and only tests, the smoke check and the benchmark's CPU-baseline
 * leg may call it.  The product path never does.
 *
 * What is computed (paper passages each function follows):
 *   - weight matrix W of a ring (Theorem 3's matrix), of the ring with a link to
 *     the farthest node (supplement, scalability experiment), of a 2-D torus and
 *     of the complete graph; checks of Section 3's requirements (entries in
 *     [0,1], symmetric, rows sum to one);
 *   - Algorithm 1 steps 4-5 in the global form of Section 3,
 *       X_{k+1} = W X_k - gamma * dF(X_k; xi_k)       (rows = workers; W = W^T);
 *     its reordering of footnote [c], and the heavy-ball variant (Section 5.3
 *     runs with momentum 0.9);
 *   - Algorithm 1 step 7, the node average;
 *   - the consensus distance M_k of the proof of Theorem 1 (eq. 10 and 13),
 *       M = (1/n) sum_i || mean_j x_j - x_i ||^2;
 *   - Algorithm 1 step 3 with footnote [a]: the mean over a minibatch of the
 *     sample gradients of F at the worker's own iterate, for four workload
 *     models (least squares, softmax regression, ReLU MLP, a BN-free
 *     ResNet-20-style CNN).
 *
 * Pins (tests marked "not gpu"): circulant spectra of the ring/torus W, dense
 * W^k powers, the node-average recursion and the unrolled recursion from the
 * proof of Theorem 1, the complete-graph reduction to minibatch SGD, the
 * closed-form affine map on a quadratic objective, the two-term recurrence and
 * the 2x2 mode recurrence of the heavy-ball variant, central finite differences
 * and PyTorch-CPU autograd (fp64) on small instances of every model.
 * Values from the paper's experiments: parity unpinned (the paper prints no
 * iterate, loss or gradient of a reproducible instance).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORC_LSQ = 0, ORC_SOFTMAX = 1, ORC_MLP = 2, ORC_RESNET20 = 3 };

/* Nearest bf16 (8-bit significand, ties to even) of v, returned as a double.  Used only by the
 * "bf16 operands" mode of the gradients: the workloads that prescribe bf16 compute round every
 * operand of a contraction (weights, stored activations, back-propagated deltas) to bf16 and
 * accumulate wider; the oracle then accumulates in fp64.  ReLU decisions are thereby taken on the
 * same rounded values as in a bf16 kernel. */
static double rbf(double v)
{
    float f = (float)v;
    uint32_t u;
    memcpy(&u, &f, 4);
    if ((u & 0x7f800000u) == 0x7f800000u) return (double)f; /* inf / nan unchanged */
    u += 0x7fffu + ((u >> 16) & 1u);
    u &= 0xffff0000u;
    memcpy(&f, &u, 4);
    return (double)f;
}
static double *rounded_copy(const double *src, size_t n)
{
    double *r = (double *)malloc(sizeof(double) * n);
    for (size_t i = 0; i < n; ++i) r[i] = rbf(src[i]);
    return r;
}

/* ------------------------------------------------------------------ topology */

/* Emit row i of a dense scratch row as CSR (ascending columns, zeros dropped). */
static int64_t emit_row(const double *row, int n, int64_t nnz, int32_t *col, double *val)
{
    for (int j = 0; j < n; ++j)
        if (row[j] != 0.0) {
            if (col) { col[nnz] = j; val[nnz] = row[j]; }
            ++nnz;
        }
    return nnz;
}

/* Ring of Theorem 3: every node averages itself and its two ring neighbours with
 * weight 1/3.  For n < 3 coinciding neighbours accumulate.  Returns nnz. */
int64_t orc_topology_ring(int32_t n, int32_t *rowptr, int32_t *col, double *val)
{
    double *row = (double *)malloc(sizeof(double) * (size_t)n);
    int64_t nnz = 0;
    if (rowptr) rowptr[0] = 0;
    for (int i = 0; i < n; ++i) {
        memset(row, 0, sizeof(double) * (size_t)n);
        row[i] += 1.0 / 3.0;
        row[(i + 1) % n] += 1.0 / 3.0;
        row[(i + n - 1) % n] += 1.0 / 3.0;
        nnz = emit_row(row, n, nnz, col, val);
        if (rowptr) rowptr[i + 1] = (int32_t)nnz;
    }
    free(row);
    return nnz;
}

/* Ring with one extra link per node to the node farthest away on the ring, i + n/2
 * (the 16-machine runs of the supplement's scalability experiment).  n must be even and
 * at least 4.  Our reading of the weights: itself, the two ring neighbours and the far
 * node at 1/4 each, which is symmetric and doubly stochastic.  Returns nnz, or -1. */
int64_t orc_topology_ring_chord(int32_t n, int32_t *rowptr, int32_t *col, double *val)
{
    if (n < 4 || (n % 2) != 0) return -1;
    double *row = (double *)malloc(sizeof(double) * (size_t)n);
    int64_t nnz = 0;
    if (rowptr) rowptr[0] = 0;
    for (int i = 0; i < n; ++i) {
        memset(row, 0, sizeof(double) * (size_t)n);
        row[i] += 0.25;
        row[(i + 1) % n] += 0.25;
        row[(i + n - 1) % n] += 0.25;
        row[(i + n / 2) % n] += 0.25;
        nnz = emit_row(row, n, nnz, col, val);
        if (rowptr) rowptr[i + 1] = (int32_t)nnz;
    }
    free(row);
    return nnz;
}

/* 2-D torus: worker i = r*dim1 + c averages itself and (r+-1, c), (r, c+-1) (indices
 * modulo the grid) with weight 1/5.  Satisfies Section 3's requirements on W. */
int64_t orc_topology_torus(int32_t dim0, int32_t dim1, int32_t *rowptr, int32_t *col, double *val)
{
    int n = dim0 * dim1;
    double *row = (double *)malloc(sizeof(double) * (size_t)n);
    int64_t nnz = 0;
    if (rowptr) rowptr[0] = 0;
    for (int r = 0; r < dim0; ++r)
        for (int c = 0; c < dim1; ++c) {
            int i = r * dim1 + c;
            memset(row, 0, sizeof(double) * (size_t)n);
            row[i] += 0.2;
            row[((r + 1) % dim0) * dim1 + c] += 0.2;
            row[((r + dim0 - 1) % dim0) * dim1 + c] += 0.2;
            row[r * dim1 + (c + 1) % dim1] += 0.2;
            row[r * dim1 + (c + dim1 - 1) % dim1] += 0.2;
            nnz = emit_row(row, n, nnz, col, val);
            if (rowptr) rowptr[i + 1] = (int32_t)nnz;
        }
    free(row);
    return nnz;
}

/* Complete graph, W = (1/n) 1 1^T: the centralized special case. */
int64_t orc_topology_complete(int32_t n, int32_t *rowptr, int32_t *col, double *val)
{
    int64_t nnz = 0;
    if (rowptr) rowptr[0] = 0;
    for (int i = 0; i < n; ++i) {
        for (int j = 0; j < n; ++j) {
            if (col) { col[nnz] = j; val[nnz] = 1.0 / (double)n; }
            ++nnz;
        }
        if (rowptr) rowptr[i + 1] = (int32_t)nnz;
    }
    return nnz;
}

/* CSR -> dense n x n (row-major). */
void orc_topology_dense(int32_t n, const int32_t *rowptr, const int32_t *col, const double *val, double *Wd)
{
    memset(Wd, 0, sizeof(double) * (size_t)n * (size_t)n);
    for (int i = 0; i < n; ++i)
        for (int p = rowptr[i]; p < rowptr[i + 1]; ++p) Wd[(size_t)i * n + col[p]] += val[p];
}

/* Section 3's requirements on W.  Returns 0 if they hold, else a code:
 * 1 malformed CSR, 2 entry outside [0,1], 3 a row sum off by more than tol,
 * 4 not symmetric (exact comparison). */
int32_t orc_topology_check(int32_t n, const int32_t *rowptr, const int32_t *col, const double *val, double tol)
{
    if (rowptr[0] != 0) return 1;
    for (int i = 0; i < n; ++i) {
        if (rowptr[i + 1] < rowptr[i]) return 1;
        double s = 0.0;
        for (int p = rowptr[i]; p < rowptr[i + 1]; ++p) {
            if (col[p] < 0 || col[p] >= n) return 1;
            if (p > rowptr[i] && col[p] <= col[p - 1]) return 1;
            if (!(val[p] >= 0.0 && val[p] <= 1.0)) return 2;
            s += val[p];
        }
        if (fabs(s - 1.0) > tol) return 3;
    }
    for (int i = 0; i < n; ++i)
        for (int p = rowptr[i]; p < rowptr[i + 1]; ++p) {
            int j = col[p], found = 0;
            for (int q = rowptr[j]; q < rowptr[j + 1]; ++q)
                if (col[q] == i) { found = (val[q] == val[p]); break; }
            if (!found) return 4;
        }
    return 0;
}

/* --------------------------------------------------------- mix, mean, consensus */

/* Algorithm 1 steps 4 and 5 for all workers:
 *   Xn[i] = sum_j W_ij X[j] - gamma G[i]. */
void orc_mix_step(int32_t n, int64_t d, const int32_t *rowptr, const int32_t *col, const double *val,
                  const double *X, const double *G, double gamma, double *Xn)
{
    for (int i = 0; i < n; ++i)
        for (int64_t c = 0; c < d; ++c) {
            double half = 0.0; /* x_{k+1/2,i} */
            for (int p = rowptr[i]; p < rowptr[i + 1]; ++p) half += val[p] * X[(size_t)col[p] * d + c];
            Xn[(size_t)i * d + c] = half - gamma * G[(size_t)i * d + c];
        }
}

/* Footnote [c] variant: update first, then average: Xn = W (X - gamma G). */
void orc_mix_step_swapped(int32_t n, int64_t d, const int32_t *rowptr, const int32_t *col, const double *val,
                          const double *X, const double *G, double gamma, double *Xn)
{
    for (int i = 0; i < n; ++i)
        for (int64_t c = 0; c < d; ++c) {
            double acc = 0.0;
            for (int p = rowptr[i]; p < rowptr[i + 1]; ++p) {
                size_t j = (size_t)col[p];
                acc += val[p] * (X[j * d + c] - gamma * G[j * d + c]);
            }
            Xn[(size_t)i * d + c] = acc;
        }
}

/* Momentum variant of steps 4-5 (Section 5.3 runs D-PSGD with learning rate 0.1 and
 * momentum 0.9 and does not say where the momentum enters; the reading taken is the
 * plain heavy-ball update of the local gradient, averaging untouched):
 *   Vn[i] = mu V[i] + G[i],   Xn[i] = sum_j W_ij X[j] - gamma Vn[i]. */
void orc_mix_step_momentum(int32_t n, int64_t d, const int32_t *rowptr, const int32_t *col, const double *val,
                           const double *X, const double *G, const double *V, double gamma, double mu, double *Xn,
                           double *Vn)
{
    for (int i = 0; i < n; ++i)
        for (int64_t c = 0; c < d; ++c) {
            size_t e = (size_t)i * d + c;
            double half = 0.0;
            for (int p = rowptr[i]; p < rowptr[i + 1]; ++p) half += val[p] * X[(size_t)col[p] * d + c];
            Vn[e] = mu * V[e] + G[e];
            Xn[e] = half - gamma * Vn[e];
        }
}

/* Algorithm 1 step 7: (1/n) sum_i x_i. */
void orc_mean(int32_t n, int64_t d, const double *X, double *xbar)
{
    for (int64_t c = 0; c < d; ++c) {
        double s = 0.0;
        for (int i = 0; i < n; ++i) s += X[(size_t)i * d + c];
        xbar[c] = s / (double)n;
    }
}

/* M = (1/n) sum_i || xbar - x_i ||^2 (eq. 10 and 13 of the proof of Theorem 1). */
double orc_consensus(int32_t n, int64_t d, const double *X)
{
    double total = 0.0;
    for (int64_t c = 0; c < d; ++c) {
        double s = 0.0;
        for (int i = 0; i < n; ++i) s += X[(size_t)i * d + c];
        double m = s / (double)n;
        for (int i = 0; i < n; ++i) {
            double e = m - X[(size_t)i * d + c];
            total += e * e;
        }
    }
    return total / (double)n;
}

/* ------------------------------------------------------------------ model sizes */

static int64_t resnet_dim(const int32_t *w)
{
    int64_t cin = w[0], base = w[3], blocks = w[4], classes = w[5];
    int64_t d = base * cin * 9 + 1, cprev = base;
    for (int s = 0; s < 3; ++s) {
        int64_t c = base << s;
        for (int j = 0; j < blocks; ++j) {
            d += c * cprev * 9 + 1 + c * c * 9 + 1;
            cprev = c;
        }
    }
    return d + classes * cprev + classes;
}

/* Length of one worker's flattened parameter vector.
 * LSQ: widths = {features}.  SOFTMAX / MLP: widths = {in, hidden..., classes}, n_layers =
 * number of weight matrices.  RESNET20: widths = {in_ch, H, W, base_ch, blocks_per_stage, classes}. */
int64_t orc_model_dim(int32_t kind, int32_t n_layers, const int32_t *widths)
{
    if (kind == ORC_LSQ) return widths[0];
    if (kind == ORC_SOFTMAX || kind == ORC_MLP) {
        int64_t d = 0;
        for (int l = 0; l < n_layers; ++l) d += (int64_t)widths[l + 1] * widths[l] + widths[l + 1];
        return d;
    }
    if (kind == ORC_RESNET20) return resnet_dim(widths);
    return -1;
}

/* ------------------------------------------------- softmax cross-entropy (mean) */

/* logits [B][C] -> mean over the batch of -log softmax(logits)[label]; if dz != NULL also
 * d(loss)/d(logits) = (softmax - onehot)/B. */
static double softmax_xent(const double *z, const int32_t *label, int B, int C, double *dz)
{
    double loss = 0.0;
    for (int b = 0; b < B; ++b) {
        const double *zb = z + (size_t)b * C;
        double mx = zb[0];
        for (int c = 1; c < C; ++c) if (zb[c] > mx) mx = zb[c];
        double se = 0.0;
        for (int c = 0; c < C; ++c) se += exp(zb[c] - mx);
        double lse = mx + log(se);
        loss += lse - zb[label[b]];
        if (dz)
            for (int c = 0; c < C; ++c)
                dz[(size_t)b * C + c] = (exp(zb[c] - lse) - (c == label[b] ? 1.0 : 0.0)) / (double)B;
    }
    return loss / (double)B;
}

/* ------------------------------------------------------------------ least squares */

/* F(x; A, y) = (1/(2B)) ||A x - y||^2,  grad = A^T (A x - y) / B. */
static double lsq_loss_grad(int F, const double *x, const double *A, const double *y, int B, double *g)
{
    double loss = 0.0;
    if (g) for (int c = 0; c < F; ++c) g[c] = 0.0;
    for (int b = 0; b < B; ++b) {
        double r = -y[b];
        for (int c = 0; c < F; ++c) r += A[(size_t)b * F + c] * x[c];
        loss += r * r;
        if (g) for (int c = 0; c < F; ++c) g[c] += A[(size_t)b * F + c] * r / (double)B;
    }
    return loss / (2.0 * (double)B);
}

/* ----------------------------------------------------------- MLP / softmax regression */

/* Fully connected layers z_l = W_l a_l + b_l, a_{l+1} = ReLU(z_l) for hidden layers
 * (ReLU'(0) = 0), softmax cross-entropy (mean over the batch) on the last z.
 * Parameters: for each layer W_l [out][in] row-major, then b_l [out]. */
static double mlp_loss_grad(int L, const int32_t *w, const double *x, const double *in, const int32_t *label,
                            int B, double *g, int bf16)
{
    double **act = (double **)calloc((size_t)L + 1, sizeof(double *)); /* act[l]: [B][w[l]] */
    act[0] = bf16 ? rounded_copy(in, (size_t)B * w[0]) : (double *)in;
    const double **Wl = (const double **)calloc((size_t)L, sizeof(double *));
    const double **bl = (const double **)calloc((size_t)L, sizeof(double *));
    size_t off = 0;
    for (int l = 0; l < L; ++l) {
        /* bf16 mode: the weight operand of every contraction is rounded; biases stay as they are */
        Wl[l] = bf16 ? rounded_copy(x + off, (size_t)w[l + 1] * w[l]) : x + off;
        off += (size_t)w[l + 1] * w[l];
        bl[l] = x + off; off += (size_t)w[l + 1];
    }
    for (int l = 0; l < L; ++l) {
        int I = w[l], O = w[l + 1];
        act[l + 1] = (double *)malloc(sizeof(double) * (size_t)B * O);
        for (int b = 0; b < B; ++b)
            for (int o = 0; o < O; ++o) {
                double z = bl[l][o];
                for (int k = 0; k < I; ++k) z += Wl[l][(size_t)o * I + k] * act[l][(size_t)b * I + k];
                if (l < L - 1 && z < 0.0) z = 0.0;
                if (l < L - 1 && bf16) z = rbf(z); /* stored hidden activation */
                act[l + 1][(size_t)b * O + o] = z;
            }
    }
    int C = w[L];
    double *dz = g ? (double *)malloc(sizeof(double) * (size_t)B * C) : NULL;
    double loss = softmax_xent(act[L], label, B, C, dz);
    if (g) {
        if (bf16) for (size_t t = 0; t < (size_t)B * C; ++t) dz[t] = rbf(dz[t]);
        size_t end = off;
        for (int l = L - 1; l >= 0; --l) {
            int I = w[l], O = w[l + 1];
            size_t boff = end - (size_t)O, woff = boff - (size_t)O * I;
            end = woff;
            for (int o = 0; o < O; ++o) {
                double sb = 0.0;
                for (int b = 0; b < B; ++b) sb += dz[(size_t)b * O + o];
                g[boff + o] = sb;
                for (int k = 0; k < I; ++k) {
                    double s = 0.0;
                    for (int b = 0; b < B; ++b) s += dz[(size_t)b * O + o] * act[l][(size_t)b * I + k];
                    g[woff + (size_t)o * I + k] = s;
                }
            }
            if (l > 0) {
                double *dprev = (double *)malloc(sizeof(double) * (size_t)B * I);
                for (int b = 0; b < B; ++b)
                    for (int k = 0; k < I; ++k) {
                        double s = 0.0;
                        for (int o = 0; o < O; ++o) s += dz[(size_t)b * O + o] * Wl[l][(size_t)o * I + k];
                        /* act[l] = ReLU(z_{l-1}); positive exactly where z_{l-1} > 0 */
                        s = act[l][(size_t)b * I + k] > 0.0 ? s : 0.0;
                        dprev[(size_t)b * I + k] = bf16 ? rbf(s) : s;
                    }
                free(dz);
                dz = dprev;
            }
        }
        free(dz);
    }
    for (int l = 1; l <= L; ++l) free(act[l]);
    if (bf16) {
        free(act[0]);
        for (int l = 0; l < L; ++l) free((void *)Wl[l]);
    }
    free(act); free(Wl); free(bl);
    return loss;
}

/* -------------------------------------------------------------- ResNet-20-style CNN */

static int conv_out(int H, int stride) { return (H + 2 - 3) / stride + 1; }

/* 3x3 convolution, zero padding 1, given stride, one scalar bias added to every output.
 * in [B][Ci][H][W], w [Co][Ci][3][3], out [B][Co][Ho][Wo]. */
static void conv_fwd(const double *in, int B, int Ci, int H, int W, const double *w, double bias, int Co,
                     int stride, double *out)
{
    int Ho = conv_out(H, stride), Wo = conv_out(W, stride);
    for (int b = 0; b < B; ++b)
        for (int o = 0; o < Co; ++o)
            for (int y = 0; y < Ho; ++y)
                for (int xx = 0; xx < Wo; ++xx) {
                    double s = bias;
                    for (int ci = 0; ci < Ci; ++ci)
                        for (int ky = 0; ky < 3; ++ky) {
                            int iy = y * stride + ky - 1;
                            if (iy < 0 || iy >= H) continue;
                            for (int kx = 0; kx < 3; ++kx) {
                                int ix = xx * stride + kx - 1;
                                if (ix < 0 || ix >= W) continue;
                                s += w[(((size_t)o * Ci + ci) * 3 + ky) * 3 + kx] *
                                     in[(((size_t)b * Ci + ci) * H + iy) * W + ix];
                            }
                        }
                    out[(((size_t)b * Co + o) * Ho + y) * Wo + xx] = s;
                }
}

/* Adjoint of conv_fwd: given dout, accumulate dw (+=), dbias (+=) and, if din != NULL, din (+=). */
static void conv_bwd(const double *in, int B, int Ci, int H, int W, const double *w, int Co, int stride,
                     const double *dout, double *dw, double *dbias, double *din)
{
    int Ho = conv_out(H, stride), Wo = conv_out(W, stride);
    for (int b = 0; b < B; ++b)
        for (int o = 0; o < Co; ++o)
            for (int y = 0; y < Ho; ++y)
                for (int xx = 0; xx < Wo; ++xx) {
                    double go = dout[(((size_t)b * Co + o) * Ho + y) * Wo + xx];
                    *dbias += go;
                    for (int ci = 0; ci < Ci; ++ci)
                        for (int ky = 0; ky < 3; ++ky) {
                            int iy = y * stride + ky - 1;
                            if (iy < 0 || iy >= H) continue;
                            for (int kx = 0; kx < 3; ++kx) {
                                int ix = xx * stride + kx - 1;
                                if (ix < 0 || ix >= W) continue;
                                size_t wi = (((size_t)o * Ci + ci) * 3 + ky) * 3 + kx;
                                size_t ii = (((size_t)b * Ci + ci) * H + iy) * W + ix;
                                dw[wi] += go * in[ii];
                                if (din) din[ii] += go * w[wi];
                            }
                        }
                }
}

/* Parameter-free shortcut.  Same shape: identity.  On a stage change (stride 2, channels
 * doubled): take every second pixel in both directions, copy the Ci input channels into the
 * first Ci output channels and leave the rest zero. */
static void shortcut_add(const double *in, int B, int Ci, int H, int W, int Co, int stride, double *out)
{
    int Ho = conv_out(H, stride), Wo = conv_out(W, stride);
    for (int b = 0; b < B; ++b)
        for (int c = 0; c < Ci; ++c)
            for (int y = 0; y < Ho; ++y)
                for (int xx = 0; xx < Wo; ++xx)
                    out[(((size_t)b * Co + c) * Ho + y) * Wo + xx] +=
                        in[(((size_t)b * Ci + c) * H + y * stride) * W + xx * stride];
}
static void shortcut_bwd(const double *dout, int B, int Ci, int H, int W, int Co, int stride, double *din)
{
    int Ho = conv_out(H, stride), Wo = conv_out(W, stride);
    for (int b = 0; b < B; ++b)
        for (int c = 0; c < Ci; ++c)
            for (int y = 0; y < Ho; ++y)
                for (int xx = 0; xx < Wo; ++xx)
                    din[(((size_t)b * Ci + c) * H + y * stride) * W + xx * stride] +=
                        dout[(((size_t)b * Co + c) * Ho + y) * Wo + xx];
}

typedef struct { int Ci, Co, H, W, stride; size_t w_off, b_off; } conv_desc;

/* BN-free ResNet-20-style network on [B][in_ch][H][W] inputs:
 *   a = ReLU(conv_stem(x) + b)
 *   3 stages x `blocks` basic blocks: u = ReLU(conv1(a) + b1); v = conv2(u) + b2;
 *                                      a = ReLU(v + shortcut(a))
 *     (channels base, 2 base, 4 base; the first conv of stages 2 and 3 has stride 2)
 *   global average pool, fully connected layer with bias, softmax cross-entropy (mean). */
static void round_all(double *v, size_t n) { for (size_t t = 0; t < n; ++t) v[t] = rbf(v[t]); }

/* bf16 mode: the image, every conv weight, every stored activation (after its ReLU) and every
 * back-propagated delta entering a convolution are rounded to bf16; biases, the pooled features
 * and the fully connected layer are not. */
static double resnet_loss_grad(const int32_t *wd, const double *x_master, const double *in_raw,
                               const int32_t *label, int B, double *g, int bf16)
{
    int cin = wd[0], H0 = wd[1], W0 = wd[2], base = wd[3], blocks = wd[4], classes = wd[5];
    int nconv = 1 + 6 * blocks;
    conv_desc *cd = (conv_desc *)calloc((size_t)nconv, sizeof(conv_desc));
    size_t off = 0;
    int q = 0, H = H0, W = W0, cprev = base;
    cd[q] = (conv_desc){cin, base, H, W, 1, off, off + (size_t)base * cin * 9};
    off = cd[q].b_off + 1; ++q;
    for (int s = 0; s < 3; ++s) {
        int c = base << s;
        for (int j = 0; j < blocks; ++j) {
            int stride = (s > 0 && j == 0) ? 2 : 1;
            cd[q] = (conv_desc){cprev, c, H, W, stride, off, off + (size_t)c * cprev * 9};
            off = cd[q].b_off + 1; ++q;
            H = conv_out(H, stride); W = conv_out(W, stride);
            cd[q] = (conv_desc){c, c, H, W, 1, off, off + (size_t)c * c * 9};
            off = cd[q].b_off + 1; ++q;
            cprev = c;
        }
    }
    size_t fcw_off = off, fcb_off = off + (size_t)classes * cprev;
    int Cl = cprev, Hl = H, Wl = W;
    /* x: conv weights as the convolutions see them; xb: biases and the FC layer (never rounded) */
    const double *xb = x_master;
    const double *x = bf16 ? rounded_copy(x_master, fcw_off) : x_master;
    const double *in = bf16 ? rounded_copy(in_raw, (size_t)B * cin * H0 * W0) : in_raw;

    /* forward; keep every block input a[j], every u[j] and the pre-ReLU sums */
    int nb = 3 * blocks;
    double **a = (double **)calloc((size_t)nb + 1, sizeof(double *)); /* post-ReLU block inputs/outputs */
    double **u = (double **)calloc((size_t)nb, sizeof(double *));
    size_t sz0 = (size_t)B * base * H0 * W0;
    a[0] = (double *)malloc(sizeof(double) * sz0);
    conv_fwd(in, B, cin, H0, W0, x + cd[0].w_off, xb[cd[0].b_off], base, 1, a[0]);
    for (size_t t = 0; t < sz0; ++t) if (a[0][t] < 0.0) a[0][t] = 0.0;
    if (bf16) round_all(a[0], sz0);
    for (int j = 0; j < nb; ++j) {
        conv_desc *c1 = &cd[1 + 2 * j], *c2 = &cd[2 + 2 * j];
        size_t szo = (size_t)B * c2->Co * c2->H * c2->W;
        u[j] = (double *)malloc(sizeof(double) * szo);
        conv_fwd(a[j], B, c1->Ci, c1->H, c1->W, x + c1->w_off, xb[c1->b_off], c1->Co, c1->stride, u[j]);
        for (size_t t = 0; t < szo; ++t) if (u[j][t] < 0.0) u[j][t] = 0.0;
        if (bf16) round_all(u[j], szo);
        a[j + 1] = (double *)malloc(sizeof(double) * szo);
        conv_fwd(u[j], B, c2->Ci, c2->H, c2->W, x + c2->w_off, xb[c2->b_off], c2->Co, 1, a[j + 1]);
        shortcut_add(a[j], B, c1->Ci, c1->H, c1->W, c1->Co, c1->stride, a[j + 1]);
        for (size_t t = 0; t < szo; ++t) if (a[j + 1][t] < 0.0) a[j + 1][t] = 0.0;
        if (bf16) round_all(a[j + 1], szo);
    }
    double *pool = (double *)malloc(sizeof(double) * (size_t)B * Cl);
    for (int b = 0; b < B; ++b)
        for (int c = 0; c < Cl; ++c) {
            double s = 0.0;
            for (int t = 0; t < Hl * Wl; ++t) s += a[nb][((size_t)b * Cl + c) * Hl * Wl + t];
            pool[(size_t)b * Cl + c] = s / (double)(Hl * Wl);
        }
    double *z = (double *)malloc(sizeof(double) * (size_t)B * classes);
    for (int b = 0; b < B; ++b)
        for (int o = 0; o < classes; ++o) {
            double s = xb[fcb_off + o];
            for (int c = 0; c < Cl; ++c) s += xb[fcw_off + (size_t)o * Cl + c] * pool[(size_t)b * Cl + c];
            z[(size_t)b * classes + o] = s;
        }
    double *dz = g ? (double *)malloc(sizeof(double) * (size_t)B * classes) : NULL;
    double loss = softmax_xent(z, label, B, classes, dz);

    if (g) {
        size_t d = fcb_off + (size_t)classes;
        memset(g, 0, sizeof(double) * d);
        double *dpool = (double *)calloc((size_t)B * Cl, sizeof(double));
        for (int b = 0; b < B; ++b)
            for (int o = 0; o < classes; ++o) {
                double go = dz[(size_t)b * classes + o];
                g[fcb_off + o] += go;
                for (int c = 0; c < Cl; ++c) {
                    g[fcw_off + (size_t)o * Cl + c] += go * pool[(size_t)b * Cl + c];
                    dpool[(size_t)b * Cl + c] += go * xb[fcw_off + (size_t)o * Cl + c];
                }
            }
        size_t szl = (size_t)B * Cl * Hl * Wl;
        double *da = (double *)malloc(sizeof(double) * szl); /* gradient w.r.t. a[j+1] */
        for (int b = 0; b < B; ++b)
            for (int c = 0; c < Cl; ++c)
                for (int t = 0; t < Hl * Wl; ++t)
                    da[((size_t)b * Cl + c) * Hl * Wl + t] = dpool[(size_t)b * Cl + c] / (double)(Hl * Wl);
        free(dpool);
        for (int j = nb - 1; j >= 0; --j) {
            conv_desc *c1 = &cd[1 + 2 * j], *c2 = &cd[2 + 2 * j];
            size_t szo = (size_t)B * c2->Co * c2->H * c2->W;
            size_t szi = (size_t)B * c1->Ci * c1->H * c1->W;
            /* through the block's final ReLU: a[j+1] > 0 exactly where its argument was > 0 */
            for (size_t t = 0; t < szo; ++t) if (!(a[j + 1][t] > 0.0)) da[t] = 0.0;
            if (bf16) round_all(da, szo);
            double *du = (double *)calloc(szo, sizeof(double));
            conv_bwd(u[j], B, c2->Ci, c2->H, c2->W, x + c2->w_off, c2->Co, 1, da, g + c2->w_off, g + c2->b_off, du);
            for (size_t t = 0; t < szo; ++t) if (!(u[j][t] > 0.0)) du[t] = 0.0;
            if (bf16) round_all(du, szo);
            double *dprev = (double *)calloc(szi, sizeof(double));
            conv_bwd(a[j], B, c1->Ci, c1->H, c1->W, x + c1->w_off, c1->Co, c1->stride, du, g + c1->w_off,
                     g + c1->b_off, dprev);
            shortcut_bwd(da, B, c1->Ci, c1->H, c1->W, c1->Co, c1->stride, dprev);
            free(du); free(da);
            da = dprev;
        }
        for (size_t t = 0; t < sz0; ++t) if (!(a[0][t] > 0.0)) da[t] = 0.0;
        if (bf16) round_all(da, sz0);
        conv_bwd(in, B, cin, H0, W0, x + cd[0].w_off, base, 1, da, g + cd[0].w_off, g + cd[0].b_off, NULL);
        free(da); free(dz);
    }
    for (int j = 0; j <= nb; ++j) free(a[j]);
    for (int j = 0; j < nb; ++j) free(u[j]);
    free(a); free(u); free(pool); free(z); free(cd);
    if (bf16) { free((void *)x); free((void *)in); }
    return loss;
}

/* ---------------------------------------------------------------- public gradient */

/* Algorithm 1 step 3 (with footnote [a]) for ONE worker: loss and, if g != NULL, the mean over the
 * B samples of grad_x F(x; sample).  inputs [B][features] fp64; targets: fp64 y[B] for LSQ, int32
 * labels[B] otherwise.  bf16_operands != 0 selects the rounding mode described at rbf() (ignored by
 * least squares).  Returns the minibatch loss. */
double orc_loss_grad(int32_t kind, int32_t n_layers, const int32_t *widths, const double *x,
                     const double *inputs, const void *targets, int32_t B, double *g, int32_t bf16_operands)
{
    switch (kind) {
    case ORC_LSQ: return lsq_loss_grad(widths[0], x, inputs, (const double *)targets, B, g);
    case ORC_SOFTMAX:
    case ORC_MLP: return mlp_loss_grad(n_layers, widths, x, inputs, (const int32_t *)targets, B, g, bf16_operands);
    case ORC_RESNET20: return resnet_loss_grad(widths, x, inputs, (const int32_t *)targets, B, g, bf16_operands);
    default: return NAN;
    }
}

/* The same for all n workers (independent of each other; OpenMP over workers when enabled).
 * X, G: [n][d]; inputs [n][B][features]; targets [n][B]; loss [n] (may be NULL). */
void orc_grad_all(int32_t kind, int32_t n_layers, const int32_t *widths, int32_t n, int64_t d,
                  const double *X, const double *inputs, const void *targets, int32_t B, double *G,
                  double *loss, int32_t bf16_operands)
{
    int64_t feat = (kind == ORC_RESNET20) ? (int64_t)widths[0] * widths[1] * widths[2] : widths[0];
#pragma omp parallel for schedule(dynamic, 1)
    for (int i = 0; i < n; ++i) {
        const void *t = (kind == ORC_LSQ) ? (const void *)((const double *)targets + (size_t)i * B)
                                          : (const void *)((const int32_t *)targets + (size_t)i * B);
        double l = orc_loss_grad(kind, n_layers, widths, X + (size_t)i * d, inputs + (size_t)i * B * feat, t, B,
                                 G + (size_t)i * d, bf16_operands);
        if (loss) loss[i] = l;
    }
}

int32_t orc_num_threads(void)
{
#ifdef _OPENMP
    extern int omp_get_max_threads(void);
    return omp_get_max_threads();
#else
    return 1;
#endif
}

// Per-worker minibatch gradients in fp32 arithmetic (Algorithm 1 step 3, footnote [a]):
// least squares, softmax regression and ReLU MLPs.  Every worker has its own parameters (row i
// of X), so each layer is a batch of n independent small GEMMs with distinct operands.
#include "dpsgd_internal.h"
#include "grad_common.h"

namespace dpsgd {
namespace {

typedef long long i64;

// ------------------------------------------------------------------------- least squares
// One workgroup per worker.  F = (1/(2B)) ||A x - y||^2, grad = A^T (A x - y) / B.
// Phase 1: residuals r_b (one wave per sample row) into LDS; phase 2: one thread per feature.
__global__ void __launch_bounds__(256)
lsq_grad_kernel(const float *__restrict__ X, i64 ld, const float *__restrict__ A, const float *__restrict__ y, int B,
                int F, float *__restrict__ G, float *__restrict__ loss)
{
    extern __shared__ float r[];   // [B]
    const int w = blockIdx.x;
    const float *x = X + (i64)w * ld;
    const float *a = A + (i64)w * B * F;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int b = wave; b < B; b += 4) {
        float s = 0.f;
        for (int c = lane; c < F; c += 64) s = a[(i64)b * F + c] * x[c] + s;
        for (int off = 32; off > 0; off >>= 1) s += __shfl_down(s, off, 64);
        if (lane == 0) r[b] = s - y[(i64)w * B + b];
    }
    __syncthreads();
    const float invB = 1.0f / (float)B;
    for (int c = threadIdx.x; c < F; c += 256) {
        float s = 0.f;
        for (int b = 0; b < B; ++b) s = a[(i64)b * F + c] * r[b] + s;
        G[(i64)w * ld + c] = s * invB;
    }
    if (loss && wave == 0) {
        float s = 0.f;
        for (int b = lane; b < B; b += 64) s = r[b] * r[b] + s;
        for (int off = 32; off > 0; off >>= 1) s += __shfl_down(s, off, 64);
        if (lane == 0) loss[w] = 0.5f * s * invB;
    }
}

// --------------------------------------------------------------- batched strided fp32 GEMM
// C[w](m,n) = sum_k A[w](m,k) B[w](k,n) (+ bias[w][n]) (ReLU) (masked by mask[w](m,n) > 0),
// every operand addressed through element strides, so that forward (A W^T), data gradient
// (dZ W) and weight gradient (dZ^T A) are the same kernel.  64x64 tile, 16-deep k steps,
// 256 threads x (4x4) outputs, next tile prefetched into registers during the FMAs.
struct GemmArgs {
    const float *A; i64 sAw, sAm, sAk;
    const float *B; i64 sBw, sBk, sBn;
    float *C;       i64 sCw, sCm, sCn;
    const float *bias; i64 sBiasw;      // may be null
    const float *mask; i64 sMw, sMm;    // may be null; unit stride along n
    int M, N, K, relu;
};

template <bool A_KFAST, bool B_NFAST>
__global__ void __launch_bounds__(256) gemm_f32_kernel(GemmArgs g)
{
    __shared__ float As[16][64 + 4];
    __shared__ float Bs[16][64 + 4];
    const int w = blockIdx.z;
    const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    const float *A = g.A + (i64)w * g.sAw;
    const float *Bm = g.B + (i64)w * g.sBw;
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    float acc[4][4] = {};
    float ra[4], rb[4];

    auto fetch = [&](int k0) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int e = tid + 256 * q;
            const int ka = A_KFAST ? (e & 15) : (e >> 6), ma = A_KFAST ? (e >> 4) : (e & 63);
            ra[q] = (m0 + ma < g.M && k0 + ka < g.K) ? A[(i64)(m0 + ma) * g.sAm + (i64)(k0 + ka) * g.sAk] : 0.f;
            const int kb = B_NFAST ? (e >> 6) : (e & 15), nb = B_NFAST ? (e & 63) : (e >> 4);
            rb[q] = (n0 + nb < g.N && k0 + kb < g.K) ? Bm[(i64)(k0 + kb) * g.sBk + (i64)(n0 + nb) * g.sBn] : 0.f;
        }
    };
    auto stage = [&]() {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int e = tid + 256 * q;
            const int ka = A_KFAST ? (e & 15) : (e >> 6), ma = A_KFAST ? (e >> 4) : (e & 63);
            As[ka][ma] = ra[q];
            const int kb = B_NFAST ? (e >> 6) : (e & 15), nb = B_NFAST ? (e & 63) : (e >> 4);
            Bs[kb][nb] = rb[q];
        }
    };

    fetch(0);
    for (int k0 = 0; k0 < g.K; k0 += 16) {
        stage();
        __syncthreads();
        if (k0 + 16 < g.K) fetch(k0 + 16);
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            float a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = a[i] * b[j] + acc[i][j];
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + ty * 4 + i;
        if (m >= g.M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n >= g.N) continue;
            float v = acc[i][j];
            if (g.bias) v += g.bias[(i64)w * g.sBiasw + n];
            if (g.relu) v = v > 0.f ? v : 0.f;
            if (g.mask) v = g.mask[(i64)w * g.sMw + (i64)m * g.sMm + n] > 0.f ? v : 0.f;
            g.C[(i64)w * g.sCw + (i64)m * g.sCm + (i64)n * g.sCn] = v;
        }
    }
}

dpsgd_status gemm_f32(hipStream_t s, int nworkers, const GemmArgs &g)
{
    dim3 grid((unsigned)((g.N + 63) / 64), (unsigned)((g.M + 63) / 64), (unsigned)nworkers);
    if (grid.y > 65535u || grid.z > 65535u) return DPSGD_EUNSUPPORTED;
    const bool akf = g.sAk == 1, bnf = g.sBn == 1;
    if (akf && bnf) hipLaunchKernelGGL((gemm_f32_kernel<true, true>), grid, dim3(256), 0, s, g);
    else if (akf) hipLaunchKernelGGL((gemm_f32_kernel<true, false>), grid, dim3(256), 0, s, g);
    else if (bnf) hipLaunchKernelGGL((gemm_f32_kernel<false, true>), grid, dim3(256), 0, s, g);
    else hipLaunchKernelGGL((gemm_f32_kernel<false, false>), grid, dim3(256), 0, s, g);
    return hip_status(hipGetLastError());
}

// Forward of a layer with few outputs (O <= 16, e.g. the 10 classes): one workgroup per worker and R sample rows; its
// four waves take every fourth 1 KB piece of the rows (lanes stride over the inputs with 16-byte loads), every lane
// keeps R x O partial sums, a wave reduction and a sum over the four waves (in wave order) finish them.  The tiled GEMM
// above would launch only a handful of workgroups for such a shape.  With a whole row per wave the launch was short of
// waves (2048 rows at 128 samples x 16 workers: two waves per SIMD, each a chain of twelve dependent round trips to
// L2: 36.8 us); with the row split over four waves the weights every workgroup pulls from L2 (120 KB, 245 MB per
// launch) set the time (30.1 us), so a workgroup takes two rows per weight piece (23.5 us; four rows, or a wave per
// 1 KB piece with four rows: 27.6 and 40.5 us).
template <int OMAX, bool VEC, int R>   // R sample rows per workgroup: a weight piece fetched from L2 serves R rows
__global__ void __launch_bounds__(256)
linear_fwd_skinny_kernel(const float *__restrict__ act, const float *__restrict__ X, i64 ld, i64 woff, i64 boff, int B, int I,
                         int O, int relu, float *__restrict__ out)
{
    typedef float f4 __attribute__((ext_vector_type(4)));
    __shared__ float part[4][R][OMAX];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int row0 = blockIdx.x * R;   // first sample row inside the worker
    const int w = blockIdx.y;
    const float *a = act + ((i64)w * B + row0) * I;
    const float *Wg = X + (i64)w * ld + woff;
    const int nr = B - row0 < R ? B - row0 : R;
    float acc[R][OMAX];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int o = 0; o < OMAX; ++o) acc[r][o] = 0.f;
    if (VEC) {   // I % 4 == 0 and 16-byte aligned rows: 4 consecutive inputs per lane and step
#pragma unroll 3
        for (int k = (wave * 64 + lane) * 4; k < I; k += 1024) {
            f4 av[R];
#pragma unroll
            for (int r = 0; r < R; ++r) av[r] = *reinterpret_cast<const f4 *>(a + (i64)(r < nr ? r : 0) * I + k);
#pragma unroll
            for (int o = 0; o < OMAX; ++o)
                if (o < O) {
                    const f4 wv = *reinterpret_cast<const f4 *>(Wg + (i64)o * I + k);
#pragma unroll
                    for (int r = 0; r < R; ++r) {
                        acc[r][o] = av[r].x * wv.x + acc[r][o];
                        acc[r][o] = av[r].y * wv.y + acc[r][o];
                        acc[r][o] = av[r].z * wv.z + acc[r][o];
                        acc[r][o] = av[r].w * wv.w + acc[r][o];
                    }
                }
        }
    } else {
        for (int k = wave * 64 + lane; k < I; k += 256) {
            float av[R];
#pragma unroll
            for (int r = 0; r < R; ++r) av[r] = a[(i64)(r < nr ? r : 0) * I + k];
#pragma unroll
            for (int o = 0; o < OMAX; ++o)
                if (o < O) {
                    const float wv = Wg[(i64)o * I + k];
#pragma unroll
                    for (int r = 0; r < R; ++r) acc[r][o] = av[r] * wv + acc[r][o];
                }
        }
    }
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int o = 0; o < OMAX; ++o) {
            float v = acc[r][o];
            for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
            if (lane == 0) part[wave][r][o] = v;
        }
    __syncthreads();
    if ((int)threadIdx.x < nr * OMAX) {
        const int r = threadIdx.x / OMAX, o = threadIdx.x % OMAX;
        if (o < O) {
            float v = ((part[0][r][o] + part[1][r][o]) + part[2][r][o]) + part[3][r][o];   // in wave order
            v += X[(i64)w * ld + boff + o];
            if (relu) v = v > 0.f ? v : 0.f;
            out[((i64)w * B + row0 + r) * O + o] = v;
        }
    }
}

// gb[w][o] = sum_b dz[w][b][o]: a wave per output, its lanes stride over the samples (a thread per output walking the
// samples one after the other was a chain of B dependent loads: 9.5 us for 10 outputs x 128 samples)
__global__ void __launch_bounds__(256)
bias_grad_kernel(const float *__restrict__ dz, int B, int O, float *__restrict__ G, i64 ld, i64 boff)
{
    const int lane = threadIdx.x & 63;
    const int o = blockIdx.x * 4 + (threadIdx.x >> 6), w = blockIdx.y;
    if (o >= O) return;
    float s = 0.f;
    for (int b = lane; b < B; b += 64) s += dz[((i64)w * B + b) * O + o];
    for (int off = 32; off > 0; off >>= 1) s += __shfl_down(s, off, 64);
    if (lane == 0) G[(i64)w * ld + boff + o] = s;
}

__global__ void __launch_bounds__(256) bf16_to_f32_kernel(const uint16_t *__restrict__ in, float *__restrict__ out, i64 count)
{
    const i64 i = (i64)blockIdx.x * 256 + threadIdx.x;
    if (i < count) out[i] = __uint_as_float((uint32_t)in[i] << 16);
}

}  // namespace

// Softmax cross-entropy over logits [n][B][C] (shared with the bf16 path): one workgroup per
// worker, one thread per sample.  dz = (softmax - onehot)/B, loss[w] = mean_b(lse - z[label]).
__global__ void __launch_bounds__(256)
softmax_xent_kernel(const float *__restrict__ z, const int *__restrict__ labels, int B, int C, float *__restrict__ dz,
                    float *__restrict__ loss, float *__restrict__ G, long long ld, long long boff)
{
    __shared__ float red[256];
    const int w = blockIdx.x;
    const float invB = 1.0f / (float)B;
    float local = 0.f;
    for (int b = threadIdx.x; b < B; b += 256) {
        const float *zb = z + ((i64)w * B + b) * C;
        float *db = dz + ((i64)w * B + b) * C;
        int lab = labels[(i64)w * B + b];
        lab = lab < 0 ? 0 : (lab >= C ? C - 1 : lab);
        float mx = zb[0];
        for (int c = 1; c < C; ++c) mx = fmaxf(mx, zb[c]);
        float se = 0.f;
        for (int c = 0; c < C; ++c) se += expf(zb[c] - mx);
        const float lse = mx + logf(se);
        local += lse - zb[lab];
        for (int c = 0; c < C; ++c) db[c] = (expf(zb[c] - lse) - (c == lab ? 1.f : 0.f)) * invB;
    }
    red[threadIdx.x] = local;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
        __syncthreads();
    }
    if (loss && threadIdx.x == 0) loss[w] = red[0] * invB;
    if (G) {   // the class layer's bias gradient: the worker's dz rows were written by this workgroup, before the barriers
               // above; a wave per class, lanes stride over the samples (the sums of bias_grad_kernel, bit for bit)
        const int lane = threadIdx.x & 63;
        for (int c = threadIdx.x >> 6; c < C; c += 4) {
            float s = 0.f;
            for (int b = lane; b < B; b += 64) s += dz[((i64)w * B + b) * C + c];
            for (int off = 32; off > 0; off >>= 1) s += __shfl_down(s, off, 64);
            if (lane == 0) G[(i64)w * ld + boff + c] = s;
        }
    }
}

size_t f32_workspace_bytes(const dpsgd_ctx *ctx, const dpsgd_model_desc &m)
{
    if (m.kind == DPSGD_MODEL_LSQ) return 256;
    const size_t n = (size_t)ctx->n, B = (size_t)m.batch;
    size_t floats = 0, widest = 0;
    const size_t L = m.widths.size() - 1;
    if (m.input_is_bf16) floats += n * B * (size_t)m.widths[0];
    for (size_t l = 1; l <= L; ++l) {
        floats += n * B * (size_t)m.widths[l];
        if ((size_t)m.widths[l] > widest) widest = (size_t)m.widths[l];
    }
    floats += 2 * n * B * widest;
    return floats * sizeof(float) + 256;
}

dpsgd_status launch_grad_f32(dpsgd_ctx *ctx, const dpsgd_model_desc &m, const float *X, const void *inputs,
                             const void *targets, float *G, float *loss)
{
    hipStream_t s = ctx->stream;
    const int n = ctx->n, B = m.batch;
    if (m.kind == DPSGD_MODEL_LSQ) {
        if (B > 8192) return DPSGD_EUNSUPPORTED;
        hipLaunchKernelGGL(lsq_grad_kernel, dim3((unsigned)n), dim3(256), (size_t)B * sizeof(float), s, X, ctx->ld,
                           (const float *)inputs, (const float *)targets, B, m.widths[0], G, loss);
        return hip_status(hipGetLastError());
    }
    const int L = (int)m.widths.size() - 1;
    float *ws = (float *)ctx->ws;
    const float *act0 = (const float *)inputs;
    if (m.input_is_bf16) {
        const i64 cnt = (i64)n * B * m.widths[0];
        hipLaunchKernelGGL(bf16_to_f32_kernel, dim3((unsigned)((cnt + 255) / 256)), dim3(256), 0, s,
                           (const uint16_t *)inputs, ws, cnt);
        act0 = ws;
        ws += cnt;
    }
    std::vector<const float *> act(L + 1);
    std::vector<i64> woff(L), boff(L);
    act[0] = act0;
    i64 off = 0, widest = 0;
    for (int l = 0; l < L; ++l) {
        woff[l] = off; off += (i64)m.widths[l + 1] * m.widths[l];
        boff[l] = off; off += m.widths[l + 1];
        act[l + 1] = ws;
        ws += (i64)n * B * m.widths[l + 1];
        if (m.widths[l + 1] > widest) widest = m.widths[l + 1];
    }
    float *dz = ws, *dz2 = ws + (i64)n * B * widest;

    dpsgd_status st;
    for (int l = 0; l < L; ++l) {
        const int I = m.widths[l], O = m.widths[l + 1];
        GemmArgs g{};
        g.A = act[l]; g.sAw = (i64)B * I; g.sAm = I; g.sAk = 1;
        g.B = X + woff[l]; g.sBw = ctx->ld; g.sBk = 1; g.sBn = I;
        g.C = (float *)act[l + 1]; g.sCw = (i64)B * O; g.sCm = O; g.sCn = 1;
        g.bias = X + boff[l]; g.sBiasw = ctx->ld;
        g.M = B; g.N = O; g.K = I; g.relu = (l < L - 1);
        if (O <= 16 && I >= 256) {
            const bool vec = (I % 4) == 0 && (woff[l] % 4) == 0 && (ctx->ld % 4) == 0 &&
                             (reinterpret_cast<uintptr_t>(X) % 16) == 0 && (reinterpret_cast<uintptr_t>(act[l]) % 16) == 0;
            constexpr int R = 2;
            dim3 sgrid((unsigned)((B + R - 1) / R), (unsigned)n);
            if (vec)
                hipLaunchKernelGGL((linear_fwd_skinny_kernel<16, true, R>), sgrid, dim3(256), 0, s, act[l], X, ctx->ld, woff[l],
                                   boff[l], B, I, O, g.relu, (float *)act[l + 1]);
            else
                hipLaunchKernelGGL((linear_fwd_skinny_kernel<16, false, R>), sgrid, dim3(256), 0, s, act[l], X, ctx->ld, woff[l],
                                   boff[l], B, I, O, g.relu, (float *)act[l + 1]);
            if ((st = hip_status(hipGetLastError())) != DPSGD_OK) return st;
            continue;
        }
        if ((st = gemm_f32(s, n, g)) != DPSGD_OK) return st;
    }
    const int C = m.widths[L];
    hipLaunchKernelGGL(softmax_xent_kernel, dim3((unsigned)n), dim3(256), 0, s, act[L], (const int *)targets, B, C, dz,
                       loss, G, (long long)ctx->ld, (long long)boff[L - 1]);   // with the class layer's bias gradient
    for (int l = L - 1; l >= 0; --l) {
        const int I = m.widths[l], O = m.widths[l + 1];
        GemmArgs g{};   // weight gradient: dW[o][i] = sum_b dz[b][o] act_l[b][i]
        g.A = dz; g.sAw = (i64)B * O; g.sAm = 1; g.sAk = O;
        g.B = act[l]; g.sBw = (i64)B * I; g.sBk = I; g.sBn = 1;
        g.C = G + woff[l]; g.sCw = ctx->ld; g.sCm = I; g.sCn = 1;
        g.M = O; g.N = I; g.K = B;
        if ((st = gemm_f32(s, n, g)) != DPSGD_OK) return st;
        if (l < L - 1)   // (the class layer's came with the softmax launch)
            hipLaunchKernelGGL(bias_grad_kernel, dim3((unsigned)((O + 3) / 4), (unsigned)n), dim3(256), 0, s, dz, B, O, G,
                               ctx->ld, boff[l]);
        if (l > 0) {   // data gradient through the ReLU: dz_prev = (dz W_l) * [act_l > 0]
            GemmArgs h{};
            h.A = dz; h.sAw = (i64)B * O; h.sAm = O; h.sAk = 1;
            h.B = X + woff[l]; h.sBw = ctx->ld; h.sBk = I; h.sBn = 1;
            h.C = dz2; h.sCw = (i64)B * I; h.sCm = I; h.sCn = 1;
            h.mask = act[l]; h.sMw = (i64)B * I; h.sMm = I;
            h.M = B; h.N = I; h.K = O;
            if ((st = gemm_f32(s, n, h)) != DPSGD_OK) return st;
            float *t = dz; dz = dz2; dz2 = t;
        }
    }
    return hip_status(hipGetLastError());
}

}  // namespace dpsgd

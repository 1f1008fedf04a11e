// Per-worker minibatch gradient of the BN-free ResNet-20-style CNN (Algorithm 1 step 3,
// footnote [a]): 3x3 stem, 3 stages of basic blocks (base, 2 base, 4 base channels; stride 2 at
// the first conv of stages 2 and 3), one scalar bias per conv, parameter-free shortcuts, global
// average pool, fully connected layer, softmax cross-entropy.
//
// Arithmetic: the image, every conv weight, every stored activation (after its ReLU) and every
// delta entering a convolution are bf16 (round to nearest even); sums are fp32; biases, pooling
// and the fully connected layer are fp32.  Activations and deltas are channel-major bf16
// ([n][B][C][H][W]) in the workspace.
//
// This file holds the shape-generic kernels (any channel count, image size, stride): one thread
// per output element for forward and data gradient, one workgroup per (worker, c_out, c_in) for
// the weight gradient.  They define the results; faster kernels for the benchmark's channel
// counts are dispatched from conv_mfma.hip and must agree with these.
#include "grad_common.h"
#include "resnet_common.h"

namespace dpsgd {
namespace {

typedef long long i64;

// ------------------------------------------------------------------------------ forward
// IN_FP32: the source is the fp32 image (rounded on load), else a bf16 tensor; both channel-major.
template <bool IN_FP32>
__global__ void __launch_bounds__(256)
conv_fwd_generic_kernel(const void *__restrict__ in, const float *__restrict__ X, i64 ld, ConvDesc c, int B, i64 total,
                        const bf16_t *__restrict__ sc, int scC, int scH, int scW, int scS, bf16_t *__restrict__ out)
{
    const i64 idx = (i64)blockIdx.x * 256 + threadIdx.x;   // over [w][b][co][y][x]
    if (idx >= total) return;
    i64 t = idx;
    const int x = (int)(t % c.Wo); t /= c.Wo;
    const int y = (int)(t % c.Ho); t /= c.Ho;
    const int co = (int)(t % c.Co); t /= c.Co;
    const int b = (int)(t % B);
    const int w = (int)(t / B);
    const float *Wg = X + (i64)w * ld + c.w_off + (i64)co * c.Ci * 9;
    float acc = 0.f;
    for (int ci = 0; ci < c.Ci; ++ci)
        for (int ky = 0; ky < 3; ++ky) {
            const int iy = y * c.stride + ky - 1;
            if (iy < 0 || iy >= c.H) continue;
            for (int kx = 0; kx < 3; ++kx) {
                const int ix = x * c.stride + kx - 1;
                if (ix < 0 || ix >= c.W) continue;
                const i64 src = ((((i64)w * B + b) * c.Ci + ci) * c.H + iy) * c.W + ix;
                const float v = IN_FP32 ? bf2f(f2bf(((const float *)in)[src])) : bf2f(((const bf16_t *)in)[src]);
                acc = v * bf2f(f2bf(Wg[(ci * 3 + ky) * 3 + kx])) + acc;
            }
        }
    float v = acc + X[(i64)w * ld + c.b_off];
    if (sc && co < scC) v += bf2f(sc[((((i64)w * B + b) * scC + co) * scH + y * scS) * scW + x * scS]);
    v = v > 0.f ? v : 0.f;
    out[idx] = f2bf(v);
}

// ------------------------------------------------------------------------ data gradient
// din[w][b][ci][iy][ix] = round( [act > 0] * ( sum_{co,ky,kx} dout[co][oy][ox] w[co][ci][ky][kx]
//                                              + shortcut delta ) ),  oy = (iy + 1 - ky)/stride.
__global__ void __launch_bounds__(256)
conv_dgrad_generic_kernel(const bf16_t *__restrict__ dout, const float *__restrict__ X, i64 ld, ConvDesc c, int B,
                          i64 total, const bf16_t *__restrict__ scd, int scC, int scH, int scW, int scS,
                          const bf16_t *__restrict__ act, bf16_t *__restrict__ din)
{
    const i64 idx = (i64)blockIdx.x * 256 + threadIdx.x;   // over [w][b][ci][iy][ix]
    if (idx >= total) return;
    i64 t = idx;
    const int ix = (int)(t % c.W); t /= c.W;
    const int iy = (int)(t % c.H); t /= c.H;
    const int ci = (int)(t % c.Ci); t /= c.Ci;
    const int b = (int)(t % B);
    const int w = (int)(t / B);
    const float *Wg = X + (i64)w * ld + c.w_off;
    float acc = 0.f;
    for (int ky = 0; ky < 3; ++ky) {
        const int ty = iy + 1 - ky;
        if (ty < 0 || ty % c.stride) continue;
        const int oy = ty / c.stride;
        if (oy >= c.Ho) continue;
        for (int kx = 0; kx < 3; ++kx) {
            const int tx = ix + 1 - kx;
            if (tx < 0 || tx % c.stride) continue;
            const int ox = tx / c.stride;
            if (ox >= c.Wo) continue;
            const bf16_t *dp = dout + ((i64)w * B + b) * c.Co * c.Ho * c.Wo + (i64)oy * c.Wo + ox;
            for (int co = 0; co < c.Co; ++co)
                acc = bf2f(dp[(i64)co * c.Ho * c.Wo]) * bf2f(f2bf(Wg[(((i64)co * c.Ci + ci) * 3 + ky) * 3 + kx])) + acc;
        }
    }
    if (scd && (iy % scS) == 0 && (ix % scS) == 0 && iy / scS < scH && ix / scS < scW)
        acc += bf2f(scd[((((i64)w * B + b) * scC + ci) * scH + iy / scS) * scW + ix / scS]);
    const bool pos = bf16_positive(act[idx]);
    din[idx] = f2bf(pos ? acc : 0.f);
}

// ---------------------------------------------------------------------- weight gradient
// One workgroup per (c_in, c_out, worker): 9 tap sums over all (b, y, x), fixed-order reduction.
template <bool IN_FP32>
__global__ void __launch_bounds__(256)
conv_wgrad_generic_kernel(const void *__restrict__ in, const bf16_t *__restrict__ dout, ConvDesc c, int B,
                          float *__restrict__ G, i64 ld)
{
    __shared__ float red[9][256];
    const int ci = blockIdx.x, co = blockIdx.y, w = blockIdx.z;
    float acc[9];
#pragma unroll
    for (int t = 0; t < 9; ++t) acc[t] = 0.f;
    const int npix = B * c.Ho * c.Wo;
    for (int p = threadIdx.x; p < npix; p += 256) {
        const int x = p % c.Wo, y = (p / c.Wo) % c.Ho, b = p / (c.Wo * c.Ho);
        const float go = bf2f(dout[((((i64)w * B + b) * c.Co + co) * c.Ho + y) * c.Wo + x]);
        if (go == 0.f) continue;
#pragma unroll
        for (int ky = 0; ky < 3; ++ky) {
            const int iy = y * c.stride + ky - 1;
            if (iy < 0 || iy >= c.H) continue;
#pragma unroll
            for (int kx = 0; kx < 3; ++kx) {
                const int ix = x * c.stride + kx - 1;
                if (ix < 0 || ix >= c.W) continue;
                const i64 src = ((((i64)w * B + b) * c.Ci + ci) * c.H + iy) * c.W + ix;
                const float v = IN_FP32 ? bf2f(f2bf(((const float *)in)[src])) : bf2f(((const bf16_t *)in)[src]);
                acc[ky * 3 + kx] = go * v + acc[ky * 3 + kx];
            }
        }
    }
#pragma unroll
    for (int t = 0; t < 9; ++t) red[t][threadIdx.x] = acc[t];
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off)
#pragma unroll
            for (int t = 0; t < 9; ++t) red[t][threadIdx.x] += red[t][threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x < 9) G[(i64)w * ld + c.w_off + ((i64)co * c.Ci + ci) * 9 + threadIdx.x] = red[threadIdx.x][0];
}

// Scalar bias gradient: sum of one worker's delta tensor (count elements), fixed order.
__global__ void __launch_bounds__(1024)
sum_delta_kernel(const bf16_t *__restrict__ d, i64 count, float *__restrict__ G, i64 ld, i64 b_off)
{
    __shared__ float red[1024];
    const int w = blockIdx.x;
    const bf16_t *p = d + (i64)w * count;
    float s0 = 0.f, s1 = 0.f;
    i64 i = threadIdx.x;
    for (; i + 1024 < count; i += 2048) {
        s0 += bf2f(p[i]);
        s1 += bf2f(p[i + 1024]);
    }
    for (; i < count; i += 1024) s0 += bf2f(p[i]);
    red[threadIdx.x] = s0 + s1;
    __syncthreads();
    for (int off = 512; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
        __syncthreads();
    }
    if (threadIdx.x == 0) G[(i64)w * ld + b_off] = red[0];
}

// ------------------------------------------------------------ head: pool, FC, loss, FC grads
// Global average pool: a [n*B*C][HW] bf16 -> pool [n*B*C] fp32, one thread per (image, channel), pixels in order.
__global__ void __launch_bounds__(256)
pool_fwd_kernel(const bf16_t *__restrict__ a, int HW, i64 total, float *__restrict__ pool)
{
    const i64 e = (i64)blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;
    const bf16_t *p = a + e * HW;
    float s = 0.f;
    int t = 0;
    if ((HW & 7) == 0)
        for (; t < HW; t += 8) {
            const uint4 v = *reinterpret_cast<const uint4 *>(p + t);
            s += bf2f((bf16_t)(v.x & 0xffff)); s += bf2f((bf16_t)(v.x >> 16));
            s += bf2f((bf16_t)(v.y & 0xffff)); s += bf2f((bf16_t)(v.y >> 16));
            s += bf2f((bf16_t)(v.z & 0xffff)); s += bf2f((bf16_t)(v.z >> 16));
            s += bf2f((bf16_t)(v.w & 0xffff)); s += bf2f((bf16_t)(v.w >> 16));
        }
    for (; t < HW; ++t) s += bf2f(p[t]);
    pool[e] = s * (1.0f / (float)HW);
}

// One workgroup per worker.  pool / dpool: [n][B][C] fp32, z: [n][B][K] fp32.
// STAGED: the worker's pooled features, FC weights (rows one float apart from a multiple of the bank count) and logits
// sit in LDS ((B (C + 1) + K (C + 1) + B K) floats of dynamic LDS) and
// every loop below reads them from there; the arithmetic and its order are the same either way, so are the bits.
template <bool STAGED>
__global__ void __launch_bounds__(256)
head_kernel(const float *__restrict__ X, i64 ld, i64 fcw_off, i64 fcb_off, int B, int HW, int C, int K,
            const int *__restrict__ labels, const float *__restrict__ pool, float *__restrict__ z,
            float *__restrict__ dpool, float *__restrict__ G, float *__restrict__ loss)
{
    __shared__ float red[256];
    extern __shared__ __attribute__((aligned(16))) float head_lds[];
    const int w = blockIdx.x, tid = threadIdx.x;
    const float *fw = X + (i64)w * ld + fcw_off, *fb = X + (i64)w * ld + fcb_off;
    const float *pw = pool + (i64)w * B * C;
    float *zw = z + (i64)w * B * K, *dpw = dpool + (i64)w * B * C;
    const int CP = STAGED ? C + 1 : C;   // row pitch of the pooled features and of the FC weights
    if (STAGED) {
        float *ps = head_lds, *fs = ps + B * CP;
        for (int e = tid; e < B * C; e += 256) ps[(e / C) * CP + e % C] = pw[e];
        for (int e = tid; e < K * C; e += 256) fs[(e / C) * CP + e % C] = fw[e];
        __syncthreads();
        pw = ps;
        fw = fs;
        zw = fs + K * CP;
    }
    const float inv_hw = 1.0f / (float)HW;
    for (int e = tid; e < B * K; e += 256) {
        const int b = e / K, o = e % K;
        float s = fb[o];
        for (int ch = 0; ch < C; ++ch) s = fw[o * CP + ch] * pw[b * CP + ch] + s;
        zw[e] = s;
    }
    __syncthreads();
    const float invB = 1.0f / (float)B;
    float local = 0.f;
    for (int b = tid; b < B; b += 256) {
        float *zb = zw + b * K;
        int lab = labels[(i64)w * B + b];
        lab = lab < 0 ? 0 : (lab >= K ? K - 1 : lab);
        float mx = zb[0];
        for (int o = 1; o < K; ++o) mx = fmaxf(mx, zb[o]);
        float se = 0.f;
        for (int o = 0; o < K; ++o) se += expf(zb[o] - mx);
        const float lse = mx + logf(se);
        local += lse - zb[lab];
        for (int o = 0; o < K; ++o) zb[o] = (expf(zb[o] - lse) - (o == lab ? 1.f : 0.f)) * invB;   // dz in place
    }
    red[tid] = local;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if (tid < off) red[tid] += red[tid + off];
        __syncthreads();
    }
    if (loss && tid == 0) loss[w] = red[0] * invB;
    for (int e = tid; e < K * C; e += 256) {
        const int o = e / C, ch = e % C;
        float s = 0.f;
        for (int b = 0; b < B; ++b) s = zw[b * K + o] * pw[b * CP + ch] + s;
        G[(i64)w * ld + fcw_off + e] = s;
    }
    for (int o = tid; o < K; o += 256) {
        float s = 0.f;
        for (int b = 0; b < B; ++b) s += zw[b * K + o];
        G[(i64)w * ld + fcb_off + o] = s;
    }
    for (int e = tid; e < B * C; e += 256) {
        const int b = e / C, ch = e % C;
        float s = 0.f;
        for (int o = 0; o < K; ++o) s = zw[b * K + o] * fw[o * CP + ch] + s;
        dpw[e] = s * inv_hw;
    }
}

// dv[w][b][c][t] = round([a > 0] * dpool[w][b][c])   (dpool already divided by H*W)
__global__ void __launch_bounds__(256)
pool_bwd_kernel(const bf16_t *__restrict__ a, const float *__restrict__ dpool, int HW, i64 total, bf16_t *__restrict__ dv)
{
    const i64 idx = (i64)blockIdx.x * 256 + threadIdx.x;   // over [w*b][c][t]
    if (idx >= total) return;
    dv[idx] = bf16_positive(a[idx]) ? f2bf(dpool[idx / HW]) : (bf16_t)0;
}

// The same for HW % 8 == 0: a thread takes 8 pixels of one (image, channel) plane, 16 bytes in and out.
__global__ void __launch_bounds__(256)
pool_bwd_vec_kernel(const bf16_t *__restrict__ a, const float *__restrict__ dpool, int HW, i64 total8, bf16_t *__restrict__ dv)
{
    const i64 u = (i64)blockIdx.x * 256 + threadIdx.x;   // over 16-byte units of [w*b][c][t]
    if (u >= total8) return;
    const uint4 v = *reinterpret_cast<const uint4 *>(a + u * 8);
    const unsigned d = f2bf(dpool[(u * 8) / HW]);
    const unsigned in[4] = {v.x, v.y, v.z, v.w};
    unsigned out[4];
#pragma unroll
    for (int h = 0; h < 4; ++h)
        out[h] = (bf16_positive((bf16_t)(in[h] & 0xffffu)) ? d : 0u) | (bf16_positive((bf16_t)(in[h] >> 16)) ? d << 16 : 0u);
    *reinterpret_cast<uint4 *>(dv + u * 8) = make_uint4(out[0], out[1], out[2], out[3]);
}

unsigned blocks_for(i64 total) { return (unsigned)((total + 255) / 256); }

}  // namespace

ResnetPlan make_resnet_plan(const dpsgd_model_desc &m)
{
    ResnetPlan p;
    const int cin = m.widths[0], H0 = m.widths[1], W0 = m.widths[2], base = m.widths[3], blocks = m.widths[4];
    p.classes = m.widths[5];
    auto out_dim = [](int h, int s) { return (h + 2 - 3) / s + 1; };
    i64 off = 0;
    int H = H0, W = W0, cprev = base;
    auto add = [&](int Ci, int Co, int h, int w, int s) {
        ConvDesc c;
        c.Ci = Ci; c.Co = Co; c.H = h; c.W = w; c.stride = s; c.Ho = out_dim(h, s); c.Wo = out_dim(w, s);
        c.w_off = off; off += (i64)Co * Ci * 9;
        c.b_off = off; off += 1;
        p.convs.push_back(c);
    };
    add(cin, base, H, W, 1);
    for (int s = 0; s < 3; ++s) {
        const int c = base << s;
        for (int j = 0; j < blocks; ++j) {
            const int stride = (s > 0 && j == 0) ? 2 : 1;
            add(cprev, c, H, W, stride);
            H = out_dim(H, stride); W = out_dim(W, stride);
            add(c, c, H, W, 1);
            cprev = c;
        }
    }
    p.fcw_off = off; off += (i64)p.classes * cprev;
    p.fcb_off = off;
    p.C_last = cprev; p.H_last = H; p.W_last = W;
    p.nblocks = 3 * blocks;
    return p;
}


// Workspace layout, shared by resnet_workspace_bytes and launch_grad_resnet.
namespace {
struct Workspace {
    std::vector<Tensor> out;              // output of every conv: out[0] = a_0, out[1+2j] = u_j, out[2+2j] = a_{j+1}
    Tensor delta[3];                      // rotating delta buffers
    std::vector<bf16_t *> wpack_f, wpack_d;
    bf16_t *image_bf16 = nullptr;         // bf16 copy of an fp32 image (channel-major, as given)
    bf16_t *image_nhwc8 = nullptr;        // image padded to 8 channels, pixel-major (MFMA stem only)
    float *pool = nullptr, *dpool = nullptr, *logits = nullptr;
    std::vector<float *> partials;        // per conv: the partial sums of its weight gradient
    size_t bytes = 0;
};

Workspace carve(const dpsgd_ctx *ctx, const dpsgd_model_desc &m, const ResnetPlan &p, unsigned char *base)
{
    Workspace w;
    size_t off = 0;
    auto take = [&](size_t b) {
        unsigned char *q = base ? base + off : nullptr;
        off += (b + 255) / 256 * 256;
        return q;
    };
    const size_t nB = (size_t)ctx->n * m.batch;
    size_t biggest = 0;
    std::vector<size_t> part;
    for (const ConvDesc &c : p.convs) {
        const size_t e = nB * c.Ho * c.Wo * c.Co;
        Tensor t;
        t.t = (bf16_t *)take(e * 2);
        if (conv_forward_writes_sign(c, w.out.empty())) t.sign = (unsigned char *)take(e / 8);
        w.out.push_back(t);
        biggest = e > biggest ? e : biggest;
        w.wpack_f.push_back((bf16_t *)take(conv_pack_bytes(c, false) * ctx->n));
        w.wpack_d.push_back((bf16_t *)take(conv_pack_bytes(c, true) * ctx->n));
        part.push_back(conv_wgrad_partial_bytes(c, m.batch) * ctx->n);
    }
    for (int i = 0; i < 3; ++i) w.delta[i].t = (bf16_t *)take(biggest * 2);
    if (!m.input_is_bf16) w.image_bf16 = (bf16_t *)take(nB * p.convs[0].Ci * p.convs[0].H * p.convs[0].W * 2);
    if (conv_stem_uses_mfma(p.convs[0])) w.image_nhwc8 = (bf16_t *)take(nB * p.convs[0].H * p.convs[0].W * 8 * 2);
    w.pool = (float *)take(nB * p.C_last * 4);
    w.dpool = (float *)take(nB * p.C_last * 4);
    w.logits = (float *)take(nB * p.classes * 4);
    for (size_t pb : part) w.partials.push_back((float *)take(pb));
    w.bytes = off + 256;
    return w;
}
}  // namespace

size_t resnet_workspace_bytes(const dpsgd_ctx *ctx, const dpsgd_model_desc &m)
{
    const ResnetPlan p = make_resnet_plan(m);
    return carve(ctx, m, p, nullptr).bytes;
}

dpsgd_status launch_grad_resnet(dpsgd_ctx *ctx, const dpsgd_model_desc &m, const float *X, const void *inputs,
                                const void *targets, float *G, float *loss)
{
    hipStream_t s = ctx->stream;
    const ResnetPlan p = make_resnet_plan(m);
    const int n = ctx->n, B = m.batch;
    const i64 nB = (i64)n * B;
    if (n > 65535 || B > 65535) return DPSGD_EUNSUPPORTED;
    for (const ConvDesc &c : p.convs)
        if (c.Ho < 1 || c.Wo < 1 || c.Ci > 65535 || c.Co > 65535) return DPSGD_EUNSUPPORTED;
    Workspace ws = carve(ctx, m, p, (unsigned char *)ctx->ws);
    auto a_of = [&](int j) { return ws.out[j == 0 ? 0 : 2 * j]; };   // block input/output j
    auto u_of = [&](int j) { return ws.out[1 + 2 * j]; };
    const ShortcutRef none{nullptr, 0, 0, 0, 1};
    dpsgd_status st;

    // bf16 operands of the convolutions in the layout the MFMA kernels read (no-op for generic convs)
    if ((st = conv_pack_weights(ctx, p.convs, X, ws.wpack_f, ws.wpack_d)) != DPSGD_OK) return st;

    // ---- forward
    const bool stem_mfma = conv_stem_uses_mfma(p.convs[0]);
    // the image as bf16, channel-major (what the stem's weight gradient contracts over)
    const bf16_t *image_chw = m.input_is_bf16 ? (const bf16_t *)inputs : ws.image_bf16;
    if (stem_mfma) {
        const ConvDesc &c = p.convs[0];
        if ((st = conv_prep_image(ctx, c, B, inputs, m.input_is_bf16, ws.image_bf16, ws.image_nhwc8)) != DPSGD_OK) return st;
        Tensor img8;
        img8.t = ws.image_nhwc8;
        if ((st = conv_forward(ctx, c, B, img8, X, ws.wpack_f[0], none, ws.out[0])) != DPSGD_OK) return st;
    } else {
        const ConvDesc &c = p.convs[0];
        const i64 total = nB * c.Ho * c.Wo * c.Co;
        if (m.input_is_bf16)
            hipLaunchKernelGGL(conv_fwd_generic_kernel<false>, dim3(blocks_for(total)), dim3(256), 0, s, inputs, X, ctx->ld,
                               c, B, total, nullptr, 0, 0, 0, 1, ws.out[0].t);
        else
            hipLaunchKernelGGL(conv_fwd_generic_kernel<true>, dim3(blocks_for(total)), dim3(256), 0, s, inputs, X, ctx->ld,
                               c, B, total, nullptr, 0, 0, 0, 1, ws.out[0].t);
    }
    for (int j = 0; j < p.nblocks; ++j) {
        const ConvDesc &c1 = p.convs[1 + 2 * j], &c2 = p.convs[2 + 2 * j];
        if (conv_block_forward_ok(ctx, c1, c2) && u_of(j).sign && a_of(j + 1).sign) {
            if ((st = conv_block_forward(ctx, c1, c2, B, a_of(j), X, ws.wpack_f[1 + 2 * j], ws.wpack_f[2 + 2 * j], u_of(j),
                                         a_of(j + 1))) != DPSGD_OK)
                return st;
            continue;
        }
        if ((st = conv_forward(ctx, c1, B, a_of(j), X, ws.wpack_f[1 + 2 * j], none, u_of(j))) != DPSGD_OK) return st;
        const ShortcutRef sc{a_of(j).t, c1.Ci, c1.H, c1.W, c1.stride};
        if ((st = conv_forward(ctx, c2, B, u_of(j), X, ws.wpack_f[2 + 2 * j], sc, a_of(j + 1))) != DPSGD_OK) return st;
    }
    const int HWl = p.H_last * p.W_last;
    hipLaunchKernelGGL(pool_fwd_kernel, dim3(blocks_for(nB * p.C_last)), dim3(256), 0, s, a_of(p.nblocks).t, HWl,
                       nB * p.C_last, ws.pool);
    {
        const size_t head_lds = ((size_t)(B + p.classes) * (p.C_last + 1) + (size_t)B * p.classes) * sizeof(float);
        if (head_lds <= 48 * 1024)
            hipLaunchKernelGGL(head_kernel<true>, dim3((unsigned)n), dim3(256), head_lds, s, X, ctx->ld, p.fcw_off, p.fcb_off, B,
                               HWl, p.C_last, p.classes, (const int *)targets, ws.pool, ws.logits, ws.dpool, G, loss);
        else
            hipLaunchKernelGGL(head_kernel<false>, dim3((unsigned)n), dim3(256), 0, s, X, ctx->ld, p.fcw_off, p.fcb_off, B, HWl,
                               p.C_last, p.classes, (const int *)targets, ws.pool, ws.logits, ws.dpool, G, loss);
    }

    // ---- backward
    Tensor dv = ws.delta[0], du = ws.delta[1], dnext = ws.delta[2];
    WgradReduceList pending;   // the sums over the weight-gradient partials, one launch after the last convolution
    {
        const i64 total = nB * HWl * p.C_last;
        if ((HWl & 7) == 0)
            hipLaunchKernelGGL(pool_bwd_vec_kernel, dim3(blocks_for(total / 8)), dim3(256), 0, s, a_of(p.nblocks).t, ws.dpool, HWl,
                               total / 8, dv.t);
        else
            hipLaunchKernelGGL(pool_bwd_kernel, dim3(blocks_for(total)), dim3(256), 0, s, a_of(p.nblocks).t, ws.dpool, HWl,
                               total, dv.t);
    }
    for (int j = p.nblocks - 1; j >= 0; --j) {
        const ConvDesc &c1 = p.convs[1 + 2 * j], &c2 = p.convs[2 + 2 * j];
        // conv2: weight and bias gradient from dv and u; du = [u > 0] * dgrad(dv)
        if ((st = conv_weight_grad(ctx, c2, B, u_of(j), dv, G, ws.partials[2 + 2 * j], &pending)) != DPSGD_OK) return st;
        if ((st = conv_data_grad(ctx, c2, B, dv, X, ws.wpack_d[2 + 2 * j], none, u_of(j), du)) != DPSGD_OK) return st;
        // conv1: from du and a_j; next dv = [a_j > 0] * (dgrad(du) + shortcut delta)
        if ((st = conv_weight_grad(ctx, c1, B, a_of(j), du, G, ws.partials[1 + 2 * j], &pending)) != DPSGD_OK) return st;
        const ShortcutRef scd{dv.t, c2.Co, c2.Ho, c2.Wo, c1.stride};
        if ((st = conv_data_grad(ctx, c1, B, du, X, ws.wpack_d[1 + 2 * j], scd, a_of(j), dnext)) != DPSGD_OK) return st;
        Tensor t = dv; dv = dnext; dnext = t;
    }
    if (stem_mfma) {   // stem: weight and bias gradient only
        Tensor img;
        img.t = const_cast<bf16_t *>(image_chw);
        if ((st = conv_weight_grad(ctx, p.convs[0], B, img, dv, G, ws.partials[0], &pending)) != DPSGD_OK) return st;
    } else {
        const ConvDesc &c = p.convs[0];
        dim3 grid((unsigned)c.Ci, (unsigned)c.Co, (unsigned)n);
        if (m.input_is_bf16)
            hipLaunchKernelGGL(conv_wgrad_generic_kernel<false>, grid, dim3(256), 0, s, inputs, dv.t, c, B, G, ctx->ld);
        else
            hipLaunchKernelGGL(conv_wgrad_generic_kernel<true>, grid, dim3(256), 0, s, inputs, dv.t, c, B, G, ctx->ld);
        hipLaunchKernelGGL(sum_delta_kernel, dim3((unsigned)n), dim3(1024), 0, s, dv.t, (i64)B * c.Ho * c.Wo * c.Co, G,
                           ctx->ld, c.b_off);
    }
    if ((st = hip_status(hipGetLastError())) != DPSGD_OK) return st;
    return conv_weight_grad_finish(ctx, &pending, G);
}

// ---- shape-generic building blocks (used directly, and as the fallback of the MFMA dispatch)
dpsgd_status conv_forward_generic(dpsgd_ctx *ctx, const ConvDesc &c, int B, Tensor in, const float *X, ShortcutRef sc,
                                  Tensor out)
{
    const i64 total = (i64)ctx->n * B * c.Ho * c.Wo * c.Co;
    hipLaunchKernelGGL(conv_fwd_generic_kernel<false>, dim3(blocks_for(total)), dim3(256), 0, ctx->stream, in.t, X, ctx->ld,
                       c, B, total, sc.t, sc.C, sc.H, sc.W, sc.S, out.t);
    return hip_status(hipGetLastError());
}

dpsgd_status conv_data_grad_generic(dpsgd_ctx *ctx, const ConvDesc &c, int B, Tensor dout, const float *X,
                                    ShortcutRef scd, Tensor act, Tensor din)
{
    const i64 total = (i64)ctx->n * B * c.H * c.W * c.Ci;
    hipLaunchKernelGGL(conv_dgrad_generic_kernel, dim3(blocks_for(total)), dim3(256), 0, ctx->stream, dout.t, X, ctx->ld, c,
                       B, total, scd.t, scd.C, scd.H, scd.W, scd.S, act.t, din.t);
    return hip_status(hipGetLastError());
}

dpsgd_status conv_weight_grad_generic(dpsgd_ctx *ctx, const ConvDesc &c, int B, Tensor in, Tensor dout, float *G)
{
    dim3 grid((unsigned)c.Ci, (unsigned)c.Co, (unsigned)ctx->n);
    hipLaunchKernelGGL(conv_wgrad_generic_kernel<false>, grid, dim3(256), 0, ctx->stream, in.t, dout.t, c, B, G, ctx->ld);
    hipLaunchKernelGGL(sum_delta_kernel, dim3((unsigned)ctx->n), dim3(1024), 0, ctx->stream, dout.t,
                       (i64)B * c.Ho * c.Wo * c.Co, G, ctx->ld, c.b_off);
    return hip_status(hipGetLastError());
}

}  // namespace dpsgd

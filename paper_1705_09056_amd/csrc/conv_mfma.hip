// 3x3 convolutions of the CNN workload as implicit GEMMs on bf16 MFMA (gfx950), and their
// dispatch: MFMA kernels for channel counts 16/32/64 on images whose width is a multiple of 8,
// the shape-generic kernels otherwise.
//
// Forward and data gradient share one kernel: out(y,x,o) = sum_{tap,c} P(y*S+ky-1, x*S+kx-1, c) *
// Weff[o][c][tap], where P is the source tensor (zero outside; for the data gradient of a stride-2
// conv the delta with zeros inserted between its pixels) and Weff the conv's weights (for the data
// gradient: channels transposed, taps reversed).  Tensors are channel-major in memory; a workgroup
// owns TH = 8 or 16 output rows of one image (16 where the image has them and the patch fits: fewer halo rows
// are fetched twice and every channel plane is touched in runs twice as long, 3-15 % faster at 32 x 32 and
// 16 x 16 pixels; 32 rows leave too few workgroups per CU and are slower): it stages the (TH-1)*S+3 source rows with their halo in LDS
// pixel-major (the transposition happens on the way in: a thread fetches 8 pixels of two channels
// and writes 8 channel pairs; pixel pitch padded by 16 bytes so that 16 lanes reading 16 bytes each
// spread over all banks), keeps its slice of the packed weights in registers for the whole tile, and
// issues v_mfma_f32_16x16x32_bf16: A = 16 consecutive output pixels x 32 contraction values (8
// channels of one tap per lane, one 16-byte LDS read), B = 32 x 16 output channels.  Accumulator
// register i of lane l is (MFMA row 4*(l/16)+i, channel l%16); two tiles are taken together with
// their rows mapped to pixels so that a lane ends up with 8 consecutive pixels of one channel:
// 16-byte loads and stores in the epilogue.
#include "resnet_common.h"

namespace dpsgd {
namespace {

typedef long long i64;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int ksteps(int ci) { return (9 * ci + 31) / 32; }
// waves of a workgroup that split the output channels: as few as keep <= 18 weight fragments per lane
constexpr int wave_cols(int ci, int co)
{
    int wc = 1;
    while (ksteps(ci) * (co / 16) / wc > 18) wc *= 2;
    return wc;
}

// ------------------------------------------------------------------------- weight packing
// wpack[w][s][t][lane][j] = Weff[o = 16 t + lane%16][c][tap], contraction index 32 s + 8 (lane/16) + j
// = tap * CI + c (CI = contraction channels rounded up to 8); zero beyond tap 8 or channel c_real.
// DGRAD: Weff[o = c_in][c = c_out][tap] = W[c_out][c_in][8 - tap].
// One launch packs every conv of the network (both operands): the jobs travel in the kernel arguments.
struct PackJob {
    long long w_off;    // the conv's weights inside a worker's parameter vector
    bf16_t *dst;        // [n][per_worker]
    int Ci, Co;         // the conv's real channel counts
    int CI, CO, KS;     // contraction channels (padded), output channels, k-steps of the packed operand
    int dgrad;
    int block0;         // first blockIdx.x of this job
};
constexpr int kMaxPackJobs = 64;
struct PackTable {
    PackJob job[kMaxPackJobs];
    int njobs;
};

// A workgroup packs one tile of 16 outputs of one job and worker.  The fp32 weights it needs are runs of
// consecutive floats (forward: the 16 rows W[o][.][.], one run; data gradient: for every c_out the 16 x 9 floats
// W[c_out][ci0 .. ci0+15][.]): they are read coalesced, rounded to bf16 into LDS, and the operand is composed from
// LDS and written as 16-byte units.
constexpr int kPackLds = 64 * 16 * 9;   // bf16 elements: 16 outputs x 64 contraction channels x 9 taps

__global__ void __launch_bounds__(256) pack_weights_kernel(const float *__restrict__ X, i64 ld, PackTable tbl)
{
    __shared__ bf16_t tile[kPackLds];
    // Workgroups are dealt to the 8 XCDs round-robin by linear id and every XCD has its own L2: with n a multiple of 8
    // the ids are renumbered so that one XCD packs all tiles of a worker, and the weights, which the forward and the
    // data-gradient tile of a convolution both read, come from memory once instead of once per L2 that wants them.
    int bx = blockIdx.x, w = blockIdx.y;
    if ((gridDim.y & 7) == 0) {
        const unsigned id = blockIdx.x + gridDim.x * blockIdx.y;
        const unsigned xcd = id & 7, slot = id >> 3;
        w = (int)((slot / gridDim.x) * 8 + xcd);
        bx = (int)(slot % gridDim.x);
    }
    // the job of this workgroup: last one whose first block is <= bx (bisection over uniform values)
    int lo = 0, hi = tbl.njobs - 1;
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if (bx >= tbl.job[mid].block0) lo = mid; else hi = mid - 1;
    }
    const PackJob &jb = tbl.job[lo];
    const int t = bx - jb.block0, tid = threadIdx.x;
    const int NT = jb.CO / 16;
    const float *Wg = X + (i64)w * ld + jb.w_off;
    const int row9 = jb.Ci * 9;   // floats of one c_out row of W
    // rows x len floats, row r at Wg[base + r * row9]; in LDS row r at tile[r * len]
    int rows, len, base;
    if (!jb.dgrad) {   // outputs are c_out 16 t .. 16 t + 15: their rows are adjacent
        rows = jb.Co - 16 * t < 16 ? jb.Co - 16 * t : 16;
        len = row9;
        base = 16 * t * row9;
    } else {           // outputs are c_in 16 t .. 16 t + 15: 16 x 9 floats of every c_out row
        rows = jb.Co;
        len = (jb.Ci - 16 * t < 16 ? jb.Ci - 16 * t : 16) * 9;
        base = 16 * t * 9;
    }
    if (!jb.dgrad) {
        for (int e = tid; e < rows * len; e += 256) tile[e] = f2bf(Wg[base + e]);   // one run
    } else {
        for (int r = tid >> 6; r < rows; r += 4)
            for (int c = tid & 63; c < len; c += 64) tile[r * len + c] = f2bf(Wg[base + (i64)r * row9 + c]);
    }
    __syncthreads();
    const int lg = 31 - __builtin_clz(jb.CI);   // CI is 8, 16, 32 or 64
    const int groups = jb.KS * 64;   // 16-byte units of this tile
    bf16_t *dst = jb.dst + (i64)w * (jb.KS * NT * 512);
    for (int u = tid; u < groups; u += 256) {
        const int lane = u & 63, s = u >> 6, ol = lane & 15;
        unsigned short v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int kk = 32 * s + 8 * (lane >> 4) + j;
            const int tap = kk >> lg, ch = kk & (jb.CI - 1);
            v[j] = 0;
            if (tap < 9) {
                if (!jb.dgrad) {
                    if (ch < jb.Ci && ol < rows) v[j] = tile[ol * len + ch * 9 + tap];
                } else {
                    if (ch < jb.Co && ol * 9 < len) v[j] = tile[ch * len + ol * 9 + (8 - tap)];
                }
            }
        }
        const u32x4 pk = {v[0] | ((unsigned)v[1] << 16), v[2] | ((unsigned)v[3] << 16), v[4] | ((unsigned)v[5] << 16),
                          v[6] | ((unsigned)v[7] << 16)};
        *reinterpret_cast<u32x4 *>(dst + ((i64)(s * NT + t) * 64 + lane) * 8) = pk;
    }
}

// --------------------------------------------------------------- forward / data gradient
struct ConvMfmaArgs {
    const bf16_t *src;      // [n*B][CI][Hs][Ws]; CI == 8 (stem): the image, pixel-major [n*B][Hs][Ws][8]
    int Hs, Ws;
    const bf16_t *wpack;    // [n][KS][CO/16][64][8]
    bf16_t *dstT;           // [n*B][CO][Hd][Wd]
    int Hd, Wd, lw, B;      // lw = log2(Wd)
    const float *X;         // forward: scalar bias at X[w*ld + b_off]
    i64 ld, b_off;
    ShortcutRef sc;         // forward: block input; data gradient: delta of the block output
    const bf16_t *actT;     // data gradient: activation whose sign masks the result (shape of dst)
    const unsigned char *sign_in;   // data gradient: the same signs as a bitmap (1 bit per element), or null
    unsigned char *sign_out;        // forward: bitmap of the output's signs, or null
};

template <int CI, int CO, int STRIDE, int DILATE, bool DGRAD, int TH>
__global__ void __launch_bounds__(256) conv3x3_mfma_kernel(ConvMfmaArgs a)
{
    constexpr int KS = ksteps(CI), NT = CO / 16, WC = wave_cols(CI, CO), NTW = NT / WC, WP = 4 / WC;
    constexpr int PP = CI + 8;   // LDS pixel pitch (bf16 elements)
    static_assert(TH % 8 == 0, "a workgroup owns whole 8-row bands of the sign bitmap");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    bf16_t *patch = reinterpret_cast<bf16_t *>(smem);
    // Workgroups are dealt to the 8 XCDs round-robin by linear id and every XCD has its own L2: with n a multiple
    // of 8 the ids are renumbered so that all workgroups of a worker run on one XCD and its packed weights are
    // fetched into one L2 instead of eight.
    int band = blockIdx.x, b = blockIdx.y, w = blockIdx.z;
    if ((gridDim.z & 7) == 0) {
        const unsigned per = gridDim.x * gridDim.y;
        const unsigned id = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
        const unsigned xcd = id & 7, slot = id >> 3, within = slot % per;
        w = (int)((slot / per) * 8 + xcd);
        band = (int)(within % gridDim.x);
        b = (int)(within / gridDim.x);
    }
    const i64 img = (i64)w * a.B + b;
    const int y0 = band * TH;
    const int Wd = a.Wd, lw = a.lw;
    const int PR = (TH - 1) * STRIDE + 3, PC = (Wd - 1) * STRIDE + 3;
    unsigned char *sign_lds = smem + PR * PC * PP * (int)sizeof(bf16_t);   // forward: TH / 8 * CO * Wd bytes behind the patch
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wc = wave % WC, wp = wave / WC;
    const int n16 = lane & 15, g = lane >> 4;

    // stage the source rows (with halo, zeros outside / between dilated pixels)
    if (CI == 8) {   // pixel-major image: a wave per patch row, a lane per pixel (16 bytes)
        const bf16_t *src = a.src + img * a.Hs * a.Ws * CI;
        for (int pr = wave; pr < PR; pr += 4) {
            const int vr = y0 * STRIDE - 1 + pr;
            const bool row_ok = vr >= 0 && vr < a.Hs;
            for (int pc = lane; pc < PC; pc += 64) {
                const int vc = pc - 1;
                u32x4 v = {0u, 0u, 0u, 0u};
                if (row_ok && vc >= 0 && vc < a.Ws) v = *reinterpret_cast<const u32x4 *>(src + (vr * a.Ws + vc) * CI);
                *reinterpret_cast<u32x4 *>(patch + (pr * PC + pc) * PP) = v;
            }
        }
    } else {
        // channel-major source: a task = (channel pair j, patch row pr, 8 source pixels xc); the thread
        // fetches the 8 pixels of both channels (16 bytes each) and writes 8 channel pairs.  Consecutive threads take
        // consecutive pixel octets of one row of a channel pair, then the next pair: the rows of a channel plane lie
        // one after the other in memory, so a wave's loads fall into runs of 16 Ws bytes instead of 64 separate lines
        // (the LDS writes of two such threads then meet in a bank two at a time: 2.971 -> 2.951 ms per CNN iteration)
        constexpr int CP2 = CI / 2, FT = 4;   // FT tasks per thread are in flight at once
        const bf16_t *src = a.src + img * CI * a.Hs * a.Ws;
        const int x8n = a.Ws >> 3, plane = a.Hs * a.Ws;
        const int ntask = CP2 * x8n * PR;
        u32x4 fa[FT], fb[FT];
        auto decode = [&](int task, int &j, int &pr, int &xc, int &vr) {
            xc = task % x8n;
            const int rest = task / x8n;
            j = rest % CP2;
            pr = rest / CP2;
            vr = y0 * STRIDE - 1 + pr;
            bool ok = task < ntask && vr >= 0;
            if (DILATE == 2) {
                ok = ok && !(vr & 1);
                vr >>= 1;
            }
            return ok && vr < a.Hs;
        };
        auto issue = [&](int round) {
#pragma unroll
            for (int q = 0; q < FT; ++q) {
                int j, pr, xc, vr;
                fa[q] = (u32x4){0u, 0u, 0u, 0u};
                fb[q] = fa[q];
                if (decode(tid + 256 * (round * FT + q), j, pr, xc, vr)) {
                    const bf16_t *p = src + (2 * j) * plane + vr * a.Ws + 8 * xc;
                    fa[q] = *reinterpret_cast<const u32x4 *>(p);
                    fb[q] = *reinterpret_cast<const u32x4 *>(p + plane);
                }
            }
        };
        auto commit = [&](int round) {
#pragma unroll
            for (int q = 0; q < FT; ++q) {
                int j, pr, xc, vr;
                if (!decode(tid + 256 * (round * FT + q), j, pr, xc, vr)) continue;
                // source pixel 8 xc + i sits at patch column (8 xc + i) * DILATE + 1
                unsigned *dst = reinterpret_cast<unsigned *>(patch + (pr * PC + 8 * xc * DILATE + 1) * PP + 2 * j);
                constexpr int step = DILATE * PP / 2;   // dwords between consecutive source pixels
                const unsigned lo[4] = {fa[q].x, fa[q].y, fa[q].z, fa[q].w}, hi[4] = {fb[q].x, fb[q].y, fb[q].z, fb[q].w};
#pragma unroll
                for (int h = 0; h < 4; ++h) {
                    dst[(2 * h) * step] = (lo[h] & 0xffffu) | (hi[h] << 16);
                    dst[(2 * h + 1) * step] = (lo[h] >> 16) | (hi[h] & 0xffff0000u);
                }
            }
        };
        issue(0);
        const int units = PR * PC * PP / 8;   // zero everything a task will not write
        for (int u = tid; u < units; u += 256) *reinterpret_cast<u32x4 *>(patch + u * 8) = (u32x4){0u, 0u, 0u, 0u};
        __syncthreads();
        commit(0);
        for (int round = 1; round * FT * 256 < ntask; ++round) {
            issue(round);
            commit(round);
        }
    }

    // this wave's weight fragments
    bf16x8 wf[KS][NTW];
    {
        const bf16_t *wp_ = a.wpack + (i64)w * (KS * NT * 512) + lane * 8;
#pragma unroll
        for (int s = 0; s < KS; ++s)
#pragma unroll
            for (int t = 0; t < NTW; ++t)
                wf[s][t] = *reinterpret_cast<const bf16x8 *>(wp_ + (s * NT + wc * NTW + t) * 512);
    }
    // per k-step offset of this lane's 8 contraction values inside the patch (relative to the
    // pixel's top-left tap): the tap and the first channel follow from 32 s + 8 g
    int koff[KS];
#pragma unroll
    for (int s = 0; s < KS; ++s) {
        const int kk = 32 * s + 8 * g;
        int tap = kk / CI;
        const int c0 = kk % CI;
        tap = tap > 8 ? 8 : tap;   // padded taps carry zero weights; read finite data
        koff[s] = ((tap / 3) * PC + (tap % 3)) * PP + c0;
    }
    __syncthreads();

    const int npair = (TH << lw) >> 5;   // pairs of M tiles = groups of 32 consecutive pixels of the band
    float bias = 0.f;
    if (!DGRAD) bias = a.X[(i64)w * a.ld + a.b_off];
    // per-image bases; everything below is 32-bit offsets inside one image
    bf16_t *dstT = a.dstT + img * CO * a.Hd * Wd;
    const bf16_t *actT = DGRAD ? a.actT + img * CO * a.Hd * Wd : nullptr;
    // sign bitmaps are stored per band of 8 rows, [image][band of 8][channel][Wd bytes], so that a workgroup reads
    // or writes TH / 8 * CO * Wd consecutive bytes that no other workgroup shares a cache line with
    const i64 sign_base = (img * (a.Hd / 8) + band * (TH / 8)) * (CO * Wd);
    const int band_px = Wd << 3;   // pixels of one 8-row band
    const unsigned char *signi = (DGRAD && a.sign_in) ? a.sign_in + sign_base : nullptr;
    unsigned char *signo = (!DGRAD && a.sign_out) ? a.sign_out + sign_base : nullptr;
    const bf16_t *scT = a.sc.t ? a.sc.t + img * a.sc.C * a.sc.H * a.sc.W : nullptr;
    const int scS = a.sc.S;

    // A wave takes two M tiles at a time and maps MFMA row r of tile tt to pixel 8 (r / 4) + 4 tt + r % 4 of
    // the group: accumulator register i of lane (n16, g) is then pixel 8 g + 4 tt + i, so the lane owns 8
    // consecutive pixels of channel n16 = 16 contiguous bytes of every channel-major tensor it touches.
    for (int mp = wp; mp < npair; mp += WP) {
        const bf16_t *pa[2];
#pragma unroll
        for (int tt = 0; tt < 2; ++tt) {
            const int pi = mp * 32 + 8 * (n16 >> 2) + 4 * tt + (n16 & 3);   // this lane's pixel as an A-operand row
            const int py = pi >> lw, px = pi & (Wd - 1);
            pa[tt] = patch + ((py * STRIDE) * PC + px * STRIDE) * PP;
        }
        const int q0 = mp * 32 + 8 * g;                     // first of this lane's 8 output pixels (one row: Wd >= 8)
        const int y = y0 + (q0 >> lw), x0 = q0 & (Wd - 1);
        // fetch what the epilogue needs (shortcut values, activation signs) before the MFMAs, to hide their latency
        float e_sc[NTW][8];
        u32x4 e_act[NTW];
#pragma unroll
        for (int t = 0; t < NTW; ++t) {
            const int o = (wc * NTW + t) * 16 + n16;
#pragma unroll
            for (int i = 0; i < 8; ++i) e_sc[t][i] = 0.f;
            e_act[t] = (u32x4){0u, 0u, 0u, 0u};
            if (DGRAD) {   // the lane's 8 pixels are one byte of the bitmap
                if (signi) e_act[t].x = signi[((q0 >> (lw + 3)) * CO + o) * Wd + ((q0 & (band_px - 1)) >> 3)];
                else e_act[t] = *reinterpret_cast<const u32x4 *>(actT + (o * a.Hd + y) * Wd + x0);
            }
            if (scT && o < a.sc.C) {
                if (scS == 1) {
                    const u32x4 v = *reinterpret_cast<const u32x4 *>(scT + (o * a.sc.H + y) * a.sc.W + x0);
                    const unsigned d[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                    for (int h = 0; h < 4; ++h) {
                        e_sc[t][2 * h] = bf2f((bf16_t)(d[h] & 0xffff));
                        e_sc[t][2 * h + 1] = bf2f((bf16_t)(d[h] >> 16));
                    }
                } else if (!DGRAD) {   // block input at (2y, 2x): every second of 16 consecutive pixels
                    const bf16_t *sp = scT + (o * a.sc.H + 2 * y) * a.sc.W + 2 * x0;
                    const u32x4 v0 = *reinterpret_cast<const u32x4 *>(sp), v1 = *reinterpret_cast<const u32x4 *>(sp + 8);
                    const unsigned d[8] = {v0.x, v0.y, v0.z, v0.w, v1.x, v1.y, v1.z, v1.w};
#pragma unroll
                    for (int i = 0; i < 8; ++i) e_sc[t][i] = bf2f((bf16_t)(d[i] & 0xffff));
                } else if (!(y & 1)) {   // delta of the block output lands on even pixels only
                    const u32x2 v = *reinterpret_cast<const u32x2 *>(scT + (o * a.sc.H + (y >> 1)) * a.sc.W + (x0 >> 1));
                    e_sc[t][0] = bf2f((bf16_t)(v.x & 0xffff));
                    e_sc[t][2] = bf2f((bf16_t)(v.x >> 16));
                    e_sc[t][4] = bf2f((bf16_t)(v.y & 0xffff));
                    e_sc[t][6] = bf2f((bf16_t)(v.y >> 16));
                }
            }
        }
        f32x4 acc[2][NTW];
#pragma unroll
        for (int tt = 0; tt < 2; ++tt)
#pragma unroll
            for (int t = 0; t < NTW; ++t) acc[tt][t] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < KS; ++s) {
#pragma unroll
            for (int tt = 0; tt < 2; ++tt) {
                const bf16x8 av = *reinterpret_cast<const bf16x8 *>(pa[tt] + koff[s]);
#pragma unroll
                for (int t = 0; t < NTW; ++t)
                    acc[tt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, wf[s][t], acc[tt][t], 0, 0, 0);
            }
        }
#pragma unroll
        for (int t = 0; t < NTW; ++t) {
            const int o = (wc * NTW + t) * 16 + n16;
            const unsigned ad[4] = {e_act[t].x, e_act[t].y, e_act[t].z, e_act[t].w};
            float r[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                float v = acc[i >> 2][t][i & 3] + e_sc[t][i];
                if (!DGRAD) {
                    v += bias;
                    v = v > 0.f ? v : 0.f;
                } else {
                    const bf16_t am = (bf16_t)((i & 1) ? (ad[i >> 1] >> 16) : (ad[i >> 1] & 0xffff));
                    const bool pos = signi ? ((ad[0] >> i) & 1u) != 0 : bf16_positive(am);
                    v = pos ? v : 0.f;
                }
                r[i] = v;
            }
            const u32x4 pk = {f2bf_pack(r[0], r[1]), f2bf_pack(r[2], r[3]), f2bf_pack(r[4], r[5]), f2bf_pack(r[6], r[7])};
            *reinterpret_cast<u32x4 *>(dstT + ((o * a.Hd + y) << lw) + x0) = pk;
            if (!DGRAD && signo) {
                // from the stored bf16 values, so that both masks agree bit for bit; after the ReLU a value is
                // positive exactly when its bf16 pattern is not zero
                const unsigned pw[4] = {pk.x, pk.y, pk.z, pk.w};
                unsigned bits = 0;
#pragma unroll
                for (int h = 0; h < 4; ++h) {
                    bits |= (pw[h] & 0xffffu) ? (1u << (2 * h)) : 0u;
                    bits |= (pw[h] >> 16) ? (2u << (2 * h)) : 0u;
                }
                sign_lds[((q0 >> (lw + 3)) * CO + o) * Wd + ((q0 & (band_px - 1)) >> 3)] = (unsigned char)bits;
            }
        }
    }
    if (!DGRAD && signo) {   // the bands' bitmap (TH / 8 * CO * Wd bytes) leaves as 16-byte units: a few requests per workgroup
        __syncthreads();
        for (int u = tid; u < (TH / 8) * CO * Wd / 16; u += 256)
            *reinterpret_cast<u32x4 *>(signo + 16 * u) = *reinterpret_cast<const u32x4 *>(sign_lds + 16 * u);
    }
}

// ------------------------------------------------- a residual block's two forward convolutions in one launch
// out = ReLU(conv2(u) + b2 + in), u = ReLU(conv1(in) + b1), both 3 x 3, stride 1, C channels in and out (the blocks
// that keep the resolution).  Launched separately, conv2 reads u back from memory right after conv1 wrote it; here the
// workgroup that owns TH output rows of one image computes the TH + 2 rows of u its second convolution needs (one halo
// row above and below, recomputed by the neighbouring band) from a source patch of TH + 4 rows, keeps them in LDS
// pixel-major - rows outside the image as the zeros conv2's padding means - and multiplies again.  u still goes to
// memory once (the backward pass needs it), with its sign bitmap; what is saved is reading it back.  The same matrix
// instructions on the same operands in the same order as conv3x3_mfma_kernel, so u and out carry the same bits.
// C = 16 or 32 (every wave keeps all C / 16 output tiles) or 64 (a wave keeps one tile of 16 output channels and takes
// all pixels); (TH + 2) W a multiple of 32, or the band the whole image and TH W a multiple of 32.
// grid (H / TH, B, n), block 256, dynamic LDS: the source patch (u takes its place later) and one band's sign bitmap.
struct ConvBlockArgs {
    const bf16_t *src;               // block input [n*B][C][H][W]
    const bf16_t *wpack1, *wpack2;   // [n][KS][C/16][64][8]
    bf16_t *uT, *yT;                 // [n*B][C][H][W]
    unsigned char *usign, *ysign;    // sign bitmaps of u and of the block output
    int H, W, lw, B;
    const float *X;
    i64 ld, b_off1, b_off2;
};

template <int C, int TH, int WMAX>   // WMAX: the widest image a launch may have (sizes the registers u waits in)
__global__ void __launch_bounds__(256, C == 16 ? 7 : 1) conv_block_fwd_kernel(ConvBlockArgs a)   // 16 channels: the LDS lets 7 workgroups share a CU
{
    constexpr int KS = ksteps(C), NT = C / 16, PP = C + 8;
    // waves that split the output channels (64 channels: one tile of 16 each), and those that split the pixels
    constexpr int WC = wave_cols(C, C), NTW = NT / WC, WP = 4 / WC;
    constexpr int PRX = TH + 4, PRU = TH + 2;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    int band = blockIdx.x, b = blockIdx.y, w = blockIdx.z;
    if ((gridDim.z & 7) == 0) {   // all workgroups of a worker on one XCD (see conv3x3_mfma_kernel)
        const unsigned per = gridDim.x * gridDim.y;
        const unsigned id = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
        const unsigned xcd = id & 7, slot = id >> 3, within = slot % per;
        w = (int)((slot / per) * 8 + xcd);
        band = (int)(within % gridDim.x);
        b = (int)(within / gridDim.x);
    }
    const i64 img = (i64)w * a.B + b;
    const int y0 = band * TH, W = a.W, H = a.H, lw = a.lw;
    const int PCX = W + 4, PCU = W + 2;
    bf16_t *xpatch = reinterpret_cast<bf16_t *>(smem);     // [PRX][PCX][PP]: image rows y0 - 2 .., columns -2 ..
    // u takes the source patch's place once conv1 has read it (its values wait in registers across one barrier):
    // 21 KB instead of 37 KB of LDS at 16 channels x 32 pixels, seven workgroups per CU instead of four
    bf16_t *upatch = xpatch;                               // [PRU][PCU][PP]: image rows y0 - 1 .., columns -1 ..
    unsigned char *sign_lds = reinterpret_cast<unsigned char *>(xpatch + PRX * PCX * PP);   // TH / 8 * C * W bytes
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n16 = lane & 15, g = lane >> 4;
    const int wc = wave % WC, wp = wave / WC;
    // a band that is the whole image: the halo rows of u lie outside it, so conv1 multiplies the image's rows only
    const bool whole = H == TH;
    const int first = whole ? W : 0, npair1 = ((whole ? TH : PRU) << lw) >> 5;   // conv1's first pixel and pairs of tiles

    {   // stage the source rows: a task = (channel pair j, patch row pr, 8 source pixels xc), pixel octets fastest
        constexpr int CP2 = C / 2, FT = 4;
        const bf16_t *src = a.src + img * C * H * W;
        const int x8n = W >> 3, plane = H * W;
        const int ntask = CP2 * x8n * PRX;
        u32x4 fa[FT], fb[FT];
        auto decode = [&](int task, int &j, int &pr, int &xc, int &vr) {
            xc = task % x8n;
            const int rest = task / x8n;
            j = rest % CP2;
            pr = rest / CP2;
            vr = y0 - 2 + pr;
            return task < ntask && vr >= 0 && vr < H;
        };
        auto issue = [&](int round) {
#pragma unroll
            for (int q = 0; q < FT; ++q) {
                int j, pr, xc, vr;
                fa[q] = (u32x4){0u, 0u, 0u, 0u};
                fb[q] = fa[q];
                if (decode(tid + 256 * (round * FT + q), j, pr, xc, vr)) {
                    const bf16_t *p = src + (2 * j) * plane + vr * W + 8 * xc;
                    fa[q] = *reinterpret_cast<const u32x4 *>(p);
                    fb[q] = *reinterpret_cast<const u32x4 *>(p + plane);
                }
            }
        };
        auto commit = [&](int round) {
#pragma unroll
            for (int q = 0; q < FT; ++q) {
                int j, pr, xc, vr;
                if (!decode(tid + 256 * (round * FT + q), j, pr, xc, vr)) continue;
                unsigned *dst = reinterpret_cast<unsigned *>(xpatch + (pr * PCX + 8 * xc + 2) * PP + 2 * j);
                constexpr int step = PP / 2;   // dwords between consecutive pixels
                const unsigned lo[4] = {fa[q].x, fa[q].y, fa[q].z, fa[q].w}, hi[4] = {fb[q].x, fb[q].y, fb[q].z, fb[q].w};
#pragma unroll
                for (int h = 0; h < 4; ++h) {
                    dst[(2 * h) * step] = (lo[h] & 0xffffu) | (hi[h] << 16);
                    dst[(2 * h + 1) * step] = (lo[h] >> 16) | (hi[h] & 0xffff0000u);
                }
            }
        };
        issue(0);
        const int units = PRX * PCX * PP / 8;   // the patch starts as zeros
        for (int u = tid; u < units; u += 256) *reinterpret_cast<u32x4 *>(xpatch + u * 8) = (u32x4){0u, 0u, 0u, 0u};
        __syncthreads();
        commit(0);
        for (int round = 1; round * FT * 256 < ntask; ++round) {
            issue(round);
            commit(round);
        }
    }

    bf16x8 wf[KS][NTW];
    int koff[KS];
    auto load_weights = [&](const bf16_t *wpack, int PC) {
        const bf16_t *wp_ = wpack + (i64)w * (KS * NT * 512) + lane * 8;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
#pragma unroll
            for (int t = 0; t < NTW; ++t) wf[s][t] = *reinterpret_cast<const bf16x8 *>(wp_ + (s * NT + wc * NTW + t) * 512);
            const int kk = 32 * s + 8 * g;
            int tap = kk / C;
            const int c0 = kk % C;
            tap = tap > 8 ? 8 : tap;   // padded taps carry zero weights; read finite data
            koff[s] = ((tap / 3) * PC + (tap % 3)) * PP + c0;
        }
    };
    // MFMA row r of tile tt is pixel 8 (r / 4) + 4 tt + r % 4 of a group of 32 (see conv3x3_mfma_kernel): accumulator
    // register i of lane (n16, g) is pixel 8 g + 4 tt + i of channel 16 (wc NTW + t) + n16
    auto multiply = [&](const bf16_t *const (&pa)[2], f32x4 (&acc)[2][NTW]) {
#pragma unroll
        for (int tt = 0; tt < 2; ++tt)
#pragma unroll
            for (int t = 0; t < NTW; ++t) acc[tt][t] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < KS; ++s) {
#pragma unroll
            for (int tt = 0; tt < 2; ++tt) {
                const bf16x8 av = *reinterpret_cast<const bf16x8 *>(pa[tt] + koff[s]);
#pragma unroll
                for (int t = 0; t < NTW; ++t)
                    acc[tt][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(av, wf[s][t], acc[tt][t], 0, 0, 0);
            }
        }
    };
    const int band_px = W << 3;   // pixels of one 8-row band of the sign bitmap
    const i64 sign_base = (img * (H / 8) + band * (TH / 8)) * (C * W);
    auto sign_bits = [](const u32x4 &pk) {   // after the ReLU a value is positive exactly when its bf16 pattern is not zero
        const unsigned pw[4] = {pk.x, pk.y, pk.z, pk.w};
        unsigned bits = 0;
#pragma unroll
        for (int h = 0; h < 4; ++h) {
            bits |= (pw[h] & 0xffffu) ? (1u << (2 * h)) : 0u;
            bits |= (pw[h] >> 16) ? (2u << (2 * h)) : 0u;
        }
        return (unsigned char)bits;
    };
    auto flush_signs = [&](unsigned char *dst) {   // the band's bitmap leaves as 16-byte units
        __syncthreads();
        for (int u = tid; u < (TH / 8) * C * W / 16; u += 256)
            *reinterpret_cast<u32x4 *>(dst + sign_base + 16 * u) = *reinterpret_cast<const u32x4 *>(sign_lds + 16 * u);
    };

    // ---- u = ReLU(conv1(in) + b1) on rows y0 - 1 .. y0 + TH
    load_weights(a.wpack1, PCX);
    __syncthreads();
    constexpr int MAXP = ((TH + 2) * WMAX / 32 + WP - 1) / WP;   // pairs of MFMA tiles per wave at the widest image
    u32x4 stash[MAXP][NTW];                              // u as conv1 leaves it, until the source patch is free
    {
        const float bias = a.X[(i64)w * a.ld + a.b_off1];
        bf16_t *uT = a.uT + img * C * H * W;
#pragma unroll
        for (int it = 0; it < MAXP; ++it) {
            const int mp = wp + WP * it;
            if (mp >= npair1) break;
            const bf16_t *pa[2];
#pragma unroll
            for (int tt = 0; tt < 2; ++tt) {
                const int pi = first + mp * 32 + 8 * (n16 >> 2) + 4 * tt + (n16 & 3);
                pa[tt] = xpatch + ((pi >> lw) * PCX + (pi & (W - 1)) + 1) * PP;
            }
            const int q0 = first + mp * 32 + 8 * g;   // first of this lane's 8 pixels (one row: W >= 8)
            const int uy = q0 >> lw, x0 = q0 & (W - 1), iy = y0 - 1 + uy;
            const bool inside = iy >= 0 && iy < H, own = uy >= 1 && uy <= TH;
            f32x4 acc[2][NTW];
            multiply(pa, acc);
#pragma unroll
            for (int t = 0; t < NTW; ++t) {
                const int o = (wc * NTW + t) * 16 + n16;
                float r[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    float v = acc[i >> 2][t][i & 3] + bias;
                    r[i] = v > 0.f ? v : 0.f;
                }
                u32x4 pk = {f2bf_pack(r[0], r[1]), f2bf_pack(r[2], r[3]), f2bf_pack(r[4], r[5]), f2bf_pack(r[6], r[7])};
                if (!inside) pk = (u32x4){0u, 0u, 0u, 0u};   // a row outside the image is conv2's zero padding
                stash[it][t] = pk;
                if (own) {
                    *reinterpret_cast<u32x4 *>(uT + ((o * H + iy) << lw) + x0) = pk;
                    const int q = q0 - W;   // pixel index inside the band's own rows
                    sign_lds[((q >> (lw + 3)) * C + o) * W + ((q & (band_px - 1)) >> 3)] = sign_bits(pk);
                }
            }
        }
    }
    __syncthreads();   // every wave has read the source patch: u may take its place
    {
#pragma unroll
        for (int it = 0; it < MAXP; ++it) {
            const int mp = wp + WP * it;
            if (mp >= npair1) break;
            const int q0 = first + mp * 32 + 8 * g;
            const int uy = q0 >> lw, x0 = q0 & (W - 1);
#pragma unroll
            for (int t = 0; t < NTW; ++t) {
                const unsigned pw[4] = {stash[it][t].x, stash[it][t].y, stash[it][t].z, stash[it][t].w};
                bf16_t *up = upatch + (uy * PCU + x0 + 1) * PP + (wc * NTW + t) * 16 + n16;
#pragma unroll
                for (int h = 0; h < 4; ++h) {
                    up[(2 * h) * PP] = (bf16_t)(pw[h] & 0xffffu);
                    up[(2 * h + 1) * PP] = (bf16_t)(pw[h] >> 16);
                }
            }
        }
        // the columns left and right of the image
        for (int e = tid; e < PRU * 2 * (C / 8); e += 256) {
            const int c8 = e % (C / 8), side = (e / (C / 8)) & 1, row = e / (2 * (C / 8));
            *reinterpret_cast<u32x4 *>(upatch + (row * PCU + (side ? W + 1 : 0)) * PP + 8 * c8) = (u32x4){0u, 0u, 0u, 0u};
        }
        if (whole) {   // the rows above and below the image, which conv1 skipped
            const int row_units = PCU * PP / 8;
            for (int e = tid; e < 2 * row_units; e += 256)
                *reinterpret_cast<u32x4 *>(upatch + ((e < row_units ? 0 : PRU - 1) * PCU * PP) + (e % row_units) * 8) =
                    (u32x4){0u, 0u, 0u, 0u};
        }
    }
    // the block input at the wave's output pixels, which conv2's epilogue adds, is requested here (u has left its
    // registers): it arrives while the bitmap leaves and the second weight set is fetched, instead of costing every
    // pair of tiles an exposed latency
    constexpr int MAXP2 = (TH * WMAX / 32 + WP - 1) / WP;
    const int npair = (TH << lw) >> 5;
    u32x4 scv[MAXP2][NTW];
    {
        const bf16_t *scT = a.src + img * C * H * W;
#pragma unroll
        for (int it = 0; it < MAXP2; ++it) {
            const int mp = wp + WP * it;
            const int q0 = mp * 32 + 8 * g;
            const int y = y0 + (q0 >> lw), x0 = q0 & (W - 1);
#pragma unroll
            for (int t = 0; t < NTW; ++t) {
                scv[it][t] = (u32x4){0u, 0u, 0u, 0u};
                if (mp < npair)
                    scv[it][t] = *reinterpret_cast<const u32x4 *>(scT + ((((wc * NTW + t) * 16 + n16) * H + y) << lw) + x0);
            }
        }
    }
    flush_signs(a.usign);   // (its barrier also completes the u patch)

    // ---- out = ReLU(conv2(u) + b2 + in)
    load_weights(a.wpack2, PCU);
    __syncthreads();        // the bitmap buffer is free again
    {
        const float bias = a.X[(i64)w * a.ld + a.b_off2];
        bf16_t *yT = a.yT + img * C * H * W;
#pragma unroll
        for (int it = 0; it < MAXP2; ++it) {
            const int mp = wp + WP * it;
            if (mp >= npair) break;
            const bf16_t *pa[2];
#pragma unroll
            for (int tt = 0; tt < 2; ++tt) {
                const int pi = mp * 32 + 8 * (n16 >> 2) + 4 * tt + (n16 & 3);
                pa[tt] = upatch + ((pi >> lw) * PCU + (pi & (W - 1))) * PP;
            }
            const int q0 = mp * 32 + 8 * g;
            const int y = y0 + (q0 >> lw), x0 = q0 & (W - 1);
            f32x4 acc[2][NTW];
            multiply(pa, acc);
#pragma unroll
            for (int t = 0; t < NTW; ++t) {
                const int o = (wc * NTW + t) * 16 + n16;
                const unsigned d[4] = {scv[it][t].x, scv[it][t].y, scv[it][t].z, scv[it][t].w};
                float r[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const float e = bf2f((bf16_t)((i & 1) ? (d[i >> 1] >> 16) : (d[i >> 1] & 0xffffu)));
                    float v = acc[i >> 2][t][i & 3] + e;
                    v += bias;
                    r[i] = v > 0.f ? v : 0.f;
                }
                const u32x4 pk = {f2bf_pack(r[0], r[1]), f2bf_pack(r[2], r[3]), f2bf_pack(r[4], r[5]), f2bf_pack(r[6], r[7])};
                *reinterpret_cast<u32x4 *>(yT + ((o * H + y) << lw) + x0) = pk;
                sign_lds[((q0 >> (lw + 3)) * C + o) * W + ((q0 & (band_px - 1)) >> 3)] = sign_bits(pk);
            }
        }
    }
    flush_signs(a.ysign);
}

bool pow2_channels(int c) { return c == 16 || c == 32 || c == 64; }
int ilog2(int v) { int l = 0; while ((1 << l) < v) ++l; return l; }

// ----------------------------------------------------------------------- weight gradient
// dW[co][ci][tap] = sum over pixels of dout[pixel][co] * in[pixel shifted by tap][ci]: for each tap a
// 16x16 (co x ci) MFMA tile whose contraction runs over 32 consecutive output pixels, so both
// operands come from the channel-major copies: A = 8 consecutive pixels of one delta channel
// (16-byte global load), B = 8 consecutive pixels of one input channel shifted by the tap.  The
// workgroup stages the input rows of an 8-row band in LDS as [ci][row][8 zeros | W | 8 zeros]; the
// kx = 0 / 2 operands are the aligned 16-byte read funnel-shifted by one element with the
// neighbouring dword.  Waves split the output-channel tiles first, then the pixels; a workgroup
// owns a strided subset of the worker's images and writes its partial sums, which
// wgrad_reduce_kernel adds in a fixed order.
struct WgradReduceJob {
    const float *part;     // the conv's partial sums, [n][splits][psz]
    i64 w_off, b_off;      // where the conv's weights and its scalar bias sit in a worker's parameter vector
    int splits, psz, tiles, ci_tiles, CIr;
    int block0;            // first blockIdx.x of this job
};
constexpr int kMaxReduceJobs = 48;
struct WgradReduceTable {
    WgradReduceJob job[kMaxReduceJobs];
    int njobs;
};
static_assert(sizeof(WgradReduceTable) <= sizeof(WgradReduceList::table), "the caller's storage holds the job table");

struct WgradMfmaArgs {
    const bf16_t *inT;     // [n*B][CIr][H][W]
    const bf16_t *doutT;   // [n*B][CO][Ho][Wo]
    int H, W, Ho, Wo, B, CIr, splits;
    float *part;           // [n][splits][(CO/16)*(CI/16)*9*256 + 1], accumulator order
};

// 16-byte units of a band's source rows a thread holds while they are in flight (8-row bands: 10 rows at stride 1,
// 17 at stride 2; 16-row bands, stride 1 only: 18 rows)
__host__ __device__ constexpr int wgrad_stage(int stride, int rb) { return rb == 16 ? 5 : stride == 1 ? 3 : 5; }

__host__ __device__ constexpr int wgrad_channel_pitch(int plane) { return (plane + 119) / 128 * 128 + 8; }

// k-steps whose delta operands a wave requests at once (16 bytes per lane each); two where four workgroups share a CU
// and leave a wave 128 registers (that is a whole band at 16 channels: 8 k-steps over 4 waves, or 4 over 2)
__host__ __device__ constexpr int wgrad_delta_ahead(int ci) { return ci <= 16 ? 2 : 4; }

// With 64 x 64 channels a wave that kept all four input-channel tiles would need 144 accumulator
// registers (one wave per SIMD); two groups of four waves split them instead.
constexpr int wgrad_wave_groups(int ci, int co) { return (ci >= 64 && co >= 64) ? 2 : 1; }

// RB: output rows per band, 8 or 16.  Every band costs a workgroup two barriers and the wait for what it requested a
// band earlier (the source rows and the delta operands, both in flight across the barriers); 16-row bands halve their
// number where the image has them.
template <int CI, int CO, int STRIDE, int RB>
__global__ void __launch_bounds__(256 * wgrad_wave_groups(CI, CO), (CI <= 16 ? 4 : 2)) conv_wgrad_mfma_kernel(WgradMfmaArgs a)
{
    constexpr int WM = (CO / 16) < 4 ? (CO / 16) : 4, WK = 4 / WM;
    constexpr int WT = wgrad_wave_groups(CI, CO), NTI = CI / 16 / WT, NT = 256 * WT;
    constexpr int kWgradStage = wgrad_stage(STRIDE, RB), kWgradDeltaAhead = wgrad_delta_ahead(CI);
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    bf16_t *band = reinterpret_cast<bf16_t *>(smem);   // [CI] planes of CP elements, each [ROWS][PLANES][WPAD]
    const int sp = blockIdx.x, w = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = (tid >> 6) & 3, th = tid >> 8;
    const int mi = wave % WM, kq = wave / WM;   // output-channel tile, share of the k-steps
    const int t0 = th * NTI;                    // first input-channel tile of this wave
    const int n16 = lane & 15, g = lane >> 4;
    // stride 1: one plane per (channel, row), [8 zeros | W | 8 zeros].  stride 2: two planes, the even
    // and the odd input columns (an output pixel x reads columns 2x-1, 2x, 2x+1 = odd[x-1], even[x], odd[x]).
    constexpr int PLANES = STRIDE;
    const int WPAD = a.Wo + 16, ROWS = (RB - 1) * STRIDE + 3;
    // channel pitch = 8 elements (16 bytes) past a multiple of 256 bytes: the 16 lanes of an operand read
    // (16 channels, 16 bytes each) then fall into 16 different groups of 4 banks
    const int CP = wgrad_channel_pitch(ROWS * PLANES * WPAD);
    // a partial result in accumulator order: [co tile][ci tile][tap][lane][4] floats, then the bias sum
    constexpr int psz = (CO / 16) * (CI / 16) * 9 * 256 + 1;

    f32x4 acc[NTI][9];
#pragma unroll
    for (int t = 0; t < NTI; ++t)
#pragma unroll
        for (int k = 0; k < 9; ++k) acc[t][k] = (f32x4){0.f, 0.f, 0.f, 0.f};
    float bsum = 0.f;

    // zero the column pads once; staging never writes them
    for (int u = tid; u < CI * ROWS * PLANES * 2; u += NT) {
        const int side = u & 1, row = (u >> 1) % (ROWS * PLANES), ci = (u >> 1) / (ROWS * PLANES);
        u32x4 z = {0u, 0u, 0u, 0u};
        *reinterpret_cast<u32x4 *>(band + ci * CP + row * WPAD + (side ? 8 + a.Wo : 0)) = z;
    }

    const int x8n = a.W / 8;
    const int kb = RB * a.Wo / 32;   // k-steps per band
    // The bands (8 output rows of one image) this workgroup handles, in order; the source rows of band
    // j+1 are fetched into registers while band j is multiplied.
    const int bands_per_img = a.Ho / RB;
    const int nb = ((a.B - sp + a.splits - 1) / a.splits) * bands_per_img;
    const int chunks = CI * ROWS * x8n;   // 16-byte units of a band's source rows, <= kWgradStage * 256
    u32x4 stg[kWgradStage];
    auto fetch_band = [&](int j) {
        const i64 img = (i64)w * a.B + sp + (j / bands_per_img) * a.splits;
        const int y0 = (j % bands_per_img) * RB;
#pragma unroll
        for (int q = 0; q < kWgradStage; ++q) {
            const int u = tid + NT * q;
            const int x8 = u % x8n, r = (u / x8n) % ROWS, ci = u / (x8n * ROWS);
            const int iy = y0 * STRIDE - 1 + r;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (u < chunks && ci < a.CIr && iy >= 0 && iy < a.H)
                v = *reinterpret_cast<const u32x4 *>(a.inT + ((img * a.CIr + ci) * a.H + iy) * a.W + x8 * 8);
            stg[q] = v;
        }
    };
    // The delta operands of kWgradDeltaAhead k-steps of a wave (a whole band's at 16-64 channels on 32-8 pixel rows) are
    // requested together - a k-step is 9 short matrix instructions, far less than a memory latency - and a group
    // ahead: the next band's first group goes out right after this band's last multiply, so it is in flight across the
    // two barriers and the staging writes of the next band instead of being waited for after them.
    u32x4 dv[kWgradDeltaAhead];
    auto request_delta = [&](int j, int ks0) {
        const i64 img = (i64)w * a.B + sp + (j / bands_per_img) * a.splits;
        const int y0 = (j % bands_per_img) * RB;
        // this lane's 8 delta pixels of k-step ks: pixels 32 ks + 8 g .. + 7 of the band (rows are contiguous)
        const bf16_t *dband = a.doutT + ((img * CO + mi * 16 + n16) * a.Ho + y0) * a.Wo + 8 * g;
#pragma unroll
        for (int e = 0; e < kWgradDeltaAhead; ++e) {
            dv[e] = (u32x4){0u, 0u, 0u, 0u};
            if (ks0 + WK * e < kb) dv[e] = *reinterpret_cast<const u32x4 *>(dband + 32 * (ks0 + WK * e));
        }
    };
    if (nb > 0) {
        fetch_band(0);
        request_delta(0, kq);
    }
    for (int j = 0; j < nb; ++j) {
        {
            __syncthreads();   // previous band fully consumed
#pragma unroll
            for (int q = 0; q < kWgradStage; ++q) {
                const int u = tid + NT * q;
                if (u >= chunks) break;
                const int x8 = u % x8n, r = (u / x8n) % ROWS, ci = u / (x8n * ROWS);
                const u32x4 v = stg[q];
                if (STRIDE == 1) {
                    *reinterpret_cast<u32x4 *>(band + ci * CP + r * WPAD + 8 + x8 * 8) = v;
                } else {
                    const u32x2 ev = {(v.x & 0xffffu) | (v.y << 16), (v.z & 0xffffu) | (v.w << 16)};
                    const u32x2 od = {(v.x >> 16) | (v.y & 0xffff0000u), (v.z >> 16) | (v.w & 0xffff0000u)};
                    bf16_t *base = band + ci * CP + (r * 2) * WPAD + 8 + x8 * 4;
                    *reinterpret_cast<u32x2 *>(base) = ev;
                    *reinterpret_cast<u32x2 *>(base + WPAD) = od;
                }
            }
            if (j + 1 < nb) fetch_band(j + 1);   // (its registers are free: in flight while the waves meet at the barrier)
            __syncthreads();
            for (int ks0 = kq; ks0 < kb; ks0 += WK * kWgradDeltaAhead) {
#pragma unroll
            for (int e = 0; e < kWgradDeltaAhead; ++e) {
                const int ks = ks0 + WK * e;
                if (ks >= kb) break;
                const int q = 32 * ks + 8 * g;          // first of this lane's 8 pixels inside the band
                const int yy = q / a.Wo, x = q % a.Wo;
                const u32x4 av = dv[e];
                if (th == 0)
                    bsum += (bf2f((bf16_t)(av.x & 0xffff)) + bf2f((bf16_t)(av.x >> 16))) +
                            (bf2f((bf16_t)(av.y & 0xffff)) + bf2f((bf16_t)(av.y >> 16))) +
                            (bf2f((bf16_t)(av.z & 0xffff)) + bf2f((bf16_t)(av.z >> 16))) +
                            (bf2f((bf16_t)(av.w & 0xffff)) + bf2f((bf16_t)(av.w >> 16)));
                const bf16x8 afrag = __builtin_bit_cast(bf16x8, av);
#pragma unroll
                for (int t = 0; t < NTI; ++t) {
#pragma unroll
                    for (int ky = 0; ky < 3; ++ky) {
                        u32x4 l, d, r;   // the operand for kx = 0, 1, 2
                        if (STRIDE == 1) {
                            const bf16_t *row = band + ((t0 + t) * 16 + n16) * CP + (yy + ky) * WPAD + 8 + x;
                            d = *reinterpret_cast<const u32x4 *>(row);
                            const unsigned prev = *reinterpret_cast<const unsigned *>(row - 2);
                            const unsigned next = *reinterpret_cast<const unsigned *>(row + 8);
                            l.x = __builtin_amdgcn_alignbit(d.x, prev, 16);
                            l.y = __builtin_amdgcn_alignbit(d.y, d.x, 16);
                            l.z = __builtin_amdgcn_alignbit(d.z, d.y, 16);
                            l.w = __builtin_amdgcn_alignbit(d.w, d.z, 16);
                            r.x = l.y;
                            r.y = l.z;
                            r.z = l.w;
                            r.w = __builtin_amdgcn_alignbit(next, d.w, 16);
                        } else {
                            const bf16_t *even = band + ((t0 + t) * 16 + n16) * CP + ((2 * yy + ky) * 2) * WPAD + 8 + x;
                            const bf16_t *odd = even + WPAD;
                            d = *reinterpret_cast<const u32x4 *>(even);
                            r = *reinterpret_cast<const u32x4 *>(odd);
                            const unsigned prev = *reinterpret_cast<const unsigned *>(odd - 2);
                            l.x = __builtin_amdgcn_alignbit(r.x, prev, 16);
                            l.y = __builtin_amdgcn_alignbit(r.y, r.x, 16);
                            l.z = __builtin_amdgcn_alignbit(r.z, r.y, 16);
                            l.w = __builtin_amdgcn_alignbit(r.w, r.z, 16);
                        }
                        acc[t][ky * 3 + 0] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(afrag, __builtin_bit_cast(bf16x8, l),
                                                                                     acc[t][ky * 3 + 0], 0, 0, 0);
                        acc[t][ky * 3 + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(afrag, __builtin_bit_cast(bf16x8, d),
                                                                                     acc[t][ky * 3 + 1], 0, 0, 0);
                        acc[t][ky * 3 + 2] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(afrag, __builtin_bit_cast(bf16x8, r),
                                                                                     acc[t][ky * 3 + 2], 0, 0, 0);
                    }
                }
            }
            // the group is consumed: the next one of this band, or the first of the next band, takes its registers
            if (ks0 + WK * kWgradDeltaAhead < kb) request_delta(j, ks0 + WK * kWgradDeltaAhead);
            else if (j + 1 < nb) request_delta(j + 1, kq);
            }
        }
    }

    // fold the pixel-split waves into wave kq == 0 (fixed order), then write this workgroup's partial
    __syncthreads();
    float *red = reinterpret_cast<float *>(smem);   // [(WK-1)*WM waves][NTI*9][64 lanes][4]
    if (WK > 1) {
        if (kq > 0) {
            float *dst = red + (size_t)((kq - 1) * WM + mi) * (NTI * 9 * 256);
#pragma unroll
            for (int t = 0; t < NTI; ++t)
#pragma unroll
                for (int k = 0; k < 9; ++k) *reinterpret_cast<f32x4 *>(dst + ((t * 9 + k) * 64 + lane) * 4) = acc[t][k];
        }
        __syncthreads();
        if (kq == 0)
            for (int o = 1; o < WK; ++o) {
                const float *src = red + (size_t)((o - 1) * WM + mi) * (NTI * 9 * 256);
#pragma unroll
                for (int t = 0; t < NTI; ++t)
#pragma unroll
                    for (int k = 0; k < 9; ++k) acc[t][k] += *reinterpret_cast<const f32x4 *>(src + ((t * 9 + k) * 64 + lane) * 4);
            }
        __syncthreads();
    }
    float *out = a.part + ((i64)w * a.splits + sp) * psz;
    if (kq == 0) {   // 16-byte stores, 1 KB per wave and tap; wgrad_reduce_kernel puts the elements in their places
#pragma unroll
        for (int t = 0; t < NTI; ++t)
#pragma unroll
            for (int k = 0; k < 9; ++k)
                *reinterpret_cast<f32x4 *>(out + (((mi * (CI / 16) + t0 + t) * 9 + k) * 64 + lane) * 4) = acc[t][k];
    }
    // bias: sum of every delta element this workgroup saw
    for (int off = 32; off > 0; off >>= 1) bsum += __shfl_down(bsum, off, 64);
    if (lane == 0 && th == 0) red[wave] = bsum;
    __syncthreads();
    if (tid == 0) out[psz - 1] = (red[0] + red[1]) + (red[2] + red[3]);
}

// G[w_off + ...] = sum over splits of the partials (ascending split), G[b_off] = sum of the bias partials, for every
// convolution of the network in one launch (the jobs travel in the kernel arguments).
// grid (sum over jobs of tiles + 1, n), block 256: block T of a job sums its (co tile, ci tile) pair T, reading along
// the accumulator order (consecutive threads, consecutive floats), turns the tile into G's [c_out][c_in][tap] order
// in LDS and writes 16 runs of up to 144 consecutive floats; the job's last block adds the bias partials.
__global__ void __launch_bounds__(256) wgrad_reduce_kernel(WgradReduceTable tbl, float *__restrict__ G, i64 ld)
{
    __shared__ float tile[16 * 16 * 9];
    int lo = 0, hi = tbl.njobs - 1;   // the job of this workgroup: last one whose first block is <= blockIdx.x
    while (lo < hi) {
        const int mid = (lo + hi + 1) >> 1;
        if ((int)blockIdx.x >= tbl.job[mid].block0) lo = mid; else hi = mid - 1;
    }
    const WgradReduceJob &jb = tbl.job[lo];
    const int T = (int)blockIdx.x - jb.block0, w = blockIdx.y, tid = threadIdx.x;
    const int splits = jb.splits, psz = jb.psz;
    const float *p = jb.part + (i64)w * splits * psz;
    if (T == jb.tiles) {
        if (tid == 0) {
            float s = 0.f;
            for (int k = 0; k < splits; ++k) s += p[(i64)k * psz + psz - 1];
            G[(i64)w * ld + jb.b_off] = s;
        }
        return;
    }
    {   // element tid of the tile's 256 per tap: lane tid / 4 (c_in = lane % 16, row group lane / 16), register tid % 4
        const int lane = tid >> 2, i = tid & 3;
        const int ol = 4 * (lane >> 4) + i, cl = lane & 15;
        float s[9];
#pragma unroll
        for (int k = 0; k < 9; ++k) s[k] = 0.f;
        for (int sp = 0; sp < splits; ++sp) {
            const float *q = p + (i64)sp * psz + (i64)T * 9 * 256 + tid;
#pragma unroll
            for (int k = 0; k < 9; ++k) s[k] += q[k * 256];
        }
#pragma unroll
        for (int k = 0; k < 9; ++k) tile[(ol * 16 + cl) * 9 + k] = s[k];
    }
    __syncthreads();
    const int o0 = (T / jb.ci_tiles) * 16, c0 = (T % jb.ci_tiles) * 16;
    const int run = (jb.CIr - c0 < 16 ? jb.CIr - c0 : 16) * 9;   // floats of one c_out row that exist
    for (int e = tid; e < 16 * 144; e += 256) {
        const int ol = e / 144, r = e % 144;
        if (r < run) G[(i64)w * ld + jb.w_off + ((i64)(o0 + ol) * jb.CIr + c0) * 9 + r] = tile[e];
    }
}

// Workgroups that share one worker's minibatch (each writes a partial sum of the whole weight gradient): few when
// the gradient is large (the partials are HBM traffic), more when the source rows of a band are many.
int wgrad_splits(int B, int co, int stride)
{
    int m = co >= 64 ? 2 : (co >= 32 ? 4 : 8);
    if (stride == 2 && m < 8) m *= 2;
    return B < m ? B : m;
}

size_t wgrad_lds_bytes(int ci, int stride, int rb, int Wo)
{
    return (size_t)ci * wgrad_channel_pitch(((rb - 1) * stride + 3) * stride * (Wo + 16)) * sizeof(bf16_t);
}

// Output rows per band of the weight-gradient kernel: 16 at stride 1 and 32 or more channels where the image has them
// and the band's source rows fit the staging registers and 64 KB of LDS (32 channels on 16 x 16 images: 45.3 -> 39.8
// us), else 8 (with 16 channels the two more staging registers do not fit beside four workgroups per CU: 54.4 -> 55.9).
int wgrad_band_rows(const ConvDesc &c)
{
    const int cip = (c.Ci + 15) / 16 * 16;
    if (c.stride == 1 && cip >= 32 && c.Ho % 16 == 0 && cip * 18 * (c.W / 8) <= wgrad_stage(1, 16) * 256 &&
        wgrad_lds_bytes(cip, 1, 16, c.Wo) <= 64 * 1024)
        return 16;
    return 8;
}

bool wgrad_mfma_ok(const ConvDesc &c)
{
    const int cip = (c.Ci + 15) / 16 * 16;
    if (!pow2_channels(c.Co) || !pow2_channels(cip)) return false;
    if (c.Ho % 8 || c.Wo % 8 || c.W % 8 || c.W > 64) return false;
    if (cip * (7 * c.stride + 3) * (c.W / 8) > wgrad_stage(c.stride, 8) * 256) return false;   // a band's source rows fit the staging registers
    if (c.stride == 1) return cip == c.Co;
    return c.stride == 2 && c.Co == 2 * c.Ci && c.Ci <= 32 && c.W == 2 * c.Wo && c.H == 2 * c.Ho;
}

template <int CI, int CO, int STRIDE>
dpsgd_status launch_wgrad(dpsgd_ctx *ctx, const ConvDesc &c, const WgradMfmaArgs &a, WgradReduceJob *job)
{
    constexpr int WM = (CO / 16) < 4 ? (CO / 16) : 4, WK = 4 / WM, WT = wgrad_wave_groups(CI, CO), NTI = CI / 16 / WT;
    const int rb = STRIDE == 1 ? wgrad_band_rows(c) : 8;
    size_t shm = wgrad_lds_bytes(CI, STRIDE, rb, a.Wo);
    const size_t red = (size_t)(WK - 1) * WM * NTI * 9 * 256 * sizeof(float);
    if (red > shm) shm = red;
    if (shm < 64) shm = 64;
    const dim3 grid((unsigned)a.splits, (unsigned)ctx->n), block(256 * WT);
    if constexpr (STRIDE == 1 && CI >= 32) {
        if (rb == 16) hipLaunchKernelGGL((conv_wgrad_mfma_kernel<CI, CO, STRIDE, 16>), grid, block, shm, ctx->stream, a);
        else hipLaunchKernelGGL((conv_wgrad_mfma_kernel<CI, CO, STRIDE, 8>), grid, block, shm, ctx->stream, a);
    } else {
        hipLaunchKernelGGL((conv_wgrad_mfma_kernel<CI, CO, STRIDE, 8>), grid, block, shm, ctx->stream, a);
    }
    constexpr int tiles = (CO / 16) * (CI / 16), psz = tiles * 9 * 256 + 1;
    job->part = a.part; job->w_off = c.w_off; job->b_off = c.b_off; job->splits = a.splits; job->psz = psz;
    job->tiles = tiles; job->ci_tiles = CI / 16; job->CIr = a.CIr; job->block0 = 0;
    return hip_status(hipGetLastError());
}

// Can the MFMA kernel produce a tensor of Hd x Wd from a source of width Ws?
bool tile_ok(int Hd, int Wd, int stride, int ci)
{
    if (Hd % 8 || !(Wd == 8 || Wd == 16 || Wd == 32 || Wd == 64)) return false;
    const size_t pr = 7 * stride + 3, pc = (size_t)(Wd - 1) * stride + 3;
    return pr * pc * (ci + 8) * 2 + 64 * 64 <= 64 * 1024;   // patch + the band's sign bitmap (at most 64 channels x 64 bytes)
}

// The stem (at most 8 input channels) runs on an image padded to 8 channels (NHWC8).
bool stem_like(const ConvDesc &c) { return c.Ci <= 8 && c.Co == 16 && c.stride == 1; }

bool fwd_mfma_ok(const ConvDesc &c)
{
    if (stem_like(c)) return tile_ok(c.Ho, c.Wo, 1, 8);
    if (!pow2_channels(c.Ci) || !pow2_channels(c.Co) || (c.W % 8) != 0) return false;   // source rows in 16-byte units
    if (c.stride == 1) return c.Ci == c.Co && tile_ok(c.Ho, c.Wo, 1, c.Ci);
    return c.stride == 2 && c.Co == 2 * c.Ci && c.Ci <= 32 && tile_ok(c.Ho, c.Wo, 2, c.Ci);
}

bool dgrad_mfma_ok(const ConvDesc &c)
{
    if (stem_like(c)) return false;
    if (!pow2_channels(c.Ci) || !pow2_channels(c.Co) || (c.Wo % 8) != 0) return false;
    if (c.stride == 1) return c.Ci == c.Co && tile_ok(c.H, c.W, 1, c.Co);
    return c.stride == 2 && c.Co == 2 * c.Ci && c.Ci <= 32 && c.H == 2 * c.Ho && c.W == 2 * c.Wo &&
           tile_ok(c.H, c.W, 1, c.Co);
}

// LDS of a workgroup that owns th output rows: the source patch and (forward) the bands' sign bitmap
size_t conv_lds_bytes(int th, int Wd, int stride, int ci, int co, bool dgrad)
{
    const size_t pr = (size_t)(th - 1) * stride + 3, pc = (size_t)(Wd - 1) * stride + 3;
    return pr * pc * (ci + 8) * sizeof(bf16_t) + (dgrad ? 0 : (size_t)co * Wd * (th / 8));
}

// Output rows per workgroup.  16 where the destination has them, the patch stays within 64 KB and the source is
// not dilated (the dilated data gradient is slower with the taller patch, which is half zeros); else 8.
// "conv_band_rows" = 8 or 16 forces one of them where it is possible.
int conv_band_rows(const dpsgd_ctx *ctx, int Hd, int Wd, int stride, int dilate, int ci, int co, bool dgrad)
{
    const bool fits = Hd % 16 == 0 && conv_lds_bytes(16, Wd, stride, ci, co, dgrad) <= 64 * 1024;
    if (ctx->opt_conv_band_rows) return (ctx->opt_conv_band_rows == 16 && fits) ? 16 : 8;
    return (fits && dilate == 1) ? 16 : 8;
}

template <int CI, int CO, int STRIDE, int DILATE, bool DGRAD>
dpsgd_status launch_conv(dpsgd_ctx *ctx, const ConvMfmaArgs &a)
{
    const int th = conv_band_rows(ctx, a.Hd, a.Wd, STRIDE, DILATE, CI, CO, DGRAD);
    const size_t shm = conv_lds_bytes(th, a.Wd, STRIDE, CI, CO, DGRAD);
    dim3 grid((unsigned)(a.Hd / th), (unsigned)a.B, (unsigned)ctx->n);
    if (th == 16)
        hipLaunchKernelGGL((conv3x3_mfma_kernel<CI, CO, STRIDE, DILATE, DGRAD, 16>), grid, dim3(256), shm, ctx->stream, a);
    else
        hipLaunchKernelGGL((conv3x3_mfma_kernel<CI, CO, STRIDE, DILATE, DGRAD, 8>), grid, dim3(256), shm, ctx->stream, a);
    return hip_status(hipGetLastError());
}

}  // namespace

namespace {
// image [n*B][C][H][W] (fp32 or bf16) -> bf16 channel-major copy (fp32 input only) and NHWC8 copy
template <bool IN_BF16>
__global__ void __launch_bounds__(256)
prep_image_kernel(const void *__restrict__ in, int C, int HW, i64 total, bf16_t *__restrict__ chw, bf16_t *__restrict__ nhwc8)
{
    const i64 idx = (i64)blockIdx.x * 256 + threadIdx.x;   // over [img][pixel]
    if (idx >= total) return;
    const i64 img = idx / HW;
    const int px = (int)(idx % HW);
    bf16_t v[8];
#pragma unroll
    for (int ch = 0; ch < 8; ++ch) {
        v[ch] = 0;
        if (ch < C) {
            const i64 src = (img * C + ch) * HW + px;
            v[ch] = IN_BF16 ? ((const bf16_t *)in)[src] : f2bf(((const float *)in)[src]);
            if (!IN_BF16 && chw) chw[src] = v[ch];
        }
    }
    if (nhwc8) {
        u32x4 pk = {(unsigned)v[0] | ((unsigned)v[1] << 16), (unsigned)v[2] | ((unsigned)v[3] << 16),
                    (unsigned)v[4] | ((unsigned)v[5] << 16), (unsigned)v[6] | ((unsigned)v[7] << 16)};
        *reinterpret_cast<u32x4 *>(nhwc8 + idx * 8) = pk;
    }
}
}  // namespace

bool conv_stem_uses_mfma(const ConvDesc &c) { return stem_like(c) && fwd_mfma_ok(c) && wgrad_mfma_ok(c); }

bool conv_forward_writes_sign(const ConvDesc &c, bool is_stem)
{
    return is_stem ? conv_stem_uses_mfma(c) : (!stem_like(c) && fwd_mfma_ok(c));
}

dpsgd_status conv_prep_image(dpsgd_ctx *ctx, const ConvDesc &c, int B, const void *image, bool image_is_bf16,
                             bf16_t *chw_bf16, bf16_t *nhwc8)
{
    const i64 total = (i64)ctx->n * B * c.H * c.W;
    if (c.Ci > 8 && nhwc8) return DPSGD_EUNSUPPORTED;
    if (image_is_bf16)
        hipLaunchKernelGGL(prep_image_kernel<true>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, ctx->stream, image,
                           c.Ci, c.H * c.W, total, chw_bf16, nhwc8);
    else
        hipLaunchKernelGGL(prep_image_kernel<false>, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, ctx->stream, image,
                           c.Ci, c.H * c.W, total, chw_bf16, nhwc8);
    return hip_status(hipGetLastError());
}

size_t conv_pack_bytes(const ConvDesc &c, bool dgrad)
{
    const bool ok = dgrad ? dgrad_mfma_ok(c) : fwd_mfma_ok(c);
    if (!ok) return 0;
    const int ci = dgrad ? c.Co : (stem_like(c) ? 8 : c.Ci), co = dgrad ? c.Ci : c.Co;
    return (size_t)ksteps(ci) * 32 * co * sizeof(bf16_t);
}

size_t conv_wgrad_partial_bytes(const ConvDesc &c, int B)
{
    if (!wgrad_mfma_ok(c)) return 0;
    const size_t cip = (size_t)(c.Ci + 15) / 16 * 16;   // partials are stored per 16 x 16 tile of (c_out, padded c_in)
    return (size_t)wgrad_splits(B, c.Co, c.stride) * ((size_t)c.Co * cip * 9 + 1) * sizeof(float);
}

dpsgd_status conv_pack_weights(dpsgd_ctx *ctx, const std::vector<ConvDesc> &convs, const float *X,
                               const std::vector<bf16_t *> &wpack_f, const std::vector<bf16_t *> &wpack_d)
{
    PackTable tbl{};
    int blocks = 0;
    auto flush = [&]() {
        if (tbl.njobs > 0)
            hipLaunchKernelGGL(pack_weights_kernel, dim3((unsigned)blocks, (unsigned)ctx->n), dim3(256), 0, ctx->stream, X,
                               ctx->ld, tbl);
        tbl.njobs = 0;
        blocks = 0;
    };
    auto add = [&](const ConvDesc &c, int CI, int CO, bool dgrad, bf16_t *dst) {
        if (tbl.njobs == kMaxPackJobs) flush();
        PackJob &jb = tbl.job[tbl.njobs++];
        jb.w_off = c.w_off; jb.dst = dst; jb.Ci = c.Ci; jb.Co = c.Co; jb.CI = CI; jb.CO = CO; jb.KS = ksteps(CI);
        jb.dgrad = dgrad ? 1 : 0; jb.block0 = blocks;
        blocks += CO / 16;   // one workgroup per tile of 16 outputs
    };
    for (size_t q = 0; q < convs.size(); ++q) {
        const ConvDesc &c = convs[q];
        if (fwd_mfma_ok(c)) add(c, stem_like(c) ? 8 : c.Ci, c.Co, false, wpack_f[q]);
        if (!stem_like(c) && dgrad_mfma_ok(c)) add(c, c.Co, c.Ci, true, wpack_d[q]);
    }
    flush();
    return hip_status(hipGetLastError());
}

dpsgd_status conv_forward(dpsgd_ctx *ctx, const ConvDesc &c, int B, Tensor in, const float *X, const bf16_t *wpack,
                          ShortcutRef sc, Tensor out)
{
    if (!fwd_mfma_ok(c)) return conv_forward_generic(ctx, c, B, in, X, sc, out);
    ConvMfmaArgs a{};
    a.src = in.t; a.Hs = c.H; a.Ws = c.W; a.wpack = wpack; a.dstT = out.t; a.Hd = c.Ho; a.Wd = c.Wo;
    a.B = B; a.X = X; a.ld = ctx->ld; a.b_off = c.b_off; a.sc = sc; a.actT = nullptr;
    a.sign_in = nullptr; a.sign_out = out.sign;
    a.lw = ilog2(a.Wd);
    if (stem_like(c)) return launch_conv<8, 16, 1, 1, false>(ctx, a);   // `in` is the image padded to 8 channels
    if (c.stride == 1) {
        if (c.Ci == 16) return launch_conv<16, 16, 1, 1, false>(ctx, a);
        if (c.Ci == 32) return launch_conv<32, 32, 1, 1, false>(ctx, a);
        return launch_conv<64, 64, 1, 1, false>(ctx, a);
    }
    if (c.Ci == 16) return launch_conv<16, 32, 2, 1, false>(ctx, a);
    return launch_conv<32, 64, 2, 1, false>(ctx, a);
}

namespace {
// Output rows per workgroup of conv_block_fwd_kernel.  8: with 16 rows (an eighth instead of a quarter of u recomputed,
// but three times the LDS and fewer workgroups per CU) the CNN iteration took 2.894 instead of 2.877 ms.
constexpr int kBlockRows = 8;
size_t conv_block_lds_bytes(int C, int W, int th)
{
    return (size_t)(th + 4) * (W + 4) * (C + 8) * sizeof(bf16_t) + (size_t)(th / 8) * C * W;
}
// 16 channels: bands of kBlockRows rows.  32 channels: only images of 16 x 16 pixels, as one band - no row of u is then
// computed twice (in 8-row bands the launch took 84.7 us against the 81.6 us of the two launches it replaces).
// 64 channels: images of 8 x 8 pixels, one band.
int conv_block_rows(const ConvDesc &c) { return c.Co == 16 ? kBlockRows : c.Co == 32 ? 16 : 8; }
}  // namespace

bool conv_block_forward_ok(const dpsgd_ctx *ctx, const ConvDesc &c1, const ConvDesc &c2)
{
    if (!ctx->opt_conv_block) return false;
    if (c1.stride != 1 || c2.stride != 1 || c1.Ci != c1.Co || c2.Ci != c1.Co || c2.Co != c1.Co) return false;
    if (!pow2_channels(c1.Co) || !fwd_mfma_ok(c1) || !fwd_mfma_ok(c2)) return false;
    if (c1.H != c2.H || c1.W != c2.W) return false;
    if (c1.Co == 16 && (c1.H % kBlockRows || !(c1.W == 16 || c1.W == 32))) return false;
    if (c1.Co == 32 && !(c1.H == 16 && c1.W == 16)) return false;
    if (c1.Co == 64 && !(c1.H == 8 && c1.W == 8)) return false;
    return conv_block_lds_bytes(c1.Co, c1.W, conv_block_rows(c1)) <= 64 * 1024;
}

dpsgd_status conv_block_forward(dpsgd_ctx *ctx, const ConvDesc &c1, const ConvDesc &c2, int B, Tensor in, const float *X,
                                const bf16_t *wpack1, const bf16_t *wpack2, Tensor u, Tensor out)
{
    if (!conv_block_forward_ok(ctx, c1, c2) || !u.sign || !out.sign) return DPSGD_EUNSUPPORTED;
    ConvBlockArgs a{};
    a.src = in.t; a.wpack1 = wpack1; a.wpack2 = wpack2; a.uT = u.t; a.yT = out.t; a.usign = u.sign; a.ysign = out.sign;
    a.H = c1.H; a.W = c1.W; a.lw = ilog2(c1.W); a.B = B; a.X = X; a.ld = ctx->ld; a.b_off1 = c1.b_off; a.b_off2 = c2.b_off;
    const int th = conv_block_rows(c1);
    const size_t shm = conv_block_lds_bytes(c1.Co, c1.W, th);
    const dim3 grid((unsigned)(c1.H / th), (unsigned)B, (unsigned)ctx->n);
    if (c1.Co == 16) hipLaunchKernelGGL((conv_block_fwd_kernel<16, kBlockRows, 32>), grid, dim3(256), shm, ctx->stream, a);
    else if (c1.Co == 32) hipLaunchKernelGGL((conv_block_fwd_kernel<32, 16, 16>), grid, dim3(256), shm, ctx->stream, a);
    else hipLaunchKernelGGL((conv_block_fwd_kernel<64, 8, 8>), grid, dim3(256), shm, ctx->stream, a);
    return hip_status(hipGetLastError());
}

dpsgd_status conv_data_grad(dpsgd_ctx *ctx, const ConvDesc &c, int B, Tensor dout, const float *X, const bf16_t *wpack_d,
                            ShortcutRef scd, Tensor act, Tensor din)
{
    if (!dgrad_mfma_ok(c)) return conv_data_grad_generic(ctx, c, B, dout, X, scd, act, din);
    ConvMfmaArgs a{};
    a.src = dout.t; a.Hs = c.Ho; a.Ws = c.Wo; a.wpack = wpack_d; a.dstT = din.t; a.Hd = c.H; a.Wd = c.W;
    a.B = B; a.X = X; a.ld = ctx->ld; a.b_off = 0; a.sc = scd; a.actT = act.t;
    a.sign_in = act.sign; a.sign_out = nullptr;
    a.lw = ilog2(a.Wd);
    if (c.stride == 1) {
        if (c.Ci == 16) return launch_conv<16, 16, 1, 1, true>(ctx, a);
        if (c.Ci == 32) return launch_conv<32, 32, 1, 1, true>(ctx, a);
        return launch_conv<64, 64, 1, 1, true>(ctx, a);
    }
    if (c.Ci == 16) return launch_conv<32, 16, 1, 2, true>(ctx, a);
    return launch_conv<64, 32, 1, 2, true>(ctx, a);
}

dpsgd_status conv_weight_grad(dpsgd_ctx *ctx, const ConvDesc &c, int B, Tensor in, Tensor dout, float *G, float *partials,
                              WgradReduceList *pending)
{
    if (!wgrad_mfma_ok(c) || !partials || !pending) return conv_weight_grad_generic(ctx, c, B, in, dout, G);
    if (pending->njobs >= kMaxReduceJobs) {   // (a network of more than 48 convolutions: sum what is pending first)
        const dpsgd_status st = conv_weight_grad_finish(ctx, pending, G);
        if (st != DPSGD_OK) return st;
    }
    WgradMfmaArgs a{};
    a.inT = in.t; a.doutT = dout.t; a.H = c.H; a.W = c.W; a.Ho = c.Ho; a.Wo = c.Wo; a.B = B; a.CIr = c.Ci;
    a.splits = wgrad_splits(B, c.Co, c.stride); a.part = partials;
    const int cip = (c.Ci + 15) / 16 * 16;
    WgradReduceJob job{};
    dpsgd_status st;
    if (c.stride == 1) {
        if (cip == 16) st = launch_wgrad<16, 16, 1>(ctx, c, a, &job);
        else if (cip == 32) st = launch_wgrad<32, 32, 1>(ctx, c, a, &job);
        else st = launch_wgrad<64, 64, 1>(ctx, c, a, &job);
    } else if (cip == 16) {
        st = launch_wgrad<16, 32, 2>(ctx, c, a, &job);
    } else {
        st = launch_wgrad<32, 64, 2>(ctx, c, a, &job);
    }
    if (st != DPSGD_OK) return st;
    WgradReduceTable *tbl = reinterpret_cast<WgradReduceTable *>(pending->table);
    job.block0 = pending->blocks;
    tbl->job[pending->njobs] = job;
    pending->njobs += 1;
    tbl->njobs = pending->njobs;
    pending->blocks += job.tiles + 1;
    return DPSGD_OK;
}

dpsgd_status conv_weight_grad_finish(dpsgd_ctx *ctx, WgradReduceList *pending, float *G)
{
    if (!pending || pending->njobs == 0) return DPSGD_OK;
    const WgradReduceTable *tbl = reinterpret_cast<const WgradReduceTable *>(pending->table);
    hipLaunchKernelGGL(wgrad_reduce_kernel, dim3((unsigned)pending->blocks, (unsigned)ctx->n), dim3(256), 0, ctx->stream, *tbl, G,
                       ctx->ld);
    pending->njobs = 0;
    pending->blocks = 0;
    return hip_status(hipGetLastError());
}

}  // namespace dpsgd

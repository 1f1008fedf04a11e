// Per-worker minibatch gradients of softmax regression / ReLU MLPs with bf16 MFMA operands
// (Algorithm 1 step 3, footnote [a]) for gfx950.
//
// Every worker multiplies its own minibatch with its OWN weights, so each layer is a batch of n
// skinny GEMMs (M = minibatch rows) with distinct weight operands: a weight is used only B times
// per pass and the kernels are bound by streaming the fp32 master weights from HBM (forward,
// data gradient) and by writing the fp32 gradient (weight gradient).  Design:
//   forward   Z[b][o]  = sum_k A[b][k] W[o][k] + bias[o]      W streamed once (non-temporal loads),
//                                                             fp32 -> bf16 in registers, staged in LDS
//                                                             (double buffered), A tile shared by the
//                                                             waves; minibatches <= 32: 512-byte rows
//                                                             of W per tile, waves split the chunk
//   dgrad     dA[b][k] = sum_o dZ[b][o] W[o][k]               W streamed once, transposed on the
//                                                             way into LDS
//   wgrad     dW[o][k] = sum_b dZ^T[o][b] A^T[k][b]           operands are tiny (L2-resident
//                                                             transposed bf16 copies), output
//                                                             streamed to G once
//   step      the weight gradient of a large layer is formed inside the kernel that applies
//             X <- W X - gamma G (ring, torus), so it never reaches memory; optionally the kernel also
//             leaves the bf16 rounding of the new weights for the next forward / dgrad.  On the
//             ring with minibatches <= 32 a wave moves whole 1 KB row pieces of X and takes the
//             gradient of its [4 rows][256 columns] strip from 4 x 4 x 4 MFMA blocks
// MFMA: v_mfma_f32_32x32x16_bf16, fp32 accumulation.  Lane l of an A (B) operand holds row
// (column) l%32 and the 8 consecutive k values 8*(l/32)..+7; accumulator register v of lane l is
// element (row (v/4)*8 + (l/32)*4 + v%4, column l%32).  (v_mfma_f32_16x16x32_bf16 on the torus and
// v_mfma_f32_4x4x4_16B_bf16 in the 1 KB-row ring kernel: layouts at those kernels.)
#include "grad_common.h"

namespace dpsgd {
namespace {

typedef long long i64;
typedef unsigned short bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef short s16x4 __attribute__((ext_vector_type(4)));

constexpr int KC = 64;        // contraction elements staged per step
constexpr int PITCH = KC + 8; // LDS row pitch in bf16 elements (144 B: 16 B aligned, spreads banks)

__device__ __forceinline__ bf16_t f2bf(float f)
{   // round to nearest, ties to even (v_cvt_pk_bf16_f32)
    const __bf16 h = (__bf16)f;
    return __builtin_bit_cast(unsigned short, h);
}
__device__ __forceinline__ unsigned pack2(float a, float b)
{
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    typedef float f32x2_t __attribute__((ext_vector_type(2)));
    const f32x2_t v = {a, b};
    return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2_t));
}
__device__ __forceinline__ float bf2f(bf16_t h) { return __uint_as_float((unsigned)h << 16); }
__device__ __forceinline__ bf16x8 frag(const bf16_t *p) { return *reinterpret_cast<const bf16x8 *>(p); }
__device__ __forceinline__ bf16x8 zero_frag()
{
    u32x4 z = {0u, 0u, 0u, 0u};
    return __builtin_bit_cast(bf16x8, z);
}

// Transposed operand copies ("T copies": minibatch index fastest) are stored in MFMA fragment order so
// that a wave fetches one operand of v_mfma_f32_32x32x16_bf16 as 1 KB of consecutive memory: rows
// (features) in groups of 32, samples in groups of 16; inside a group first the half (samples 0-7,
// 8-15), then the row, then the 8 samples.  Per worker a copy holds round_up(rows, 32) * Bp elements.
__device__ __forceinline__ i64 tfrag_off(int r, int b, int Bp)
{
    return ((i64)(r >> 5) * (Bp >> 4) + (b >> 4)) * 512 + ((b >> 3) & 1) * 256 + (r & 31) * 8 + (b & 7);
}
__device__ __forceinline__ i64 tfrag_worker(int w, int rows, int Bp) { return (i64)w * ((rows + 31) / 32 * 32) * Bp; }

// The bf16 weight copy of a layer ("bf16_shadow") is stored per worker in 32 x 32 tiles, [O/32][K/32][32][32]: the
// fused kernel writes a wave's tile as 2 KB of consecutive memory (whole cache lines per store instruction), and
// the forward / data-gradient kernels read the tiles of their [64][128] blocks as runs of 8 KB.
__device__ __forceinline__ i64 shadow_tile(int o, int k, int K) { return ((i64)(o >> 5) * (K >> 5) + (k >> 5)) * 1024; }
// Copies written by the [16 rows][1 KB] fused kernel (K % 256 == 0) are stored in its own tiles instead, [O/16][K/256][16][256]:
// a wave's store of one row is 512 consecutive bytes, and a reader's 128-wide piece of a row 256.
__device__ __forceinline__ i64 shadow_strip(int o, int k, int K)
{
    return ((i64)(o >> 4) * (K >> 8) + (k >> 8)) * 4096 + (o & 15) * 256 + (k & 255);
}

// Which of the 64 rows of a [64 rows][512 bytes] fp32 weight tile the piece r = 2 wave + half + 8 q is (wave 0..3, half
// of the wave, instruction q 0..7), i.e. which rows one wave's load instructions touch.  The HBM channels serve a wave
// faster when all its pieces lie a multiple of 32 KB apart (see mix_ring_fat_kernel): with rows of 16 KB or a multiple
// (K % 4096 == 0) the halves of a wave take rows two apart and the wave keeps to rows of one parity (-5 and -7 us per
// iteration in the data gradient and the forward of the 4096 x 4096 layer of configs[3]); else consecutive rows (for
// 12 KB rows, halves eight rows apart were measured and are slightly slower).  A permutation of 0..63 either way.
__device__ __forceinline__ int weight_tile_row(int r, int K)
{
    return (K & 4095) == 0 ? (r & ~7) + ((r >> 1) & 1) + 2 * (r & 1) + 4 * ((r >> 2) & 1) : r;
}

// Workgroups are dealt to the 8 XCDs round-robin by linear id and every XCD has its own L2.  For a grid
// (tiles, 1, n) with n a multiple of 8 the ids are renumbered so that all tiles of a worker run on one XCD and
// the worker's activation (or delta) matrix is fetched into one L2 instead of eight.
__device__ __forceinline__ void worker_tile_on_one_xcd(int &tile, int &w)
{
    tile = blockIdx.x;
    w = blockIdx.z;
    if (gridDim.y == 1 && (gridDim.z & 7) == 0) {
        const unsigned id = blockIdx.x + gridDim.x * blockIdx.z;
        const unsigned xcd = id & 7, slot = id >> 3;
        w = (int)((slot / gridDim.x) * 8 + xcd);
        tile = (int)(slot % gridDim.x);
    }
}

// ------------------------------------------------------------------ input preparation
// in: [n*B][F] fp32 or bf16 -> a [n][B][F] bf16 (only when the input is fp32) and
// at = its T copy (zero padded samples).  32x32 tiles through LDS.
template <bool IN_BF16>
__global__ void __launch_bounds__(256)
prep_input_kernel(const void *__restrict__ in, bf16_t *__restrict__ a, bf16_t *__restrict__ at, int B, int Bp, int F)
{
    __shared__ bf16_t tile[32][33];
    const int w = blockIdx.z, b0 = blockIdx.y * 32, f0 = blockIdx.x * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 x 8
    for (int r = ty; r < 32; r += 8) {
        const int b = b0 + r, f = f0 + tx;
        bf16_t v = 0;
        if (b < B && f < F) {
            const i64 idx = ((i64)w * B + b) * F + f;
            v = IN_BF16 ? ((const bf16_t *)in)[idx] : f2bf(((const float *)in)[idx]);
            if (!IN_BF16) a[idx] = v;
        }
        tile[r][tx] = v;
    }
    __syncthreads();
    if (threadIdx.x < 128) {   // one 16-byte chunk (8 samples of one feature) per thread
        const int r = threadIdx.x & 31, c = threadIdx.x >> 5;
        const int f = f0 + r, b = b0 + 8 * c;
        if (f < F) {
            unsigned short e[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) e[j] = tile[8 * c + j][r];
            u32x4 pk = {e[0] | ((unsigned)e[1] << 16), e[2] | ((unsigned)e[3] << 16), e[4] | ((unsigned)e[5] << 16),
                        e[6] | ((unsigned)e[7] << 16)};
            *reinterpret_cast<u32x4 *>(at + tfrag_worker(w, F, Bp) + tfrag_off(f, b, Bp)) = pk;
        }
    }
}

// The same for bf16 inputs whose rows are 16-byte aligned (F % 8 == 0): 64 features x 32 samples per
// workgroup, 16-byte loads (8 features of a sample) and 16-byte stores (8 samples of a feature).
__global__ void __launch_bounds__(256)
prep_input_vec_kernel(const bf16_t *__restrict__ in, bf16_t *__restrict__ at, int B, int Bp, int F)
{
    __shared__ bf16_t tile[32][72];   // [sample][feature], pitch 144 bytes
    const int w = blockIdx.z, b0 = blockIdx.y * 32, f0 = blockIdx.x * 64;
    {
        const int r = threadIdx.x >> 3, c8 = threadIdx.x & 7;   // sample row, group of 8 features
        const int b = b0 + r, f = f0 + 8 * c8;
        u32x4 v = {0u, 0u, 0u, 0u};
        if (b < B && f < F) v = *reinterpret_cast<const u32x4 *>(in + ((i64)w * B + b) * F + f);
        *reinterpret_cast<u32x4 *>(&tile[r][8 * c8]) = v;
    }
    __syncthreads();
    {
        const int r = threadIdx.x & 63, c = threadIdx.x >> 6;   // feature, group of 8 samples
        const int f = f0 + r, b = b0 + 8 * c;
        if (f < F) {
            unsigned short e[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) e[j] = tile[8 * c + j][r];
            u32x4 pk = {e[0] | ((unsigned)e[1] << 16), e[2] | ((unsigned)e[3] << 16), e[4] | ((unsigned)e[5] << 16),
                        e[6] | ((unsigned)e[7] << 16)};
            *reinterpret_cast<u32x4 *>(at + tfrag_worker(w, F, Bp) + tfrag_off(f, b, Bp)) = pk;
        }
    }
}

// --------------------------------------------------------------------------- forward
struct FwdArgs {
    const bf16_t *act;     // [n][B][K]
    const float *X;        // replicas
    i64 ld, woff, boff;
    int B, Bp, K, O;
    bf16_t *h;             // [n][B][O]   (hidden layers)
    bf16_t *ht;            // T copy of h (hidden layers)
    float *z;              // [n][B][O]   (last layer, fp32 logits)
    const bf16_t *wb;      // bf16 copy of the weights left by the previous fused step, or null
    int wb_strips;         // its layout: 0 = 32 x 32 tiles (shadow_tile), 1 = [16][256] tiles (shadow_strip)
    // class layer only (mlp_fwd_last_kernel), or null: softmax cross-entropy in the same launch
    const int *labels;     // [n][B]
    bf16_t *sm_dz;         // [n][B][O] deltas of the class layer
    bf16_t *sm_dzt;        // their T copy
    float *loss_part;      // [n][ceil(B / 32)]: each workgroup's sum of the sample losses
};

// Epilogue of one 32 x 32 accumulator tile of the forward product: lane owns output column o and the 16 rows
// bt + (v/4)*8 + half*4 + v%4.  Adds the bias; hidden layers: ReLU, bf16 activation in [b][o] order and in the
// T copy (zero padded samples); last layer: fp32 logits.
template <bool LAST>
__device__ __forceinline__ void fwd_store_tile(const FwdArgs &g, int w, int o, int bt, int half, float bias, const f32x16 &acc)
{
#pragma unroll
    for (int grp = 0; grp < 4; ++grp) {
        const int bb = bt + grp * 8 + half * 4;   // 4 consecutive rows bb..bb+3
        float v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[i] = acc[grp * 4 + i] + bias;
            if (!LAST) v[i] = v[i] > 0.f ? v[i] : 0.f;
        }
        if (LAST) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (bb + i < g.B) g.z[((i64)w * g.B + bb + i) * g.O + o] = v[i];
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                if (bb + i < g.B) g.h[((i64)w * g.B + bb + i) * g.O + o] = f2bf(v[i]);
                else v[i] = 0.f;
            }
            if (bb < g.Bp) {
                u32x2 p = {pack2(v[0], v[1]), pack2(v[2], v[3])};
                *reinterpret_cast<u32x2 *>(g.ht + tfrag_worker(w, g.O, g.Bp) + tfrag_off(o, bb, g.Bp)) = p;
            }
        }
    }
}

// grid (ceil(O / (32 WN)), ceil(B / (32 WM MT)), n), block 256 = WM x WN waves.
template <int WM, int WN, int MT, bool VEC, bool LAST>
__global__ void __launch_bounds__(256) mlp_fwd_kernel(FwdArgs g)
{
    constexpr int TO = 32 * WN, MBLK = 32 * WM * MT;
    constexpr int WQ = TO / 16;     // float4 units of the W tile per thread
    constexpr int AQ = MBLK / 32;   // 16-byte units of the A tile per thread
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    bf16_t *Wt = reinterpret_cast<bf16_t *>(smem);          // [2][TO][PITCH]
    bf16_t *At = Wt + 2 * TO * PITCH;                        // [2][MBLK][PITCH]
    int w, tile;
    worker_tile_on_one_xcd(tile, w);
    const int o0 = tile * TO, b0 = blockIdx.y * MBLK;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int l32 = lane & 31, half = lane >> 5;
    const float *Wg = g.X + (i64)w * g.ld + g.woff;
    const bf16_t *Ag = g.act + (i64)w * g.B * g.K;

    // The weights (fp32, from HBM) are fetched TWO chunks ahead into two register sets, the activations (bf16, L2
    // resident) one chunk ahead: with a large minibatch there are few workgroups per CU and the bytes each keeps in
    // flight bound the rate.  VEC loads are branch-free (an element outside the matrix reads a clamped address and
    // is replaced by zero), so that the loads of one fetch are issued back to back and waited for by count.
    u32x4 areg[AQ];
    auto fetch_w = [&](int k0, f32x4 (&wreg)[WQ]) {
#pragma unroll
        for (int q = 0; q < WQ; ++q) {
            const int u = tid + 256 * q, row = u >> 4, kq = (u & 15) * 4;
            const int o = o0 + row, k = k0 + kq;
            f32x4 v = {0.f, 0.f, 0.f, 0.f};
            if (VEC) {   // K % 8 == 0: a group of four is inside the row or outside it
                v = __builtin_nontemporal_load(   // stage() replaces what lies outside the matrix by zero
                    reinterpret_cast<const f32x4 *>(Wg + (i64)(o < g.O ? o : g.O - 1) * g.K + (k < g.K ? k : 0)));
            } else if (o < g.O) {
                const float *p = Wg + (i64)o * g.K + k;
                if (k < g.K) v.x = p[0];
                if (k + 1 < g.K) v.y = p[1];
                if (k + 2 < g.K) v.z = p[2];
                if (k + 3 < g.K) v.w = p[3];
            }
            wreg[q] = v;
        }
    };
    auto fetch_a = [&](int k0) {
#pragma unroll
        for (int q = 0; q < AQ; ++q) {
            const int u = tid + 256 * q, row = u >> 3, kq = (u & 7) * 8;
            const int b = b0 + row, k = k0 + kq;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (VEC) {
                v = *reinterpret_cast<const u32x4 *>(Ag + (i64)(b < g.B ? b : g.B - 1) * g.K + (k < g.K ? k : 0));
            } else if (b < g.B) {
                const bf16_t *p = Ag + (i64)b * g.K + k;
                unsigned short e[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) e[i] = (k + i < g.K) ? p[i] : (unsigned short)0;
                v.x = e[0] | ((unsigned)e[1] << 16); v.y = e[2] | ((unsigned)e[3] << 16);
                v.z = e[4] | ((unsigned)e[5] << 16); v.w = e[6] | ((unsigned)e[7] << 16);
            }
            areg[q] = v;
        }
    };
    // k0: the chunk the registers hold (VEC: decides which of the clamped loads lie outside the matrix)
    auto stage = [&](int buf, const f32x4 (&wreg)[WQ], int k0) {
        bf16_t *Wb = Wt + buf * TO * PITCH, *Ab = At + buf * MBLK * PITCH;
#pragma unroll
        for (int q = 0; q < WQ; ++q) {
            const int u = tid + 256 * q, row = u >> 4, kq = (u & 15) * 4;
            u32x2 p = {pack2(wreg[q].x, wreg[q].y), pack2(wreg[q].z, wreg[q].w)};
            if (VEC && !(o0 + row < g.O && k0 + kq < g.K)) p = (u32x2){0u, 0u};
            *reinterpret_cast<u32x2 *>(Wb + row * PITCH + kq) = p;
        }
#pragma unroll
        for (int q = 0; q < AQ; ++q) {
            const int u = tid + 256 * q, row = u >> 3, kq = (u & 7) * 8;
            u32x4 v = areg[q];
            if (VEC && !(b0 + row < g.B && k0 + kq < g.K)) v = (u32x4){0u, 0u, 0u, 0u};
            *reinterpret_cast<u32x4 *>(Ab + row * PITCH + kq) = v;
        }
    };

    f32x16 acc[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[m][v] = 0.f;
    auto multiply = [&](int buf) {
        const bf16_t *Wb = Wt + buf * TO * PITCH + (wn * 32 + l32) * PITCH + 8 * half;
        const bf16_t *Ab = At + buf * MBLK * PITCH + (wm * MT * 32 + l32) * PITCH + 8 * half;
#pragma unroll
        for (int ks = 0; ks < KC / 16; ++ks) {
            const bf16x8 bw = frag(Wb + ks * 16);
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                const bf16x8 aa = frag(Ab + m * 32 * PITCH + ks * 16);
                acc[m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aa, bw, acc[m], 0, 0, 0);
            }
        }
    };

    // Workgroups start their walk over the contraction at different chunks: started together at chunk 0 they
    // would all read the same column range of W at the same time, rows a multiple of 4 KB apart.
    const int nchunks = (g.K + KC - 1) / KC;
    const int start = (int)((unsigned)(tile * 5 + w * 3) % (unsigned)nchunks);
    auto chunk_k = [&](int c) { const int cc = c + start; return (cc >= nchunks ? cc - nchunks : cc) * KC; };
    f32x4 w_even[WQ], w_odd[WQ];   // weights of the even and of the odd chunks on their way
    fetch_w(chunk_k(0), w_even);
    fetch_a(chunk_k(0));
    fetch_w(chunk_k(nchunks > 1 ? 1 : 0), w_odd);
    stage(0, w_even, chunk_k(0));
    __syncthreads();
    // one step: chunk c is multiplied from LDS buffer c % 2 while the activations of chunk c + 1 and the weights of
    // chunk c + 2 are on their way (the activations are requested first: staging waits for them, not for the younger
    // weight loads).  Past the end the fetches repeat the last chunk (values never used): no branch around a load.
    auto step = [&](int c, f32x4 (&w_this)[WQ], const f32x4 (&w_next)[WQ]) {
        const int last = nchunks - 1;
        fetch_a(chunk_k(c + 1 < nchunks ? c + 1 : last));
        __builtin_amdgcn_sched_barrier(0);   // keep this order of issue: the wait for the activations counts on it
        fetch_w(chunk_k(c + 2 < nchunks ? c + 2 : last), w_this);   // chunk c's weights are in LDS: its registers are free
        __builtin_amdgcn_sched_barrier(0);
        multiply(c & 1);
        __builtin_amdgcn_sched_barrier(0);
        stage((c & 1) ^ 1, w_next, chunk_k(c + 1 < nchunks ? c + 1 : last));   // (past the end: written, never read)
        __syncthreads();
    };
    for (int c = 0; c < nchunks; c += 2) {
        step(c, w_even, w_odd);
        if (c + 1 < nchunks) step(c + 1, w_odd, w_even);
    }

    // epilogue: lane owns output column o, 16 rows per m-tile
    const int o = o0 + wn * 32 + l32;
    if (o >= g.O) return;
    const float bias = g.X[(i64)w * g.ld + g.boff + o];
#pragma unroll
    for (int m = 0; m < MT; ++m) fwd_store_tile<LAST>(g, w, o, b0 + (wm * MT + m) * 32, half, bias, acc[m]);
}

// Minibatches of more than 64 rows (one 128-row block of the minibatch per workgroup, so the weights are read once):
// the product above with chunks of 128 contraction elements, so that a row of the weight tile is 512 consecutive
// bytes (with 64 the kernel above streams 4.2 TB/s of weights at 3072 x 1024 x 32 workers, bound by the 256-byte
// pieces, whatever the prefetch distance).  One LDS buffer of (64 + 128) rows x 272 bytes (three workgroups per CU)
// instead of two: the next chunk waits in registers while the current one is multiplied, and goes to LDS between
// two barriers.  Rows 16-byte aligned and K % 8 == 0 (the VEC case of the kernel above); loads are branch-free
// (clamped addresses; what lies outside the matrix is replaced by zero on its way to LDS).
// grid (ceil(O / 64), ceil(B / 128), n), block 256 = 2 x 2 waves, each two 32 x 32 tiles.
constexpr int KCW = 128;
constexpr int PITCHW = KCW + 8;

template <bool LAST>
__global__ void __launch_bounds__(256, 3) mlp_fwd_wide_kernel(FwdArgs g)
{
    constexpr int TO = 64, MBLK = 128, MT = 2, WQ = 8, AQ = 8;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    bf16_t *Wt = reinterpret_cast<bf16_t *>(smem);   // [TO][PITCHW]
    bf16_t *At = Wt + TO * PITCHW;                    // [MBLK][PITCHW]
    int w, tile;
    worker_tile_on_one_xcd(tile, w);
    const int o0 = tile * TO, b0 = blockIdx.y * MBLK;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int l32 = lane & 31, half = lane >> 5;
    const float *Wg = g.X + (i64)w * g.ld + g.woff;
    const bf16_t *Ag = g.act + (i64)w * g.B * g.K;

    f32x4 wreg[WQ];
    u32x4 areg[AQ];
    // unit u = tid + 256 q.  W: row u / 32, floats (u % 32) * 4 .. + 3 (a wave instruction: two rows x 512 bytes);
    // A: row u / 16, elements (u % 16) * 8 .. + 7
    auto fetch = [&](int k0) {
#pragma unroll
        for (int q = 0; q < AQ; ++q) {
            const int u = tid + 256 * q, b = b0 + (u >> 4), k = k0 + (u & 15) * 8;
            areg[q] = *reinterpret_cast<const u32x4 *>(Ag + (i64)(b < g.B ? b : g.B - 1) * g.K + (k < g.K ? k : 0));
        }
#pragma unroll
        for (int q = 0; q < WQ; ++q) {
            const int u = tid + 256 * q, o = o0 + weight_tile_row(u >> 5, g.K), k = k0 + (u & 31) * 4;
            wreg[q] = __builtin_nontemporal_load(
                reinterpret_cast<const f32x4 *>(Wg + (i64)(o < g.O ? o : g.O - 1) * g.K + (k < g.K ? k : 0)));
        }
    };
    auto stage = [&](int k0) {
#pragma unroll
        for (int q = 0; q < WQ; ++q) {
            const int u = tid + 256 * q, row = weight_tile_row(u >> 5, g.K), kq = (u & 31) * 4;
            u32x2 p = {pack2(wreg[q].x, wreg[q].y), pack2(wreg[q].z, wreg[q].w)};
            if (!(o0 + row < g.O && k0 + kq < g.K)) p = (u32x2){0u, 0u};
            *reinterpret_cast<u32x2 *>(Wt + row * PITCHW + kq) = p;
        }
#pragma unroll
        for (int q = 0; q < AQ; ++q) {
            const int u = tid + 256 * q, row = u >> 4, kq = (u & 15) * 8;
            u32x4 v = areg[q];
            if (!(b0 + row < g.B && k0 + kq < g.K)) v = (u32x4){0u, 0u, 0u, 0u};
            *reinterpret_cast<u32x4 *>(At + row * PITCHW + kq) = v;
        }
    };

    f32x16 acc[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[m][v] = 0.f;

    // workgroups start their walk over the contraction at different chunks (see the kernel above)
    const int nchunks = (g.K + KCW - 1) / KCW;
    const int start = (int)((unsigned)(tile * 5 + w * 3) % (unsigned)nchunks);
    auto chunk_k = [&](int c) { const int cc = c + start; return (cc >= nchunks ? cc - nchunks : cc) * KCW; };
    fetch(chunk_k(0));
    stage(chunk_k(0));
    __syncthreads();
    const bf16_t *Wb = Wt + (wn * 32 + l32) * PITCHW + 8 * half;
    const bf16_t *Ab = At + (wm * MT * 32 + l32) * PITCHW + 8 * half;
    for (int c = 0; c < nchunks; ++c) {
        const int nxt = chunk_k(c + 1 < nchunks ? c + 1 : c);   // past the end: the last chunk again, never used
        fetch(nxt);
        __builtin_amdgcn_sched_barrier(0);   // the loads are on their way before the first LDS read
#pragma unroll
        for (int ks = 0; ks < KCW / 16; ++ks) {
            const bf16x8 bw = frag(Wb + ks * 16);
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                const bf16x8 aa = frag(Ab + m * 32 * PITCHW + ks * 16);
                acc[m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aa, bw, acc[m], 0, 0, 0);
            }
        }
        __syncthreads();   // every wave has read chunk c
        stage(nxt);
        __syncthreads();
    }

    const int o = o0 + wn * 32 + l32;
    if (o >= g.O) return;
    const float bias = g.X[(i64)w * g.ld + g.boff + o];
#pragma unroll
    for (int m = 0; m < MT; ++m) fwd_store_tile<LAST>(g, w, o, b0 + (wm * MT + m) * 32, half, bias, acc[m]);
}

// Minibatches of at most 32 rows: the same product with a [64 outputs][128 k] weight tile, so that a row of the
// tile is 512 consecutive bytes of W (256-byte pieces of rows 12-16 KB apart stream ~10 % slower from HBM).  The
// four waves are 2 output tiles x 2 halves of each 128-wide chunk of the contraction; the two halves meet in LDS
// at the end.  grid (ceil(O / 64), ceil(B / 32), n), block 256.
constexpr int KC2 = 128;
constexpr int PITCH2 = KC2 + 8;

template <bool VEC, bool LAST, bool WB16>
__global__ void __launch_bounds__(256) mlp_fwd_ksplit_kernel(FwdArgs g)
{
    constexpr int TO = 64, MBLK = 32;
    constexpr int WQ = TO * KC2 / 4 / 256;    // float4 units of the W tile per thread (8)
    constexpr int BQ = TO * KC2 / 8 / 256;    // 16-byte units of a bf16 W tile per thread (4)
    constexpr int AQ = MBLK * KC2 / 8 / 256;  // 16-byte units of the A tile per thread (2)
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    bf16_t *Wt = reinterpret_cast<bf16_t *>(smem);          // [2][TO][PITCH2]
    bf16_t *At = Wt + 2 * TO * PITCH2;                       // [2][MBLK][PITCH2]
    int w, tile;
    worker_tile_on_one_xcd(tile, w);
    const int o0 = tile * TO, b0 = blockIdx.y * MBLK;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wn = wave & 1, wk = wave >> 1;
    const int l32 = lane & 31, half = lane >> 5;
    const float *Wg = g.X + (i64)w * g.ld + g.woff;
    const bf16_t *Wb16 = WB16 ? g.wb + (i64)w * g.O * g.K : nullptr;
    const bf16_t *Ag = g.act + (i64)w * g.B * g.K;

    f32x4 wreg[WB16 ? 1 : WQ];
    u32x4 breg0[WB16 ? BQ : 1];
    u32x4 areg[AQ];
    // already rounded weights (O % 64 == 0 and K % 128 == 0 hold): 16-byte unit u of the [64][128] block is, in the
    // 32 x 32-tile layout, unit u % 128 of tile u / 128 (8 tiles of 2 KB); in the [16][256] layout, 8 columns of row u / 16
    auto unit_w16 = [&](int u, int &row, int &kq) {
        if (g.wb_strips) {
            row = u >> 4;
            kq = (u & 15) * 8;
        } else {
            const int t = u >> 7, within = u & 127;
            row = (t >> 2) * 32 + (within >> 2);
            kq = (t & 3) * 32 + (within & 3) * 8;
        }
    };
    auto fetch_w16 = [&](int k0, u32x4 (&br)[WB16 ? BQ : 1]) {
#pragma unroll
        for (int q = 0; q < (WB16 ? BQ : 0); ++q) {
            int row, kq;
            unit_w16(tid + 256 * q, row, kq);
            const i64 off = g.wb_strips ? shadow_strip(o0 + row, k0 + kq, g.K)
                                        : shadow_tile(o0 + row, k0 + kq, g.K) + (row & 31) * 32 + (kq & 31);
            br[q] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(Wb16 + off));
        }
    };
    auto stage_w16 = [&](int buf, const u32x4 (&br)[WB16 ? BQ : 1]) {
        bf16_t *Wb = Wt + buf * TO * PITCH2;
#pragma unroll
        for (int q = 0; q < (WB16 ? BQ : 0); ++q) {
            int row, kq;
            unit_w16(tid + 256 * q, row, kq);
            *reinterpret_cast<u32x4 *>(Wb + row * PITCH2 + kq) = br[q];
        }
    };
    auto tile_row = [&](int r) { return weight_tile_row(r, g.K); };   // the 512-byte piece r = (tid + 256 q) / 32
    auto fetch_w32 = [&](int k0) {
#pragma unroll
        for (int q = 0; q < (WB16 ? 0 : WQ); ++q) {
            const int u = tid + 256 * q, row = tile_row(u >> 5), kq = (u & 31) * 4;
            const int o = o0 + row, k = k0 + kq;
            f32x4 v = {0.f, 0.f, 0.f, 0.f};
            if (o < g.O) {
                const float *p = Wg + (i64)o * g.K + k;
                if (VEC) {
                    if (k < g.K) v = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(p));
                } else {
                    if (k < g.K) v.x = p[0];
                    if (k + 1 < g.K) v.y = p[1];
                    if (k + 2 < g.K) v.z = p[2];
                    if (k + 3 < g.K) v.w = p[3];
                }
            }
            wreg[q] = v;
        }
    };
    auto stage_w32 = [&](int buf) {
        bf16_t *Wb = Wt + buf * TO * PITCH2;
#pragma unroll
        for (int q = 0; q < (WB16 ? 0 : WQ); ++q) {
            const int u = tid + 256 * q, row = tile_row(u >> 5), kq = (u & 31) * 4;
            u32x2 p = {pack2(wreg[q].x, wreg[q].y), pack2(wreg[q].z, wreg[q].w)};
            *reinterpret_cast<u32x2 *>(Wb + row * PITCH2 + kq) = p;
        }
    };
    auto fetch_a = [&](int k0) {
#pragma unroll
        for (int q = 0; q < AQ; ++q) {
            const int u = tid + 256 * q, row = u >> 4, kq = (u & 15) * 8;
            const int b = b0 + row, k = k0 + kq;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (b < g.B) {
                const bf16_t *p = Ag + (i64)b * g.K + k;
                if (VEC) {
                    if (k < g.K) v = *reinterpret_cast<const u32x4 *>(p);
                } else {
                    unsigned short e[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) e[i] = (k + i < g.K) ? p[i] : (unsigned short)0;
                    v.x = e[0] | ((unsigned)e[1] << 16); v.y = e[2] | ((unsigned)e[3] << 16);
                    v.z = e[4] | ((unsigned)e[5] << 16); v.w = e[6] | ((unsigned)e[7] << 16);
                }
            }
            areg[q] = v;
        }
    };
    auto stage_a = [&](int buf) {
        bf16_t *Ab = At + buf * MBLK * PITCH2;
#pragma unroll
        for (int q = 0; q < AQ; ++q) {
            const int u = tid + 256 * q, row = u >> 4, kq = (u & 15) * 8;
            *reinterpret_cast<u32x4 *>(Ab + row * PITCH2 + kq) = areg[q];
        }
    };

    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;

    // staggered start, as in mlp_fwd_kernel
    const int nchunks = (g.K + KC2 - 1) / KC2;
    const int start = (int)((unsigned)(tile * 5 + w * 3) % (unsigned)nchunks);
    auto chunk_k = [&](int c) { const int cc = c + start; return (cc >= nchunks ? cc - nchunks : cc) * KC2; };
    auto multiply = [&](int buf) {
        const bf16_t *Wb = Wt + buf * TO * PITCH2 + (wn * 32 + l32) * PITCH2 + wk * (KC2 / 2) + 8 * half;
        const bf16_t *Ab = At + buf * MBLK * PITCH2 + l32 * PITCH2 + wk * (KC2 / 2) + 8 * half;
#pragma unroll
        for (int ks = 0; ks < KC2 / 32; ++ks)
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag(Ab + ks * 16), frag(Wb + ks * 16), acc, 0, 0, 0);
    };
    // (fetching the half-size bf16 chunks two ahead, to keep as many bytes in flight as with fp32 weights, was measured
    // and is slower: 400 against 387 us; so is fetching the fp32 chunks two ahead with branch-free loads: 635 against
    // 615 us - with three workgroups per CU the memory system is already saturated, unlike in mlp_fwd_kernel's case)
    fetch_w16(chunk_k(0), breg0);
    fetch_w32(chunk_k(0));
    fetch_a(chunk_k(0));
    stage_w16(0, breg0);
    stage_w32(0);
    stage_a(0);
    // chunk c + 2 is requested at the end of step c, before the barrier (its registers are free once chunk c + 1 is
    // staged): it is in flight while the waves wait for each other, not only during the short multiply of step c + 1
    if (nchunks > 1) {
        fetch_w16(chunk_k(1), breg0);
        fetch_w32(chunk_k(1));
        fetch_a(chunk_k(1));
    }
    __syncthreads();
    for (int c = 0; c < nchunks; ++c) {
        const int buf = c & 1;
        multiply(buf);
        if (c + 1 < nchunks) {
            stage_w16(buf ^ 1, breg0);
            stage_w32(buf ^ 1);
            stage_a(buf ^ 1);
        }
        if (c + 2 < nchunks) {
            fetch_w16(chunk_k(c + 2), breg0);
            fetch_w32(chunk_k(c + 2));
            fetch_a(chunk_k(c + 2));
        }
        __syncthreads();
    }

    // the upper halves hand their sums to the lower ones (the staging buffers are free after the last barrier)
    float *red = reinterpret_cast<float *>(smem);   // [2 output tiles][16][64]
    if (wk == 1) {
#pragma unroll
        for (int v = 0; v < 16; ++v) red[(wn * 16 + v) * 64 + lane] = acc[v];
    }
    __syncthreads();
    if (wk == 1) return;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] += red[(wn * 16 + v) * 64 + lane];

    // epilogue: lane owns output column o, 16 rows
    const int o = o0 + wn * 32 + l32;
    if (o >= g.O) return;
    fwd_store_tile<LAST>(g, w, o, b0, half, g.X[(i64)w * g.ld + g.boff + o], acc);
}

// Class layer (at most 32 outputs): the tile above would be 3/4 padding and one workgroup per worker
// would walk the whole contraction alone.  Here a workgroup owns 32 samples of one worker and its 8
// waves split K; operands come straight from global memory (activations bf16, weights fp32 rounded
// in registers), the partial tiles meet in LDS.  grid (ceil(B / 32), n), block 512.  K % 16 == 0.
// With g.sm_dz set the launch goes on to the softmax cross-entropy of its 32 samples (the arithmetic of
// softmax_xent_bf16_kernel, a thread per sample) and leaves the sum of their losses in g.loss_part.
__global__ void __launch_bounds__(512) mlp_fwd_last_kernel(FwdArgs g)
{
    constexpr int NW = 8;
    __shared__ float red[NW][16][64];
    __shared__ float zs[32][33];
    const int w = blockIdx.y, b0 = blockIdx.x * 32;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int b = b0 + l32, o = l32;
    const bool b_ok = b < g.B, o_ok = o < g.O;
    const bf16_t *ap = g.act + ((i64)w * g.B + (b_ok ? b : 0)) * g.K + 8 * half;
    const float *wp = g.X + (i64)w * g.ld + g.woff + (i64)(o_ok ? o : 0) * g.K + 8 * half;
    const int steps = g.K / 16;
    const int s0 = (int)((i64)steps * wave / NW), s1 = (int)((i64)steps * (wave + 1) / NW);
    f32x16 acc;
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    for (int st = s0; st < s1; ++st) {
        bf16x8 av = zero_frag(), bv = zero_frag();
        if (b_ok) av = frag(ap + st * 16);
        if (o_ok) {
            const f32x4 lo = *reinterpret_cast<const f32x4 *>(wp + st * 16);
            const f32x4 hi = *reinterpret_cast<const f32x4 *>(wp + st * 16 + 4);
            const u32x4 pk = {pack2(lo.x, lo.y), pack2(lo.z, lo.w), pack2(hi.x, hi.y), pack2(hi.z, hi.w)};
            bv = __builtin_bit_cast(bf16x8, pk);
        }
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, bv, acc, 0, 0, 0);
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) red[wave][v][lane] = acc[v];
    __syncthreads();
    // element v of lane l: sample b0 + (v/4)*8 + (l/32)*4 + v%4, output l%32; 16 x 64 elements over 512 threads
    for (int e = threadIdx.x; e < 16 * 64; e += 512) {
        const int v = e >> 6, l = e & 63;
        const int bb = b0 + (v >> 2) * 8 + (l >> 5) * 4 + (v & 3), oo = l & 31;
        if (bb >= g.B || oo >= g.O) continue;
        float sum = 0.f;
#pragma unroll
        for (int q = 0; q < NW; ++q) sum += red[q][v][l];
        sum += g.X[(i64)w * g.ld + g.boff + oo];
        g.z[((i64)w * g.B + bb) * g.O + oo] = sum;
        if (g.sm_dz) zs[bb - b0][oo] = sum;
    }
    if (!g.sm_dz) return;
    __syncthreads();
    if (threadIdx.x >= 64) return;
    float local = 0.f;
    if (threadIdx.x < 32) {
        const int bb = b0 + (int)threadIdx.x, C = g.O;
        bf16_t *dzt = g.sm_dzt + tfrag_worker(w, C, g.Bp);
        if (bb >= g.B) {   // a padded sample: zeros in the T copy
            if (bb < g.Bp)
                for (int c = 0; c < C; ++c) dzt[tfrag_off(c, bb, g.Bp)] = 0;
        } else {
            const float *zb = zs[threadIdx.x];
            const float invB = 1.0f / (float)g.B;
            int lab = g.labels[(i64)w * g.B + bb];
            lab = lab < 0 ? 0 : (lab >= C ? C - 1 : lab);
            float mx = zb[0];
            for (int c = 1; c < C; ++c) mx = fmaxf(mx, zb[c]);
            float se = 0.f;
            for (int c = 0; c < C; ++c) se += expf(zb[c] - mx);
            const float lse = mx + logf(se);
            local = lse - zb[lab];
            for (int c = 0; c < C; ++c) {
                const bf16_t v = f2bf((expf(zb[c] - lse) - (c == lab ? 1.f : 0.f)) * invB);
                g.sm_dz[((i64)w * g.B + bb) * C + c] = v;
                dzt[tfrag_off(c, bb, g.Bp)] = v;
            }
        }
    }
    for (int off = 16; off > 0; off >>= 1) local += __shfl_down(local, off, 64);
    if (threadIdx.x == 0) g.loss_part[(i64)w * gridDim.x + blockIdx.x] = local;
}

// ------------------------------------------------------------- softmax cross-entropy
// z fp32 [n][B][C] -> dz bf16 [n][B][C], dzt = its T copy (zero padded samples), loss[n].
__global__ void __launch_bounds__(256)
softmax_xent_bf16_kernel(const float *__restrict__ z, const int *__restrict__ labels, int B, int Bp, int C,
                         bf16_t *__restrict__ dz, bf16_t *__restrict__ dzt, float *__restrict__ loss)
{
    __shared__ float red[256];
    const int w = blockIdx.x;
    const float invB = 1.0f / (float)B;
    float local = 0.f;
    for (int b = threadIdx.x; b < Bp; b += 256) {
        if (b >= B) {
            for (int c = 0; c < C; ++c) dzt[tfrag_worker(w, C, Bp) + tfrag_off(c, b, Bp)] = 0;
            continue;
        }
        const float *zb = z + ((i64)w * B + b) * C;
        int lab = labels[(i64)w * B + b];
        lab = lab < 0 ? 0 : (lab >= C ? C - 1 : lab);
        float mx = zb[0];
        for (int c = 1; c < C; ++c) mx = fmaxf(mx, zb[c]);
        float se = 0.f;
        for (int c = 0; c < C; ++c) se += expf(zb[c] - mx);
        const float lse = mx + logf(se);
        local += lse - zb[lab];
        for (int c = 0; c < C; ++c) {
            const bf16_t v = f2bf((expf(zb[c] - lse) - (c == lab ? 1.f : 0.f)) * invB);
            dz[((i64)w * B + b) * C + c] = v;
            dzt[tfrag_worker(w, C, Bp) + tfrag_off(c, b, Bp)] = v;
        }
    }
    red[threadIdx.x] = local;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) red[threadIdx.x] += red[threadIdx.x + off];
        __syncthreads();
    }
    if (loss && threadIdx.x == 0) loss[w] = red[0] * invB;
}

// ----------------------------------------------------------------------- weight gradient
struct WgradArgs {
    const bf16_t *dzt;   // T copy of dZ [n][B][O]
    const bf16_t *at;    // T copy of A  [n][B][K]
    float *G;
    i64 ld, woff, boff;
    int Bp, K, O;
};

// grid (ceil(K / 256), ceil(O / 128), n); wave = 32 rows o, walks 8 tiles of 32 columns k.
// SKINNY (few outputs, e.g. the class layer): grid (ceil(K / 128), ceil(O / 32), n); the four waves
// share the 32 rows o and take one tile of 32 columns k each.
template <bool SKINNY>
__global__ void __launch_bounds__(256) mlp_wgrad_kernel(WgradArgs g)
{
    const int w = blockIdx.z;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int o_base = SKINNY ? blockIdx.y * 32 : blockIdx.y * 128 + wave * 32;
    if (o_base >= g.O) return;
    const int o = o_base + l32;            // row this lane feeds into the A operand
    const bool o_ok = o < g.O;
    const int steps = g.Bp / 16;
    // fragment (32-row group, step st) of a T copy: 512 elements, this lane's 8 at 8 * lane
    const bf16_t *Ap = g.dzt + tfrag_worker(w, g.O, g.Bp) + (i64)(o_base >> 5) * steps * 512 + lane * 8;
    float *Gw = g.G + (i64)w * g.ld + g.woff;

    if (blockIdx.x == 0 && (!SKINNY || wave == 0)) {   // bias gradient: gb[o] = sum_b dZ[b][o]
        float s = 0.f;
        if (o_ok)
            for (int st = 0; st < steps; ++st)
#pragma unroll
                for (int j = 0; j < 8; ++j) s += bf2f(Ap[st * 512 + j]);
        s += __shfl_down(s, 32, 64);
        if (half == 0 && o_ok) g.G[(i64)w * g.ld + g.boff + o] = s;
    }

    for (int t = 0; t < (SKINNY ? 1 : 8); ++t) {
        const int k_base = SKINNY ? blockIdx.x * 128 + wave * 32 : blockIdx.x * 256 + t * 32;
        if (k_base >= g.K) break;
        const int k = k_base + l32;
        const bool k_ok = k < g.K;
        const bf16_t *Bp_ = g.at + tfrag_worker(w, g.K, g.Bp) + (i64)(k_base >> 5) * steps * 512 + lane * 8;
        f32x16 acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.f;
        for (int st = 0; st < steps; ++st) {
            const bf16x8 a = o_ok ? frag(Ap + st * 512) : zero_frag();
            const bf16x8 b = k_ok ? frag(Bp_ + st * 512) : zero_frag();
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
        }
        if (k_ok) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int orow = o_base + (v >> 2) * 8 + half * 4 + (v & 3);
                if (orow < g.O) __builtin_nontemporal_store(acc[v], Gw + (i64)orow * g.K + k);
            }
        }
    }
}

// ------------------------------------------------------------------------- data gradient
struct DgradArgs {
    const bf16_t *dz;     // [n][B][O]
    const float *X;
    i64 ld, woff;
    const bf16_t *hprev;  // [n][B][K] post-ReLU activations of the layer below (mask)
    bf16_t *dzp;          // [n][B][K]
    bf16_t *dzpt;         // T copy of dzp
    int B, Bp, K, O;
    const bf16_t *wb;     // bf16 copy of the weights left by the previous fused step, or null
    int wb_strips;        // its layout: 0 = 32 x 32 tiles (shadow_tile), 1 = [16][256] tiles (shadow_strip)
};

// grid (ceil(K / (32 WN)), ceil(B / (32 WM MT)), n), block 256.
template <int WM, int WN, int MT, bool VEC, bool WB16 = false>
__global__ void __launch_bounds__(256) mlp_dgrad_kernel(DgradArgs g)
{
    constexpr int TK = 32 * WN, MBLK = 32 * WM * MT;
    constexpr int WQ = TK / 16;     // float4 units of the [64 o][TK k] W tile per thread
    constexpr int BQ = TK / 32;     // 16-byte units of the bf16 W tile per thread
    constexpr int DQ = MBLK / 32;   // 16-byte units of the dZ tile per thread
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    constexpr int WP = TK + 8;                               // pitch of the W tile (bf16 elements)
    bf16_t *Wt = reinterpret_cast<bf16_t *>(smem);          // [2][KC o][WP]    as in memory: rows o, k contiguous
    bf16_t *Dt = Wt + 2 * KC * WP;                           // [2][MBLK][PITCH] rows b, o contiguous
    int w, tile;
    worker_tile_on_one_xcd(tile, w);
    const int kt0 = tile * TK, b0 = blockIdx.y * MBLK;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int l32 = lane & 31, half = lane >> 5;
    const float *Wg = g.X + (i64)w * g.ld + g.woff;
    const bf16_t *Wb16 = WB16 ? g.wb + (i64)w * g.O * g.K : nullptr;
    const bf16_t *Dg = g.dz + (i64)w * g.B * g.O;

    f32x4 wreg[WB16 ? 1 : WQ];
    u32x4 breg0[WB16 ? BQ : 1];
    u32x4 dreg[DQ];
    // already rounded weights (O % 64 == 0 and K % TK == 0 hold): 16-byte unit u of the [64][TK] block is, in the
    // 32 x 32-tile layout, unit u % 128 of tile u / 128 (2 x TK / 32 tiles of 2 KB); in the [16][256] layout, 8 columns
    // of row u / (TK / 8)
    auto unit_w16 = [&](int u, int &orow, int &kq) {
        if (g.wb_strips) {
            orow = u / (TK / 8);
            kq = (u % (TK / 8)) * 8;
        } else {
            const int t = u >> 7, within = u & 127;
            orow = (t / (TK / 32)) * 32 + (within >> 2);
            kq = (t % (TK / 32)) * 32 + (within & 3) * 8;
        }
    };
    auto fetch_w16 = [&](int oc, u32x4 (&br)[WB16 ? BQ : 1]) {
#pragma unroll
        for (int q = 0; q < (WB16 ? BQ : 0); ++q) {
            int orow, kq;
            unit_w16(tid + 256 * q, orow, kq);
            const i64 off = g.wb_strips ? shadow_strip(oc + orow, kt0 + kq, g.K)
                                        : shadow_tile(oc + orow, kt0 + kq, g.K) + (orow & 31) * 32 + (kq & 31);
            br[q] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(Wb16 + off));
        }
    };
    auto stage_w16 = [&](int buf, const u32x4 (&br)[WB16 ? BQ : 1]) {
        bf16_t *Wb = Wt + buf * KC * WP;
#pragma unroll
        for (int q = 0; q < (WB16 ? BQ : 0); ++q) {
            int orow, kq;
            unit_w16(tid + 256 * q, orow, kq);
            *reinterpret_cast<u32x4 *>(Wb + orow * WP + kq) = br[q];
        }
    };
    // fp32 weights (unless the bf16 copy is used) and the delta tile
    // which row of the [64 o][TK k] tile unit u = tid + 256 q takes (TK = 128: a row piece is 512 bytes, half a wave)
    auto tile_row = [&](int u) {
        const int r = u / (TK / 4);
        return TK == 128 ? weight_tile_row(r, g.K) : r;
    };
    auto fetch = [&](int oc) {
#pragma unroll
        for (int q = 0; q < (WB16 ? 0 : WQ); ++q) {
            const int u = tid + 256 * q, orow = tile_row(u), kq = (u % (TK / 4)) * 4;
            const int o = oc + orow, k = kt0 + kq;
            f32x4 v = {0.f, 0.f, 0.f, 0.f};
            if (o < g.O) {
                const float *p = Wg + (i64)o * g.K + k;
                if (VEC) {
                    if (k < g.K) v = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(p));
                } else {
                    if (k < g.K) v.x = p[0];
                    if (k + 1 < g.K) v.y = p[1];
                    if (k + 2 < g.K) v.z = p[2];
                    if (k + 3 < g.K) v.w = p[3];
                }
            }
            wreg[q] = v;
        }
#pragma unroll
        for (int q = 0; q < DQ; ++q) {
            const int u = tid + 256 * q, row = u >> 3, oq = (u & 7) * 8;
            const int b = b0 + row, o = oc + oq;
            u32x4 v = {0u, 0u, 0u, 0u};
            if (b < g.B) {
                const bf16_t *p = Dg + (i64)b * g.O + o;
                if (VEC) {
                    if (o < g.O) v = *reinterpret_cast<const u32x4 *>(p);
                } else {
                    unsigned short e[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) e[i] = (o + i < g.O) ? p[i] : (unsigned short)0;
                    v.x = e[0] | ((unsigned)e[1] << 16); v.y = e[2] | ((unsigned)e[3] << 16);
                    v.z = e[4] | ((unsigned)e[5] << 16); v.w = e[6] | ((unsigned)e[7] << 16);
                }
            }
            dreg[q] = v;
        }
    };
    auto stage = [&](int buf) {
        bf16_t *Wb = Wt + buf * KC * WP, *Db = Dt + buf * MBLK * PITCH;
#pragma unroll
        for (int q = 0; q < (WB16 ? 0 : WQ); ++q) {
            const int u = tid + 256 * q, orow = tile_row(u), kq = (u % (TK / 4)) * 4;
            u32x2 p = {pack2(wreg[q].x, wreg[q].y), pack2(wreg[q].z, wreg[q].w)};
            *reinterpret_cast<u32x2 *>(Wb + orow * WP + kq) = p;
        }
#pragma unroll
        for (int q = 0; q < DQ; ++q) {
            const int u = tid + 256 * q, row = u >> 3, oq = (u & 7) * 8;
            *reinterpret_cast<u32x4 *>(Db + row * PITCH + oq) = dreg[q];
        }
    };

    f32x16 acc[MT];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[m][v] = 0.f;

    const int nchunks = (g.O + KC - 1) / KC;
    auto multiply = [&](int buf) {
        // B operand: column k of the tile, 8 consecutive o (the transpose happens in these reads:
        // consecutive lanes read consecutive k of one LDS row)
        const bf16_t *Wb = Wt + buf * KC * WP + (8 * half) * WP + wn * 32 + l32;
        const bf16_t *Db = Dt + buf * MBLK * PITCH + (wm * MT * 32 + l32) * PITCH + 8 * half;
#pragma unroll
        for (int ks = 0; ks < KC / 16; ++ks) {
            unsigned short e[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) e[j] = Wb[(ks * 16 + j) * WP];
            u32x4 pk = {e[0] | ((unsigned)e[1] << 16), e[2] | ((unsigned)e[3] << 16), e[4] | ((unsigned)e[5] << 16),
                        e[6] | ((unsigned)e[7] << 16)};
            const bf16x8 bw = __builtin_bit_cast(bf16x8, pk);
#pragma unroll
            for (int m = 0; m < MT; ++m) {
                const bf16x8 aa = frag(Db + m * 32 * PITCH + ks * 16);
                acc[m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(aa, bw, acc[m], 0, 0, 0);
            }
        }
    };
    fetch_w16(0, breg0);
    fetch(0);
    stage_w16(0, breg0);
    stage(0);
    // chunk c + 2 is requested at the end of step c, before the barrier (see mlp_fwd_ksplit_kernel)
    if (nchunks > 1) {
        fetch_w16(KC, breg0);
        fetch(KC);
    }
    __syncthreads();
    for (int c = 0; c < nchunks; ++c) {
        const int buf = c & 1;
        multiply(buf);
        if (c + 1 < nchunks) {
            stage_w16(buf ^ 1, breg0);
            stage(buf ^ 1);
        }
        if (c + 2 < nchunks) {
            fetch_w16((c + 2) * KC, breg0);
            fetch((c + 2) * KC);
        }
        __syncthreads();
    }

    const int k = kt0 + wn * 32 + l32;
    if (k >= g.K) return;
#pragma unroll
    for (int m = 0; m < MT; ++m) {
        const int bt = b0 + (wm * MT + m) * 32;
#pragma unroll
        for (int grp = 0; grp < 4; ++grp) {
            const int bb = bt + grp * 8 + half * 4;
            float v[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                v[i] = 0.f;
                if (bb + i < g.B) {
                    const i64 idx = ((i64)w * g.B + bb + i) * g.K + k;
                    const bf16_t hp = g.hprev[idx];
                    const bool pos = (hp & 0x7fffu) != 0 && (hp & 0x8000u) == 0;   // ReLU'(z) = [z > 0]
                    v[i] = pos ? acc[m][grp * 4 + i] : 0.f;
                    g.dzp[idx] = f2bf(v[i]);
                }
            }
            if (bb < g.Bp) {
                u32x2 p = {pack2(v[0], v[1]), pack2(v[2], v[3])};
                *reinterpret_cast<u32x2 *>(g.dzpt + tfrag_worker(w, g.K, g.Bp) + tfrag_off(k, bb, g.Bp)) = p;
            }
        }
    }
}

// ------------------------------------------------ backward of the class layer in one launch
// A layer with at most 16 outputs (the 10 classes) has next to no arithmetic: its weight gradient, its data gradient
// and the bias gradient of the layer below are each a few FMAs per element of the activation matrix h below it, and
// as three launches of the tiled kernels above they are 3/4 padding.  Here a thread owns one column k of h and the
// SG groups of 256 / SG threads of a workgroup deal the samples among themselves in octets (group s takes octets s,
// s + SG, ...; SG = 4 for minibatches of 64 rows and more, else 1: a thread walks all samples):
// dW[c][k] += dZ[b][c] h[b][k], dZ'[b][k] = [h[b][k] > 0] sum_c dZ[b][c] bf16(W[c][k]), db'[k] += bf16(dZ'[b][k]) -
// the operands and roundings of the kernels it replaces (bf16 deltas, activations and weights, fp32 sums).  A thread
// requests up to 32 samples of its column at once (the launch is bound by that round trip, not by arithmetic); the
// SG partial sums of dW and db' meet in LDS and are added in group order.  The worker's deltas sit in LDS as fp32.
// grid (ceil(K SG / 256), n), block 256; C <= CP <= 16 (the arithmetic is unrolled for CP outputs), Bp <= 256.
struct ClassBwdArgs {
    const bf16_t *dz;     // [n][B][C] deltas of the class layer
    const bf16_t *h;      // [n][B][K] post-ReLU activations of the layer below
    const float *X;
    float *G;
    i64 ld, woff, boff, boff_below;
    bf16_t *dzp;          // [n][B][K] deltas of the layer below, or null when nothing reads them
    bf16_t *dzpt;         // their T copy
    int B, Bp, K, C;
    // with the softmax in the class layer's forward launch: its per-workgroup loss sums, to be added up here
    const float *loss_part;   // [n][chunks] or null
    int chunks;
    float *loss;              // [n]
};

template <int CP, int SG>
__global__ void __launch_bounds__(256) mlp_class_bwd_kernel(ClassBwdArgs g)
{
    constexpr int NCOL = 256 / SG;
    __shared__ float dzs[256][16];
    __shared__ float red[SG > 1 ? SG : 1][CP + 1][SG > 1 ? NCOL : 1];
    const int lane = threadIdx.x % NCOL, sg = threadIdx.x / NCOL;
    const int w = blockIdx.y, k = blockIdx.x * NCOL + lane;
    const bool k_ok = k < g.K;
    for (int e = threadIdx.x; e < g.Bp * 16; e += 256) {
        const int b = e >> 4, c = e & 15;
        dzs[b][c] = (b < g.B && c < g.C) ? bf2f(g.dz[((i64)w * g.B + b) * g.C + c]) : 0.f;
    }
    __syncthreads();
    if (blockIdx.x == 0 && (int)threadIdx.x < g.C) {   // bias gradient of the class layer
        float s = 0.f;
        for (int b = 0; b < g.B; ++b) s += dzs[b][threadIdx.x];
        g.G[(i64)w * g.ld + g.boff + threadIdx.x] = s;
    }
    if (blockIdx.x == 0 && threadIdx.x == 64 && g.loss_part && g.loss) {   // the worker's loss: partial sums in order
        float s = 0.f;
        for (int c = 0; c < g.chunks; ++c) s += g.loss_part[(i64)w * g.chunks + c];
        g.loss[w] = s * (1.0f / (float)g.B);
    }
    float wb[CP], gw[CP];
#pragma unroll
    for (int c = 0; c < CP; ++c) {
        wb[c] = (k_ok && c < g.C) ? bf2f(f2bf(g.X[(i64)w * g.ld + g.woff + (i64)c * g.K + k])) : 0.f;
        gw[c] = 0.f;
    }
    const bf16_t *hp = g.h + (i64)w * g.B * g.K + (k_ok ? k : 0);
    bf16_t *dst_t = g.dzpt + tfrag_worker(w, g.K, g.Bp);
    float db = 0.f;
    const int noct = g.Bp >> 3;
    for (int base = 0; base < noct; base += 4 * SG) {
        bf16_t hv[4][8];
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            const int b0 = (base + SG * jj + sg) * 8;
#pragma unroll
            for (int j = 0; j < 8; ++j) hv[jj][j] = b0 + j < g.B ? hp[(i64)(b0 + j) * g.K] : (bf16_t)0;
        }
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
            const int oc = base + SG * jj + sg;
            if (oc >= noct) break;
            const int b0 = oc * 8;
            unsigned short out[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int b = b0 + j;
                const bf16_t hraw = hv[jj][j];
                const float hf = bf2f(hraw);
                float da = 0.f;
#pragma unroll
                for (int c = 0; c < CP; ++c) {
                    const float d = dzs[b][c];
                    da = __builtin_fmaf(d, wb[c], da);
                    gw[c] = __builtin_fmaf(d, hf, gw[c]);
                }
                const bool pos = (hraw & 0x7fffu) != 0 && (hraw & 0x8000u) == 0;   // ReLU'(z) = [z > 0]
                const bf16_t v = f2bf(pos ? da : 0.f);
                out[j] = v;
                db += bf2f(v);
                if (g.dzp && b < g.B && k_ok) g.dzp[((i64)w * g.B + b) * g.K + k] = v;
            }
            const u32x4 pk = {(unsigned)out[0] | ((unsigned)out[1] << 16), (unsigned)out[2] | ((unsigned)out[3] << 16),
                              (unsigned)out[4] | ((unsigned)out[5] << 16), (unsigned)out[6] | ((unsigned)out[7] << 16)};
            if (k_ok) *reinterpret_cast<u32x4 *>(dst_t + tfrag_off(k, b0, g.Bp)) = pk;
        }
    }
    if (SG == 1) {
        if (!k_ok) return;
#pragma unroll
        for (int c = 0; c < CP; ++c)
            if (c < g.C) g.G[(i64)w * g.ld + g.woff + (i64)c * g.K + k] = gw[c];
        g.G[(i64)w * g.ld + g.boff_below + k] = db;
        return;
    }
#pragma unroll
    for (int c = 0; c < CP; ++c) red[sg][c][lane] = gw[c];
    red[sg][CP][lane] = db;
    __syncthreads();
    if (!k_ok) return;
    // the groups' partial sums in group order; group s writes the outputs c = s, s + SG, ... (c = CP: the bias below)
    for (int c = sg; c <= CP; c += SG) {
        float t = red[0][c][lane];
#pragma unroll
        for (int q = 1; q < SG; ++q) t += red[q][c][lane];
        if (c == CP) g.G[(i64)w * g.ld + g.boff_below + k] = t;
        else if (c < g.C) g.G[(i64)w * g.ld + g.woff + (i64)c * g.K + k] = t;
    }
}

int round_up(int v, int m) { return (v + m - 1) / m * m; }

struct Tiling { int wm, wn, mt; };
Tiling pick_tiling(int B)
{
    if (B <= 32) return {1, 4, 1};
    if (B <= 64) return {1, 4, 2};
    return {2, 2, 2};
}

template <int WM, int WN, int MT>
dpsgd_status fwd_launch(hipStream_t s, int n, const FwdArgs &a, bool vec, bool last)
{
    constexpr int TO = 32 * WN, MBLK = 32 * WM * MT;
    if (WM == 2 && WN == 2 && MT == 2 && vec && !a.wb) {   // 128-row minibatch blocks: 512-byte row pieces
        dim3 grid((unsigned)((a.O + 63) / 64), (unsigned)((a.B + 127) / 128), (unsigned)n);
        const size_t shm = (size_t)(64 + 128) * PITCHW * sizeof(bf16_t);
        if (last) hipLaunchKernelGGL(mlp_fwd_wide_kernel<true>, grid, dim3(256), shm, s, a);
        else hipLaunchKernelGGL(mlp_fwd_wide_kernel<false>, grid, dim3(256), shm, s, a);
        return hip_status(hipGetLastError());
    }
    dim3 grid((unsigned)((a.O + TO - 1) / TO), (unsigned)((a.B + MBLK - 1) / MBLK), (unsigned)n);
    const size_t shm = (size_t)2 * (TO + MBLK) * PITCH * sizeof(bf16_t);
    if (vec && last) hipLaunchKernelGGL((mlp_fwd_kernel<WM, WN, MT, true, true>), grid, dim3(256), shm, s, a);
    else if (vec) hipLaunchKernelGGL((mlp_fwd_kernel<WM, WN, MT, true, false>), grid, dim3(256), shm, s, a);
    else if (last) hipLaunchKernelGGL((mlp_fwd_kernel<WM, WN, MT, false, true>), grid, dim3(256), shm, s, a);
    else hipLaunchKernelGGL((mlp_fwd_kernel<WM, WN, MT, false, false>), grid, dim3(256), shm, s, a);
    return hip_status(hipGetLastError());
}

dpsgd_status fwd_ksplit_launch(hipStream_t s, int n, const FwdArgs &a, bool vec, bool last)
{
    dim3 grid((unsigned)((a.O + 63) / 64), (unsigned)((a.B + 31) / 32), (unsigned)n);
    const size_t shm = (size_t)2 * (64 + 32) * PITCH2 * sizeof(bf16_t);
    if (a.wb && vec && !last && (a.O % 64) == 0 && (a.K % 128) == 0)
        hipLaunchKernelGGL((mlp_fwd_ksplit_kernel<true, false, true>), grid, dim3(256), shm, s, a);
    else if (vec && last) hipLaunchKernelGGL((mlp_fwd_ksplit_kernel<true, true, false>), grid, dim3(256), shm, s, a);
    else if (vec) hipLaunchKernelGGL((mlp_fwd_ksplit_kernel<true, false, false>), grid, dim3(256), shm, s, a);
    else if (last) hipLaunchKernelGGL((mlp_fwd_ksplit_kernel<false, true, false>), grid, dim3(256), shm, s, a);
    else hipLaunchKernelGGL((mlp_fwd_ksplit_kernel<false, false, false>), grid, dim3(256), shm, s, a);
    return hip_status(hipGetLastError());
}

template <int WM, int WN, int MT>
dpsgd_status dgrad_launch(hipStream_t s, int n, const DgradArgs &a, bool vec)
{
    constexpr int TK = 32 * WN, MBLK = 32 * WM * MT;
    dim3 grid((unsigned)((a.K + TK - 1) / TK), (unsigned)((a.B + MBLK - 1) / MBLK), (unsigned)n);
    const size_t shm = (size_t)2 * (KC * (TK + 8) + MBLK * PITCH) * sizeof(bf16_t);
    if (a.wb && vec && (a.O % KC) == 0 && (a.K % TK) == 0)
        hipLaunchKernelGGL((mlp_dgrad_kernel<WM, WN, MT, true, true>), grid, dim3(256), shm, s, a);
    else if (vec) hipLaunchKernelGGL((mlp_dgrad_kernel<WM, WN, MT, true>), grid, dim3(256), shm, s, a);
    else hipLaunchKernelGGL((mlp_dgrad_kernel<WM, WN, MT, false>), grid, dim3(256), shm, s, a);
    return hip_status(hipGetLastError());
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// gb[o] = sum_b dZ[b][o] from the transposed copy (used when the weight gradient itself is fused away)
__global__ void __launch_bounds__(256)
bias_grad_bf16_kernel(const bf16_t *__restrict__ dzt, int O, int Bp, float *__restrict__ G, i64 ld, i64 boff)
{
    const int o = blockIdx.x * 256 + threadIdx.x, w = blockIdx.y;
    if (o >= O) return;
    const bf16_t *p = dzt + tfrag_worker(w, O, Bp);
    float s = 0.f;
    for (int b = 0; b < Bp; b += 8) {
        const bf16_t *q = p + tfrag_off(o, b, Bp);
#pragma unroll
        for (int j = 0; j < 8; ++j) s += bf2f(q[j]);
    }
    G[(i64)w * ld + boff + o] = s;
}

// ------------------------------------------------- weight gradient fused into mix + step (ring)
// X[i][tile] <- w (X[i-1] + X[i] + X[i+1])[tile] - gamma * (dZ_i^T A_i)[tile] for one weight matrix,
// in place, without the gradient ever reaching HBM (Algorithm 1 steps 3-5 in one pass; footnote [b]:
// steps 3 and 4 are independent).  A wave owns a 32 x 32 tile of the matrix for ALL workers and
// walks the ring keeping x_{i-1}, x_i, x_{i+1} in registers in the MFMA accumulator layout; the
// worker's gradient tile comes from two bf16 MFMAs per 16 minibatch rows on L2-resident operands.
struct FusedArgs {
    float *X;
    i64 ld, woff;
    const bf16_t *dzt;   // T copy of dZ [n][B][O]
    const bf16_t *at;    // T copy of A  [n][B][K]
    int n, K, O, Bp;
    float w, gamma;
    double *partials;    // one per wave (CONS only)
    bf16_t *shadow;      // SHADOW: [n][O/32][K/32][32][32] bf16, receives the rounding of the new weights
};

template <bool CONS, bool SHADOW>
__global__ void __launch_bounds__(256, 3) mlp_fused_ring_kernel(FusedArgs a)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int k0 = blockIdx.x * 128 + wave * 32, o0 = blockIdx.y * 32;
    const int steps = a.Bp / 16;
    // element v of this lane: row o0 + (v/4)*8 + half*4 + v%4, column k0 + l32
    float *xt = a.X + a.woff + (i64)(o0 + half * 4) * a.K + k0 + l32;
    auto row_off = [&](int v) { return (i64)((v >> 2) * 8 + (v & 3)) * a.K; };
    const bf16_t *ap = a.dzt + (i64)(o0 >> 5) * steps * 512 + lane * 8;
    const bf16_t *bp = a.at + (i64)(k0 >> 5) * steps * 512 + lane * 8;

    // xh: worker 0's original tile (the ring's wrap-around, and the shift of the consensus sums);
    // xn / xf: the tiles of workers i+1 and i+2, fetched one and two steps ahead
    float xm[16], xc[16], xh[16], xn[16], xf[16], s1[16], s2[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        xm[v] = xt[(i64)(a.n - 1) * a.ld + row_off(v)];
        xc[v] = xt[row_off(v)];
        xh[v] = xc[v];
        xn[v] = xt[(i64)(1 % a.n) * a.ld + row_off(v)];
        s1[v] = 0.f;
    }
    // The operands of a worker's first 32 minibatch rows (the minibatch is padded to a multiple of 32, so there
    // are always two steps) are fetched while the previous worker is computed; issued before the tile of worker
    // i + 2, they can be waited for without waiting for that tile.  Both fetches are unconditional so that the
    // wait counts stay exact: past the last worker the tile fetch reads one cached line of the operand array
    // instead (values never used), the operand fetch repeats the last worker's.
    bf16x8 pa0 = frag(ap), pb0 = frag(bp), pa1 = frag(ap + 512), pb1 = frag(bp + 512);
    // SHADOW: byte offset of this lane's pair of columns inside the wave's 32 x 32 bf16 tile; the odd lane writes one
    // row further down than the even lane
    const unsigned shadow_lane = (unsigned)(((half * 4 + (l32 & 1)) * 32 + (l32 & ~1)) * 2);
    for (int i = 0; i < a.n; ++i) {
        {
            const bool far = i + 2 < a.n;
            const float *src = far ? xt + (i64)(i + 2) * a.ld : reinterpret_cast<const float *>(a.dzt) + lane;
            const i64 rs = far ? (i64)a.K : 0;
#pragma unroll
            for (int v = 0; v < 16; ++v) xf[v] = __builtin_nontemporal_load(src + ((v >> 2) * 8 + (v & 3)) * rs);
        }
        f32x16 acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.f;
        const bf16_t *ai = ap + (i64)i * a.O * a.Bp, *bi = bp + (i64)i * a.K * a.Bp;
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pa0, pb0, acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pa1, pb1, acc, 0, 0, 0);
        for (int st = 2; st < steps; st += 2) {
            pa0 = frag(ai + st * 512);
            pb0 = frag(bi + st * 512);
            pa1 = frag(ai + st * 512 + 512);
            pb1 = frag(bi + st * 512 + 512);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pa0, pb0, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pa1, pb1, acc, 0, 0, 0);
        }
        {
            const int nw = i + 1 < a.n ? i + 1 : i;
            const bf16_t *an = ap + (i64)nw * a.O * a.Bp, *bn = bp + (i64)nw * a.K * a.Bp;
            pa0 = frag(an);
            pb0 = frag(bn);
            pa1 = frag(an + 512);
            pb1 = frag(bn + 512);
        }
        const bool last = i + 1 == a.n;
        float *dst = xt + (i64)i * a.ld;
        // SHADOW: rows v and v+1 of two neighbouring lanes (columns c, c+1) are exchanged so that the even lane holds
        // both columns of row v and the odd lane both of row v+1: 4-byte stores of two bf16 values
        // (a wave-uniform base plus a 32-bit byte offset per lane; the copy is stored in 32 x 32 tiles, so the wave's
        // tile is 2 KB of consecutive memory and a store instruction covers two whole cache lines)
        char *sbase = SHADOW ? reinterpret_cast<char *>(a.shadow + (i64)i * a.O * a.K + shadow_tile(o0, k0, a.K)) : nullptr;
        float keep = 0.f;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const float nxt = last ? xh[v] : xn[v];   // the ring closes on worker 0's original tile
            // the order and roundings of the ring mix kernel: three fused multiply-adds after the first product
            float mix = a.w * xm[v];
            mix = __builtin_fmaf(a.w, xc[v], mix);
            mix = __builtin_fmaf(a.w, nxt, mix);
            const float o = __builtin_fmaf(-a.gamma, acc[v], mix);
            __builtin_nontemporal_store(o, dst + row_off(v));
            if (CONS) {   // per element the sum of (x - shift); the squares need no per-element sum
                const float e = o - xh[v];
                s1[v] += e;
                s2[v & 3] += e * e;
            }
            if (SHADOW) {
                if (!(v & 1)) {
                    keep = o;
                } else {
                    const bool odd = l32 & 1;
                    const float send = odd ? keep : o;   // the odd lane gives away row v-1, the even lane row v
                    const float recv = __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(send), 0xB1, 0xf, 0xf, true));
                    const unsigned pk = odd ? pack2(recv, o) : pack2(keep, recv);
                    const unsigned rowb = (unsigned)(((v >> 2) * 8 + (v & 3) - 1) * 32) * 2u;   // row of v - 1 inside the tile, bytes
                    __builtin_nontemporal_store(pk, reinterpret_cast<unsigned *>(sbase + (shadow_lane + rowb)));
                }
            }
            xm[v] = xc[v];
            xc[v] = nxt;
            xn[v] = xf[v];   // (a clamped fetch is never used: worker n-1's successor is taken from xh)
        }
    }
    if (CONS) {
        float m2 = (s2[0] + s2[1]) + (s2[2] + s2[3]);
        const float inv_n = 1.0f / (float)a.n;
#pragma unroll
        for (int v = 0; v < 16; ++v) m2 -= s1[v] * s1[v] * inv_n;
        double t = (double)m2;
        for (int off = 32; off > 0; off >>= 1) t += __shfl_down(t, off, 64);
        if (lane == 0) a.partials[((i64)blockIdx.y * gridDim.x + blockIdx.x) * 4 + wave] = t;
    }
}

// The 32 x 32-tile pass for minibatches of more than 32 rows (4 to 8 operand steps per worker).  Fetched into
// registers two steps at a time, the operands cost a wave one L2 round trip per pair of steps, one after the
// other.  Here a worker's operands - the 32 rows of dZ^T all four waves share and each wave's 32 columns of the
// activations, steps KB each, consecutive in the fragment-ordered copies - travel from L2 straight into LDS
// (16 bytes per lane, no registers), asynchronously: they are requested as soon as every wave has read the
// previous worker's from LDS, and land while the wave forms and stores that worker's update.  One round trip per
// worker, hidden; two workgroup barriers per worker.  grid (K / 128, O / 32), block 256, dynamic LDS 5 * steps KB.
template <bool CONS>
__global__ void __launch_bounds__(256, 3) mlp_fused_ring_lds_kernel(FusedArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char fused_lds[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int l32 = lane & 31, half = lane >> 5;
    const int k0 = blockIdx.x * 128 + wave * 32, o0 = blockIdx.y * 32;
    const int steps = a.Bp / 16;
    u32x4 *lds_a = reinterpret_cast<u32x4 *>(fused_lds);               // [steps][64]: dZ^T rows o0 .. o0 + 31
    u32x4 *lds_b = lds_a + (1 + wave) * steps * 64;                    // [steps][64]: this wave's activation columns
    // element v of this lane: row o0 + (v/4)*8 + half*4 + v%4, column k0 + l32
    float *xt = a.X + a.woff + (i64)(o0 + half * 4) * a.K + k0 + l32;
    auto row_off = [&](int v) { return (i64)((v >> 2) * 8 + (v & 3)) * a.K; };
    const bf16_t *ap = a.dzt + (i64)(o0 >> 5) * steps * 512 + lane * 8;
    const bf16_t *bp = a.at + (i64)(k0 >> 5) * steps * 512 + lane * 8;
    // worker w's operands on their way to LDS: this wave's own activation steps and every fourth step of dZ^T
    auto request_ops = [&](int w) {
        const bf16_t *aw = ap + (i64)w * a.O * a.Bp, *bw = bp + (i64)w * a.K * a.Bp;
        for (int st = 0; st < steps; ++st) __builtin_amdgcn_global_load_lds(bw + st * 512, lds_b + st * 64, 16, 0, 0);
        for (int st = wave; st < steps; st += 4) __builtin_amdgcn_global_load_lds(aw + st * 512, lds_a + st * 64, 16, 0, 0);
    };

    float xm[16], xc[16], xh[16], xn[16], xf[16], s1[16], s2[4] = {0.f, 0.f, 0.f, 0.f};
    request_ops(0);
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        xm[v] = xt[(i64)(a.n - 1) * a.ld + row_off(v)];
        xc[v] = xt[row_off(v)];
        xh[v] = xc[v];
        xn[v] = xt[(i64)(1 % a.n) * a.ld + row_off(v)];
        s1[v] = 0.f;
    }
    __builtin_amdgcn_s_waitcnt(0);   // everything requested so far has arrived (vmcnt = 0)
    __syncthreads();
    for (int i = 0; i < a.n; ++i) {
        {   // the tile of worker i + 2 (past the last worker: one cached line of the operand array, values never used)
            const bool far = i + 2 < a.n;
            const float *src = far ? xt + (i64)(i + 2) * a.ld : reinterpret_cast<const float *>(a.dzt) + lane;
            const i64 rs = far ? (i64)a.K : 0;
#pragma unroll
            for (int v = 0; v < 16; ++v) xf[v] = __builtin_nontemporal_load(src + ((v >> 2) * 8 + (v & 3)) * rs);
        }
        f32x16 acc;
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[v] = 0.f;
        {   // two steps at a time (the minibatch is padded to a multiple of 32), the next pair read ahead of the MFMAs
            u32x4 pa0 = lds_a[lane], pb0 = lds_b[lane], pa1 = lds_a[64 + lane], pb1 = lds_b[64 + lane];
            for (int st = 2; st < steps; st += 2) {
                const u32x4 na0 = lds_a[st * 64 + lane], nb0 = lds_b[st * 64 + lane];
                const u32x4 na1 = lds_a[st * 64 + 64 + lane], nb1 = lds_b[st * 64 + 64 + lane];
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, pa0), __builtin_bit_cast(bf16x8, pb0), acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, pa1), __builtin_bit_cast(bf16x8, pb1), acc, 0, 0, 0);
                pa0 = na0; pb0 = nb0; pa1 = na1; pb1 = nb1;
            }
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, pa0), __builtin_bit_cast(bf16x8, pb0), acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, pa1), __builtin_bit_cast(bf16x8, pb1), acc, 0, 0, 0);
        }
        __syncthreads();   // every wave has read worker i's operands
        if (i + 1 < a.n) request_ops(i + 1);
        const bool last = i + 1 == a.n;
        float *dst = xt + (i64)i * a.ld;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const float nxt = last ? xh[v] : xn[v];   // the ring closes on worker 0's original tile
            // the order and roundings of the ring mix kernel: three fused multiply-adds after the first product
            float mix = a.w * xm[v];
            mix = __builtin_fmaf(a.w, xc[v], mix);
            mix = __builtin_fmaf(a.w, nxt, mix);
            const float o = __builtin_fmaf(-a.gamma, acc[v], mix);
            __builtin_nontemporal_store(o, dst + row_off(v));
            if (CONS) {
                const float e = o - xh[v];
                s1[v] += e;
                s2[v & 3] += e * e;
            }
            xm[v] = xc[v];
            xc[v] = nxt;
            xn[v] = xf[v];
        }
        // The next worker's operands must be in LDS, for every wave, before anyone reads them.  (This also waits for
        // the 16 stores above, which were issued after the operand requests; the compiler puts the same full wait in
        // front of the barrier by itself.)
        __builtin_amdgcn_s_waitcnt(0);
        __syncthreads();
    }
    if (CONS) {
        float m2 = (s2[0] + s2[1]) + (s2[2] + s2[3]);
        const float inv_n = 1.0f / (float)a.n;
#pragma unroll
        for (int v = 0; v < 16; ++v) m2 -= s1[v] * s1[v] * inv_n;
        double t = (double)m2;
        for (int off = 32; off > 0; off >>= 1) t += __shfl_down(t, off, 64);
        if (lane == 0) a.partials[((i64)blockIdx.y * gridDim.x + blockIdx.x) * 4 + wave] = t;
    }
}

// The same pass for minibatches of at most 32 rows with a workgroup tile of [16 rows][1 KB]: every load and store
// instruction of a wave covers 1 KB of one row of the weight matrix (the 32 x 32 layout above touches 128-byte
// pieces of two rows), which streams ~10 % faster from HBM.  Wave wv owns rows o0 + 4 wv .. + 3 and all 256 columns,
// lane l the four columns k0 + 4 l .. + 3.  The gradient of that [4][256] strip comes from v_mfma_f32_4x4x4_16B_bf16:
// 16 independent 4 x 4 blocks, block l / 4 taking row l % 4 of A from lane l and column l % 4 of B, so with the same
// four rows of dZ^T in every block and tile t handing column 4 l + t of the activations to lane l, register r of
// tile t is the gradient at (row r, column 4 l + t): the four tiles are the four components of the lane's float4.
// A strip that thin reuses nothing, so the operands go through LDS: per worker the 256 activation columns x 32
// samples (16 KB, one consecutive block of the T copy) and the 16 dZ rows, fetched one worker ahead into registers
// and written to the other of two buffers; one barrier per worker.  grid (K / 256, O / 16), block 256.
constexpr int ROWS_PLANE = 66;   // 16-byte units per (sample octet, tile) plane of the activation buffer: 64 lanes + 2 of padding

// RS: which elements of the workgroup's [16 rows][256 cols] a wave owns.  0: rows 4 wave .. + 3, all 256 columns (an
// instruction covers 1 KB of one row).  1 or 2 (K = 8192 or 4096, i.e. RS rows = 32 KB): waves 2 g and 2 g + 1 share
// eight rows RS apart and take 128 columns each; an instruction covers two 512-byte pieces of rows RS apart (lanes
// 0-31 / 32-63) and the wave's eight pieces lie 32 KB apart, which the HBM channels serve faster (see
// mix_ring_fat_kernel): an in-place walk with this kernel's traffic moves 6.1 TB/s that way against 5.75.
// The same elements get the same sums: the three maps give the same bits.
template <bool CONS, bool SHADOW, int RS>
__global__ void __launch_bounds__(256, 3) mlp_fused_ring_rows_kernel(FusedArgs a)
{
    __shared__ u32x4 bt[2][16 * ROWS_PLANE];   // [octet][tile t][lane]: samples 8 octet .. + 7 of column 4 lane + t
    __shared__ u32x4 at[2][64];                // [octet][row 0..15] of dZ^T
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    // RS 3 (rows of 4, 8 or 12 KB: K a multiple of 1024): the workgroup owns 16 rows of a block of 32, wave rows 8 apart
    // (a multiple of 32 KB), whole 1 KB pieces: rows 4 half + wave + 8 r of block blockIdx.y / 2, half = blockIdx.y % 2
    const int k0 = blockIdx.x * 256, o0 = RS == 3 ? (blockIdx.y >> 1) * 32 : blockIdx.y * 16;
    // element (r, t) of this lane: row o0 + row0 + rstep r, column k0 + col0 + t
    //   RS 0: row0 = 4 wave, rstep = 1, col0 = 4 lane
    //   RS 2: row0 = wave / 2 + 2 (lane / 32), rstep = 4 (rows wave / 2 + 2 j, j = 2 r + lane / 32), col0 = 128 (wave % 2) + 4 (lane % 32)
    //   RS 1: row0 = 8 (wave / 2) + lane / 32, rstep = 2 (rows 8 (wave / 2) + j)
    const int row0 = RS == 0 ? 4 * wave : RS == 2 ? (wave >> 1) + 2 * (lane >> 5) : RS == 1 ? 8 * (wave >> 1) + (lane >> 5)
                                                                                   : 4 * (int)(blockIdx.y & 1) + wave;
    constexpr int rstep = RS == 0 ? 1 : RS == 2 ? 4 : RS == 1 ? 2 : 8;
    // the workgroup's 16 rows of dZ^T sit in LDS slots 0 .. 15; slot of this lane's row r: slot0 + sstep r
    const int slot0 = RS == 3 ? wave : row0;
    constexpr int sstep = RS == 3 ? 4 : rstep;
    const int col0 = (RS == 0 || RS == 3) ? 4 * lane : 128 * (wave & 1) + 4 * (lane & 31);
    const int bslot_read = col0 >> 2;   // this lane's slot in a plane of the activation buffer
    const i64 rstride = (i64)rstep * a.K;
    float *xt = a.X + a.woff + (i64)(o0 + row0) * a.K + k0 + col0;
    auto load_tile = [&](const float *p, i64 rs, float (&x)[16]) {
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(p + r * rs));
            x[4 * r] = v.x; x[4 * r + 1] = v.y; x[4 * r + 2] = v.z; x[4 * r + 3] = v.w;
        }
    };
    // operands in fragment order (tfrag_off) with Bp = 32: per 32 rows [sample group of 16][half][row][8 samples].
    // Activations: the block of columns k0 .. k0 + 255 is 1024 consecutive 16-byte units; unit u = tid + 256 q is
    // column (u / 128) * 32 + u % 32, octet (u / 32) % 4, and goes to plane (octet, column % 4), slot column / 4.
    const u32x4 *bsrc = reinterpret_cast<const u32x4 *>(a.at + (i64)(k0 >> 5) * 1024) + tid;
    const int bslot = (((tid >> 5) & 3) * 4 + (tid & 3)) * ROWS_PLANE + (tid >> 7) * 8 + ((tid & 31) >> 2);
    // dZ^T: lane (octet = lane / 16, row = lane % 16) of every wave fetches one unit; wave 0 writes them
    const int aoc = lane >> 4;
    // slot lane % 16 holds row (o0 % 32) + slot, or (RS 3) row 4 half + slot % 4 + 8 (slot / 4) of the block
    const int arow = RS == 3 ? 4 * (int)(blockIdx.y & 1) + (lane & 3) + 8 * ((lane & 15) >> 2) : (o0 & 31) + (lane & 15);
    const u32x4 *asrc = reinterpret_cast<const u32x4 *>(
        a.dzt + ((i64)(o0 >> 5) * 2 + (aoc >> 1)) * 512 + (aoc & 1) * 256 + arow * 8);
    const i64 b_worker = (i64)a.K * 4, a_worker = (i64)a.O * 4;   // 16-byte units per worker (32 samples x 2 bytes)
    u32x4 breg[4], areg;
    auto fetch_ops = [&](int worker) {
#pragma unroll
        for (int q = 0; q < 4; ++q) breg[q] = bsrc[worker * b_worker + 256 * q];
        areg = asrc[worker * a_worker];
    };
    auto stage_ops = [&](int buf) {
#pragma unroll
        for (int q = 0; q < 4; ++q) bt[buf][bslot + 16 * q] = breg[q];
        if (wave == 0) at[buf][lane] = areg;
    };

    // Four tile buffers rotate through the roles (previous worker, this worker, next worker, being fetched): the tile
    // requested at the start of step i is first read in the epilogue of step i + 1, a whole step later, and no register
    // is copied from one role to the next (a copy at the end of step i would have to wait for the fetch of step i).
    float ta[16], tb[16], tc[16], td[16], xh[16], s1[16], s2[4] = {0.f, 0.f, 0.f, 0.f};
    fetch_ops(0);
    load_tile(xt + (i64)(a.n - 1) * a.ld, rstride, ta);
    load_tile(xt, rstride, tb);
    load_tile(xt + (i64)(1 % a.n) * a.ld, rstride, tc);
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        xh[v] = tb[v];
        s1[v] = 0.f;
    }
    stage_ops(0);
    fetch_ops(1 < a.n ? 1 : 0);
    __syncthreads();
    // one worker: xm, xc, xn hold the tiles of workers i - 1, i, i + 1; xf receives worker i + 2's.  The operands of
    // worker i + 1 were requested before the barrier that ended step i - 1 (a step and a barrier ahead of the moment
    // they are written to LDS, so that no wave reaches the barrier late because of them).  Both fetches are
    // unconditional (exact wait counts): past the last worker the operand fetch repeats the last worker's and the tile
    // fetch reads one cached line of the operand array (values never used); the operands are requested before the
    // tile so that they can be waited for without waiting for the tile.
    auto step = [&](int i, const float (&xm)[16], const float (&xc)[16], const float (&xn)[16], float (&xf)[16]) {
        const int buf = i & 1;
        {
            const bool far = i + 2 < a.n;
            const float *src = far ? xt + (i64)(i + 2) * a.ld : reinterpret_cast<const float *>(a.dzt) + 4 * lane;
            load_tile(src, far ? rstride : 0, xf);
        }
        f32x4 acc[4];
#pragma unroll
        for (int t = 0; t < 4; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll 1
        for (int oc = 0; oc < 4; ++oc) {
            const u32x4 av = at[buf][oc * 16 + slot0 + sstep * (lane & 3)];
            const s16x4 alo = __builtin_bit_cast(s16x4, u32x2{av.x, av.y}), ahi = __builtin_bit_cast(s16x4, u32x2{av.z, av.w});
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const u32x4 bv = bt[buf][(oc * 4 + t) * ROWS_PLANE + bslot_read];
                acc[t] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(alo, __builtin_bit_cast(s16x4, u32x2{bv.x, bv.y}), acc[t], 0, 0, 0);
                acc[t] = __builtin_amdgcn_mfma_f32_4x4x4bf16_1k(ahi, __builtin_bit_cast(s16x4, u32x2{bv.z, bv.w}), acc[t], 0, 0, 0);
            }
        }
        const bool last = i + 1 == a.n;
        float *dst = xt + (i64)i * a.ld;
        bf16_t *sdst = SHADOW ? a.shadow + (i64)i * a.O * a.K + shadow_strip(o0 + row0, k0 + col0, a.K) : nullptr;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            f32x4 out;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const int v = 4 * r + t;
                const float nxt = last ? xh[v] : xn[v];   // the ring closes on worker 0's original tile
                float mix = a.w * xm[v];     // order and roundings of the ring mix kernel
                mix = __builtin_fmaf(a.w, xc[v], mix);
                mix = __builtin_fmaf(a.w, nxt, mix);
                const float o = __builtin_fmaf(-a.gamma, acc[t][r], mix);
                out[t] = o;
                if (CONS) {
                    const float e = o - xh[v];
                    s1[v] += e;
                    s2[t] += e * e;
                }
            }
            __builtin_nontemporal_store(out, reinterpret_cast<f32x4 *>(dst + (i64)r * rstride));
            if (SHADOW) {   // the lane's four columns of the row, 8 bytes; the wave's row piece is 512 consecutive bytes
                const u32x2 pk = {pack2(out.x, out.y), pack2(out.z, out.w)};
                __builtin_nontemporal_store(pk, reinterpret_cast<u32x2 *>(sdst + r * rstep * 256));
            }
        }
        stage_ops(buf ^ 1);   // every wave has read this buffer's previous contents before the barrier that ended step i - 1
        fetch_ops(i + 2 < a.n ? i + 2 : a.n - 1);
        __syncthreads();
    };
    for (int i = 0;;) {
        step(i, ta, tb, tc, td);
        if (++i >= a.n) break;
        step(i, tb, tc, td, ta);
        if (++i >= a.n) break;
        step(i, tc, td, ta, tb);
        if (++i >= a.n) break;
        step(i, td, ta, tb, tc);
        if (++i >= a.n) break;
    }
    if (CONS) {
        float m2 = (s2[0] + s2[1]) + (s2[2] + s2[3]);
        const float inv_n = 1.0f / (float)a.n;
#pragma unroll
        for (int v = 0; v < 16; ++v) m2 -= s1[v] * s1[v] * inv_n;
        double t = (double)m2;
        for (int off = 32; off > 0; off >>= 1) t += __shfl_down(t, off, 64);
        if (lane == 0) a.partials[((i64)blockIdx.y * gridDim.x + blockIdx.x) * 4 + wave] = t;
    }
}

// ---------------------------------------- torus fusion, one wave per grid column (C <= 16 columns)
// A workgroup owns one 16 x 32 tile (outputs x inputs) of the weight matrix for ALL workers; wave c takes grid
// column c and walks down it like the ring kernel walks the ring: the tiles of workers (r-1, c), (r, c),
// (r+1, c) stay in its registers.  The row neighbours (r, c-1) and (r, c+1) belong to the neighbouring waves: at
// every grid row each wave publishes its original tile in LDS (two buffers, one workgroup barrier per grid row).
// The gradient tile is two v_mfma_f32_16x16x32_bf16 per 32 minibatch rows, one for the even and one for the odd
// input columns, so that a lane owns two adjacent columns of four rows: every access is 8 bytes per lane and 16
// lanes cover a 128-byte line.  8 registers per tile keep the kernel at 4 waves per SIMD.
// KT such groups of C waves sit side by side along the inputs (KT x 128-byte row segments per workgroup): two for up
// to 8 grid columns, one beyond (the 16 waves of a workgroup are then all columns of one group).
// grid (K / (32 KT), O / 16), block 64 C KT <= 1024, dynamic LDS KT * 2 * C * 2 KB.
struct FusedTorusColArgs {
    float *X;
    i64 ld, woff;
    const bf16_t *dzt;   // T copy of dZ [n][B][O]
    const bf16_t *at;    // T copy of A  [n][B][K]
    int R, C, K, O, Bp;  // grid rows and columns (n = R C)
    float w, gamma;
    double *partials;    // one per workgroup (CONS only)
};

template <bool CONS, int KT, int MAXC>   // MAXC: the most grid columns (waves per group) a launch may have
__global__ void __launch_bounds__(64 * MAXC * KT) mlp_fused_torus_cols_kernel(FusedTorusColArgs a)
{
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int n16 = lane & 15, q = lane >> 4;
    const int C = a.C, R = a.R;
    // KT groups of C waves sit side by side along the inputs: per worker the workgroup touches 16 rows x KT x 128 B
    const int c = wave % C, kt = wave / C;
    f32x4 *tiles = reinterpret_cast<f32x4 *>(smem) + kt * (2 * C * 128);   // per group [2][C][2][64]: a tile as 2 groups of 4 registers
    const int k0 = (blockIdx.x * KT + kt) * 32, o0 = blockIdx.y * 16;
    const int steps = a.Bp / 32;
    // registers 2 i + j of this lane: row o0 + 4 q + i, column k0 + 2 n16 + j
    float *xt = a.X + a.woff + (i64)(o0 + 4 * q) * a.K + k0 + 2 * n16;
    // operands in fragment order (tfrag_off): this lane's row and its samples 32 s + 8 q .. + 7
    auto op_off = [&](int row) {
        return ((i64)(row >> 5) * (a.Bp >> 4) + (q >> 1)) * 512 + (q & 1) * 256 + (row & 31) * 8;
    };
    const bf16_t *ap = a.dzt + op_off(o0 + n16);            // A: 16 outputs
    const bf16_t *be = a.at + op_off(k0 + 2 * n16);         // B of the even columns
    const bf16_t *bo = a.at + op_off(k0 + 2 * n16 + 1);     // B of the odd columns
    const int cl = (c + C - 1) % C, cr = (c + 1) % C;

    float up[8], cur[8], down[8], first[8], last[8], ahead[8], shift[8], s1[8], s2[8];
    auto load_tile = [&](float *dst, int r) {
        const float *p = xt + (i64)(r * C + c) * a.ld;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const f32x2 v = __builtin_nontemporal_load(reinterpret_cast<const f32x2 *>(p + (i64)i * a.K));
            dst[2 * i] = v.x;
            dst[2 * i + 1] = v.y;
        }
    };
    load_tile(up, R - 1);
    load_tile(cur, 0);
    load_tile(down, 1);
#pragma unroll
    for (int v = 0; v < 8; ++v) {
        first[v] = cur[v];
        last[v] = up[v];
        s1[v] = 0.f;
        s2[v] = 0.f;
        shift[v] = 0.f;
    }
    // the operands of the first 32 samples of the next worker are fetched one grid row ahead
    bf16x8 af0 = frag(ap + (i64)c * a.O * a.Bp), be0 = frag(be + (i64)c * a.K * a.Bp), bo0 = frag(bo + (i64)c * a.K * a.Bp);
    for (int r = 0; r < R; ++r) {
        f32x4 *mine = tiles + ((r & 1) * C + c) * 128;
        mine[lane] = (f32x4){cur[0], cur[1], cur[2], cur[3]};
        mine[64 + lane] = (f32x4){cur[4], cur[5], cur[6], cur[7]};
        __syncthreads();
        if (r + 3 < R) load_tile(ahead, r + 2);
        else {   // grid row R - 1 was fetched before the walk and kept: every tile is read once; the last grid row wraps to row 0
#pragma unroll
            for (int v = 0; v < 8; ++v) ahead[v] = r + 3 == R ? last[v] : first[v];
        }
        const int worker = r * C + c;
        f32x4 acc_e = {0.f, 0.f, 0.f, 0.f}, acc_o = {0.f, 0.f, 0.f, 0.f};
        const i64 aw = (i64)worker * a.O * a.Bp, bw = (i64)worker * a.K * a.Bp;
        acc_e = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af0, be0, acc_e, 0, 0, 0);
        acc_o = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af0, bo0, acc_o, 0, 0, 0);
        if (r + 1 < R) {
            const i64 an = aw + (i64)C * a.O * a.Bp, bn = bw + (i64)C * a.K * a.Bp;
            af0 = frag(ap + an);
            be0 = frag(be + bn);
            bo0 = frag(bo + bn);
        }
        for (int st = 1; st < steps; ++st) {
            const bf16x8 af = frag(ap + aw + st * 1024);
            acc_e = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af, frag(be + bw + st * 1024), acc_e, 0, 0, 0);
            acc_o = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af, frag(bo + bw + st * 1024), acc_o, 0, 0, 0);
        }
        const f32x4 *lt = tiles + ((r & 1) * C + cl) * 128, *rt = tiles + ((r & 1) * C + cr) * 128;
        if (CONS && r == 0) {   // the shift of the consensus sums: worker 0's original tile, the same for every wave
            const f32x4 z0 = tiles[lane], z1 = tiles[64 + lane];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                shift[i] = z0[i];
                shift[4 + i] = z1[i];
            }
        }
        float *dst = xt + (i64)worker * a.ld;
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const f32x4 lv = lt[h * 64 + lane], rv = rt[h * 64 + lane];
            float o4[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int v = 4 * h + e;          // register 2 i + j with i = v / 2, j = v % 2
                float m = a.w * up[v];            // one product, then fused multiply-adds: fixed roundings
                m = __builtin_fmaf(a.w, lv[e], m);
                m = __builtin_fmaf(a.w, cur[v], m);
                m = __builtin_fmaf(a.w, rv[e], m);
                m = __builtin_fmaf(a.w, down[v], m);
                const float g = (v & 1) ? acc_o[v >> 1] : acc_e[v >> 1];
                const float o = __builtin_fmaf(-a.gamma, g, m);
                o4[e] = o;
                if (CONS) {
                    const float d = o - shift[v];
                    s1[v] += d;
                    s2[v] += d * d;
                }
                up[v] = cur[v];
                cur[v] = down[v];
                down[v] = ahead[v];
            }
            __builtin_nontemporal_store((f32x2){o4[0], o4[1]}, reinterpret_cast<f32x2 *>(dst + (i64)(2 * h) * a.K));
            __builtin_nontemporal_store((f32x2){o4[2], o4[3]}, reinterpret_cast<f32x2 *>(dst + (i64)(2 * h + 1) * a.K));
        }
    }
    if (CONS) {
        // per element: sums over the C waves of a group first (s1 enters squared), then over the tile
        __syncthreads();
        float *red = reinterpret_cast<float *>(smem) + kt * (C * 1024);   // per group [C][2][8][64]
#pragma unroll
        for (int v = 0; v < 8; ++v) {
            red[((c * 2 + 0) * 8 + v) * 64 + lane] = s1[v];
            red[((c * 2 + 1) * 8 + v) * 64 + lane] = s2[v];
        }
        __syncthreads();
        if (c == 0) {
            const float inv_n = 1.0f / (float)(R * C);
            float m2 = 0.f;
#pragma unroll
            for (int v = 0; v < 8; ++v) {
                float t1 = 0.f, t2 = 0.f;
                for (int w2 = 0; w2 < C; ++w2) {
                    t1 += red[((w2 * 2 + 0) * 8 + v) * 64 + lane];
                    t2 += red[((w2 * 2 + 1) * 8 + v) * 64 + lane];
                }
                m2 += t2 - t1 * t1 * inv_n;
            }
            double t = (double)m2;
            for (int off = 32; off > 0; off >>= 1) t += __shfl_down(t, off, 64);
            if (lane == 0) a.partials[((i64)blockIdx.y * gridDim.x + blockIdx.x) * KT + kt] = t;
        }
    }
}

// ---------------------------------------- fusion for any W of at most 64 workers: every worker's tile in LDS
// The ring and torus kernels above keep a walk's few live tiles in registers; a general sparse W has no such walk.
// Here a workgroup owns a [16 rows][32 M columns] tile of the weight matrix for ALL workers and first brings the n
// tiles into LDS (2 M KB each, in the register order of the lanes that fetched them; n M <= 64, i.e. 128 KB), which
// also makes the in-place update safe: nothing is written before everything has been read.  After the barrier wave
// v takes workers v, v + NW, ...: the gradient tile from v_mfma_f32_16x16x32_bf16 as in the torus kernel (even and
// odd input columns, a lane owns two adjacent floats of four rows), the combination sum_j W_ij x_j from LDS in CSR
// order (one product, then fused multiply-adds: the roundings of the CSR mix kernel), and the row goes back to X.
// The operands of a wave's next worker are fetched while it works on the current one (the first before the barrier).
// grid (K / (32 M), O / 16), block 64 NW (NW = 8 waves, 16 for a slab of more than 64 KB), dynamic LDS
// max(n M 2 KB, NW (8 M + 1) 256 B).
struct FusedSlabArgs {
    float *X;
    i64 ld, woff;
    const bf16_t *dzt;   // T copy of dZ [n][B][O]
    const bf16_t *at;    // T copy of A  [n][B][K]
    const int *rowptr, *colidx;   // W as CSR, device
    const float *vals;
    int n, K, O, Bp;
    float gamma;
    double *partials;    // one per workgroup (CONS only)
};

template <bool CONS, int M, int NW>
__global__ void __launch_bounds__(64 * NW) mlp_fused_slab_kernel(FusedSlabArgs a)
{
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    f32x4 *tiles = reinterpret_cast<f32x4 *>(smem);   // [n][M][2][64]: a tile as 2 groups of 4 registers per lane
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int n16 = lane & 15, q = lane >> 4;
    const int k0 = blockIdx.x * (32 * M), o0 = blockIdx.y * 16;
    const int steps = a.Bp / 32;
    // registers 2 i + j of group m of this lane: row o0 + 4 q + i, column k0 + 32 m + 2 n16 + j
    float *xt = a.X + a.woff + (i64)(o0 + 4 * q) * a.K + k0 + 2 * n16;
    // operands in fragment order (tfrag_off): this lane's row and its samples 32 s + 8 q .. + 7
    auto op_off = [&](int row) {
        return ((i64)(row >> 5) * (a.Bp >> 4) + (q >> 1)) * 512 + (q & 1) * 256 + (row & 31) * 8;
    };
    const bf16_t *ap = a.dzt + op_off(o0 + n16);   // A: 16 outputs
    i64 be_off[M], bo_off[M];                      // B of the even and of the odd columns of group m
#pragma unroll
    for (int m = 0; m < M; ++m) {
        be_off[m] = op_off(k0 + 32 * m + 2 * n16);
        bo_off[m] = op_off(k0 + 32 * m + 2 * n16 + 1);
    }
    bf16x8 af0, be0[M], bo0[M];
    auto fetch_ops = [&](int worker) {
        af0 = frag(ap + (i64)worker * a.O * a.Bp);
#pragma unroll
        for (int m = 0; m < M; ++m) {
            be0[m] = frag(a.at + (i64)worker * a.K * a.Bp + be_off[m]);
            bo0[m] = frag(a.at + (i64)worker * a.K * a.Bp + bo_off[m]);
        }
    };
    fetch_ops(wave < a.n ? wave : 0);

    // ---- all tiles into LDS, four per wave at a time (16 loads in flight per lane)
    const int items = a.n * M;
    for (int t0 = wave; t0 < items; t0 += 4 * NW) {
        f32x2 v[4][4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int t = t0 + u * NW < items ? t0 + u * NW : t0;
            const float *p = xt + (i64)(t / M) * a.ld + 32 * (t % M);
#pragma unroll
            for (int i = 0; i < 4; ++i) v[u][i] = __builtin_nontemporal_load(reinterpret_cast<const f32x2 *>(p + (i64)i * a.K));
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int t = t0 + u * NW;
            if (t < items) {
                tiles[(t * 2 + 0) * 64 + lane] = (f32x4){v[u][0].x, v[u][0].y, v[u][1].x, v[u][1].y};
                tiles[(t * 2 + 1) * 64 + lane] = (f32x4){v[u][2].x, v[u][2].y, v[u][3].x, v[u][3].y};
            }
        }
    }
    __syncthreads();

    float shift[M][8], s1[M][8], s2[2] = {0.f, 0.f};
#pragma unroll
    for (int m = 0; m < M; ++m) {   // the shift of the consensus sums: worker 0's original tile
        const f32x4 z0 = tiles[(m * 2 + 0) * 64 + lane], z1 = tiles[(m * 2 + 1) * 64 + lane];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            shift[m][i] = z0[i];
            shift[m][4 + i] = z1[i];
            s1[m][i] = 0.f;
            s1[m][4 + i] = 0.f;
        }
    }
    for (int w = wave; w < a.n; w += NW) {
        const int e0 = a.rowptr[w], e1 = a.rowptr[w + 1];
        const i64 aw = (i64)w * a.O * a.Bp, bw = (i64)w * a.K * a.Bp;
        f32x4 acc_e[M], acc_o[M];
#pragma unroll
        for (int m = 0; m < M; ++m) {
            acc_e[m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af0, be0[m], (f32x4){0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
            acc_o[m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af0, bo0[m], (f32x4){0.f, 0.f, 0.f, 0.f}, 0, 0, 0);
        }
        fetch_ops(w + NW < a.n ? w + NW : w);   // (past the wave's last worker: the same again, values never used)
        for (int st = 1; st < steps; ++st) {
            const bf16x8 af = frag(ap + aw + st * 1024);
#pragma unroll
            for (int m = 0; m < M; ++m) {
                acc_e[m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af, frag(a.at + bw + be_off[m] + st * 1024), acc_e[m], 0, 0, 0);
                acc_o[m] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(af, frag(a.at + bw + bo_off[m] + st * 1024), acc_o[m], 0, 0, 0);
            }
        }
        float *dst = xt + (i64)w * a.ld;
#pragma unroll
        for (int m = 0; m < M; ++m) {
            float mix[8];
            {
                const int j = a.colidx[e0];
                const float wv = a.vals[e0];
                const f32x4 x0 = tiles[((j * M + m) * 2 + 0) * 64 + lane], x1 = tiles[((j * M + m) * 2 + 1) * 64 + lane];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    mix[i] = wv * x0[i];
                    mix[4 + i] = wv * x1[i];
                }
            }
            for (int e = e0 + 1; e < e1; ++e) {
                const int j = a.colidx[e];
                const float wv = a.vals[e];
                const f32x4 x0 = tiles[((j * M + m) * 2 + 0) * 64 + lane], x1 = tiles[((j * M + m) * 2 + 1) * 64 + lane];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    mix[i] = __builtin_fmaf(wv, x0[i], mix[i]);
                    mix[4 + i] = __builtin_fmaf(wv, x1[i], mix[4 + i]);
                }
            }
            float o8[8];
#pragma unroll
            for (int v = 0; v < 8; ++v) {   // register 2 i + j with i = v / 2, j = v % 2
                const float g = (v & 1) ? acc_o[m][v >> 1] : acc_e[m][v >> 1];
                const float o = __builtin_fmaf(-a.gamma, g, mix[v]);
                o8[v] = o;
                if (CONS) {
                    const float d = o - shift[m][v];
                    s1[m][v] += d;
                    s2[v & 1] += d * d;
                }
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
                __builtin_nontemporal_store((f32x2){o8[2 * i], o8[2 * i + 1]}, reinterpret_cast<f32x2 *>(dst + 32 * m + (i64)i * a.K));
        }
    }
    if (CONS) {
        // per element the sums of (x - shift) over the waves (they enter squared); the squares need no per-element sum
        __syncthreads();
        float *red = reinterpret_cast<float *>(smem);   // [NW][8 M + 1][64]
#pragma unroll
        for (int m = 0; m < M; ++m)
#pragma unroll
            for (int v = 0; v < 8; ++v) red[(wave * (8 * M + 1) + m * 8 + v) * 64 + lane] = s1[m][v];
        red[(wave * (8 * M + 1) + 8 * M) * 64 + lane] = s2[0] + s2[1];
        __syncthreads();
        if (wave == 0) {
            const float inv_n = 1.0f / (float)a.n;
            float m2 = 0.f;
            for (int w2 = 0; w2 < NW; ++w2) m2 += red[(w2 * (8 * M + 1) + 8 * M) * 64 + lane];
            for (int v = 0; v < 8 * M; ++v) {
                float t1 = 0.f;
                for (int w2 = 0; w2 < NW; ++w2) t1 += red[(w2 * (8 * M + 1) + v) * 64 + lane];
                m2 -= t1 * t1 * inv_n;
            }
            double t = (double)m2;
            for (int off = 32; off > 0; off >>= 1) t += __shfl_down(t, off, 64);
            if (lane == 0) a.partials[(i64)blockIdx.y * gridDim.x + blockIdx.x] = t;
        }
    }
}

}  // namespace

// Workspace layout shared by the size query and the launches.
namespace {
struct MlpWs {
    bf16_t *a0 = nullptr, *at0 = nullptr;
    std::vector<bf16_t *> h, ht, dzt;   // per layer output l = 1..L: h/ht for hidden layers, dzt for all
    float *logits = nullptr, *loss_part = nullptr;
    bf16_t *dz[2] = {nullptr, nullptr};
    size_t bytes = 0;
};

MlpWs carve(const dpsgd_ctx *ctx, const dpsgd_model_desc &m, unsigned char *base)
{
    MlpWs w;
    const size_t n = (size_t)ctx->n, B = (size_t)m.batch, Bp = (size_t)round_up(m.batch, 32);
    const int L = (int)m.widths.size() - 1;
    size_t off = 0;
    auto take = [&](size_t b) {
        unsigned char *q = base ? base + off : nullptr;
        off += (b + 255) / 256 * 256;
        return q;
    };
    auto r32 = [](int rows) { return (size_t)((rows + 31) / 32 * 32); };   // rows of a T copy
    if (!m.input_is_bf16) w.a0 = (bf16_t *)take(n * B * (size_t)m.widths[0] * 2);
    w.at0 = (bf16_t *)take(n * r32(m.widths[0]) * Bp * 2);
    w.h.assign(L + 1, nullptr);
    w.ht.assign(L + 1, nullptr);
    w.dzt.assign(L + 1, nullptr);
    size_t widest = 0;
    for (int l = 1; l <= L; ++l) {
        if (l < L) {
            w.h[l] = (bf16_t *)take(n * B * (size_t)m.widths[l] * 2);
            w.ht[l] = (bf16_t *)take(n * r32(m.widths[l]) * Bp * 2);
        }
        w.dzt[l] = (bf16_t *)take(n * r32(m.widths[l]) * Bp * 2);
        widest = widest > (size_t)m.widths[l] ? widest : (size_t)m.widths[l];
    }
    w.logits = (float *)take(n * B * (size_t)m.widths[L] * 4);
    w.loss_part = (float *)take(n * ((B + 31) / 32) * 4);
    for (int i = 0; i < 2; ++i) w.dz[i] = (bf16_t *)take(n * B * widest * 2);
    w.bytes = off + 256;
    return w;
}

// A layer's weight gradient can be fused into the mix when a kernel exists for the topology (Theorem 3's ring; a
// torus with 3 to 16 columns and at least 3 grid rows; any other W of at most 64 workers) and its tiles divide the matrix.
bool torus_cols(const dpsgd_ctx *ctx) { return ctx->torus_uniform && ctx->dim1 >= 3 && ctx->dim1 <= 16 && ctx->dim0 >= 3; }

// Any other W of at most 64 workers: the kernel that holds every worker's tile in LDS ("fused_slab": 0 never, 1 where
// no walk kernel exists, 2 also instead of the torus walk).
bool slab_fusion(const dpsgd_ctx *ctx)
{
    if (ctx->opt_fused_slab == 0 || ctx->ring_uniform || ctx->n > 64 || !ctx->d_rowptr) return false;
    return ctx->opt_fused_slab == 2 || !torus_cols(ctx);
}

bool layer_fusable(const dpsgd_ctx *ctx, int K, int O, i64 woff)
{
    if (ctx->opt_mix_force_csr || woff < 0 || (i64)K * O < (1 << 20)) return false;
    if (ctx->ring_uniform) return (K % 128) == 0 && (O % 32) == 0;
    if (torus_cols(ctx) || slab_fusion(ctx))
        return (K % 32) == 0 && (O % 32) == 0 && (woff % 2) == 0 && (ctx->ld % 2) == 0;   // 8-byte accesses
    return false;
}

dpsgd_status run_mlp_bf16(dpsgd_ctx *ctx, const dpsgd_model_desc &m, float *X, const void *inputs, const void *targets,
                          float *G, float *loss, bool fuse, float *consensus)
{
    hipStream_t s = ctx->stream;
    const int n = ctx->n, B = m.batch, Bp = round_up(B, 32);
    const int L = (int)m.widths.size() - 1;
    if (n > 65535) return DPSGD_EUNSUPPORTED;
    MlpWs ws = carve(ctx, m, (unsigned char *)ctx->ws);
    std::vector<const bf16_t *> act(L), actt(L);   // act[l]: input of layer l, [n][B][w_l]; actt[l]: [n][w_l][Bp]
    act[0] = m.input_is_bf16 ? (const bf16_t *)inputs : ws.a0;
    actt[0] = ws.at0;
    for (int l = 1; l < L; ++l) {
        act[l] = ws.h[l];
        actt[l] = ws.ht[l];
    }
    std::vector<i64> woff(L), boff(L);
    i64 off = 0;
    for (int l = 0; l < L; ++l) {
        woff[l] = off; off += (i64)m.widths[l + 1] * m.widths[l];
        boff[l] = off; off += m.widths[l + 1];
    }

    // "bf16_shadow": which layers read the bf16 weights the previous call left, which leave them for the next one.
    // Only hidden layers qualify (their weights are read twice, by the forward and by the data gradient; for the
    // first layer the extra write would cost what the forward saves), only on the ring kernel, never under capture
    // (a recorded call could not know what the buffer holds when it is replayed).
    std::vector<const bf16_t *> wb_use(L, nullptr);
    std::vector<bf16_t *> wb_emit(L, nullptr);
    const bool base_ok = aligned16(X) && (ctx->ld % 4) == 0;
    // layers the [16 rows][1 KB] ring kernel takes; a copy it writes is in its own tile layout, and a reader is told
    // the layout the copy was written in (the minibatch, hence the kernel, may differ between the two calls)
    std::vector<char> rows_kernel(L, 0), strips_use(L, 0);
    for (int l = 0; l < L; ++l)
        rows_kernel[l] = ctx->ring_uniform && ctx->opt_ring_rows && Bp == 32 && (m.widths[l] % 256) == 0 &&
                         (m.widths[l + 1] % 32) == 0 && (woff[l] % 4) == 0 && base_ok;
    if (fuse) {
        const bool was_valid = ctx->shadow_valid && ctx->shadow_X == X && ctx->shadow_model.kind == m.kind &&
                               ctx->shadow_model.compute_bf16 == m.compute_bf16 &&
                               ctx->shadow_model.widths == m.widths && (int)ctx->shadow_off.size() == L &&
                               (int)ctx->shadow_strips.size() == L;
        ctx->shadow_valid = false;
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
        if (hipStreamIsCapturing(s, &cap) != hipSuccess) cap = hipStreamCaptureStatusNone;
        if (ctx->opt_bf16_shadow && ctx->ring_uniform && cap == hipStreamCaptureStatusNone) {
            std::vector<int64_t> soff(L, -1);
            size_t elems = 0;
            for (int l = 1; l < L; ++l) {
                if (!layer_fusable(ctx, m.widths[l], m.widths[l + 1], woff[l])) continue;
                soff[l] = (int64_t)elems;
                elems += (size_t)n * m.widths[l] * m.widths[l + 1];
            }
            if (elems * sizeof(bf16_t) > ctx->shadow_bytes) {
                if (hipStreamSynchronize(s) != hipSuccess) return DPSGD_EDEVICE;
                if (ctx->shadow) (void)hipFree(ctx->shadow);
                ctx->shadow = nullptr;
                ctx->shadow_bytes = 0;
                if (hipMalloc(&ctx->shadow, elems * sizeof(bf16_t)) != hipSuccess) {
                    (void)hipGetLastError();
                    return DPSGD_ENOMEM;
                }
                ctx->shadow_bytes = elems * sizeof(bf16_t);
            } else if (was_valid && soff == ctx->shadow_off) {
                for (int l = 1; l < L; ++l)
                    if (soff[l] >= 0) {
                        wb_use[l] = (const bf16_t *)ctx->shadow + soff[l];
                        strips_use[l] = ctx->shadow_strips[l];
                    }
            }
            for (int l = 1; l < L; ++l)
                if (soff[l] >= 0) wb_emit[l] = (bf16_t *)ctx->shadow + soff[l];
            ctx->shadow_off = soff;
            ctx->shadow_strips = rows_kernel;
        }
    }

    {   // bf16 copy (if needed) and transposed copy of the inputs
        const int F = m.widths[0];
        dim3 grid((unsigned)((F + 31) / 32), (unsigned)(Bp / 32), (unsigned)n);
        if (m.input_is_bf16 && (F % 8) == 0 && aligned16(inputs))
            hipLaunchKernelGGL(prep_input_vec_kernel, dim3((unsigned)((F + 63) / 64), (unsigned)(Bp / 32), (unsigned)n),
                               dim3(256), 0, s, (const bf16_t *)inputs, ws.at0, B, Bp, F);
        else if (m.input_is_bf16)
            hipLaunchKernelGGL(prep_input_kernel<true>, grid, dim3(256), 0, s, inputs, ws.a0, ws.at0, B, Bp, F);
        else
            hipLaunchKernelGGL(prep_input_kernel<false>, grid, dim3(256), 0, s, inputs, ws.a0, ws.at0, B, Bp, F);
    }
    const Tiling t = pick_tiling(B);
    dpsgd_status st = DPSGD_OK;
    // a class layer of at most 16 outputs on top of a hidden layer: its backward is one launch (mlp_class_bwd_kernel)
    // and the softmax rides in its forward launch
    const bool class_path = L > 1 && m.widths[L] <= 16 && Bp <= 256 && ctx->opt_class_bwd &&
                            !(fuse && layer_fusable(ctx, m.widths[L - 1], m.widths[L], woff[L - 1]));
    bool softmax_in_fwd = false;
    for (int l = 0; l < L && st == DPSGD_OK; ++l) {
        FwdArgs a{};
        a.act = act[l]; a.X = X; a.ld = ctx->ld; a.woff = woff[l]; a.boff = boff[l];
        a.B = B; a.Bp = Bp; a.K = m.widths[l]; a.O = m.widths[l + 1];
        const bool last = (l == L - 1);
        if (last) a.z = ws.logits; else { a.h = ws.h[l + 1]; a.ht = ws.ht[l + 1]; }
        a.wb = wb_use[l];
        a.wb_strips = strips_use[l];
        const bool vec = base_ok && (a.K % 8) == 0 && (woff[l] % 4) == 0 && aligned16(act[l]);
        if (last && vec && a.O <= 32 && (a.K % 16) == 0 && a.K >= 256) {
            if (class_path) {
                a.labels = (const int *)targets; a.sm_dz = ws.dz[0]; a.sm_dzt = ws.dzt[L]; a.loss_part = ws.loss_part;
                softmax_in_fwd = true;
            }
            hipLaunchKernelGGL(mlp_fwd_last_kernel, dim3((unsigned)((B + 31) / 32), (unsigned)n), dim3(512), 0, s, a);
            st = hip_status(hipGetLastError());
        } else if (t.mt == 1) st = fwd_ksplit_launch(s, n, a, vec, last);
        else if (t.wm == 1) st = fwd_launch<1, 4, 2>(s, n, a, vec, last);
        else st = fwd_launch<2, 2, 2>(s, n, a, vec, last);
    }
    if (st != DPSGD_OK) return st;
    const int C = m.widths[L];
    int cur = 0;
    if (!softmax_in_fwd)
        hipLaunchKernelGGL(softmax_xent_bf16_kernel, dim3((unsigned)n), dim3(256), 0, s, ws.logits, (const int *)targets, B, Bp,
                           C, ws.dz[cur], ws.dzt[L], loss);
    std::vector<char> fused(L, 0);
    bool bias_below_done = false;
    for (int l = L - 1; l >= 0 && st == DPSGD_OK; --l) {
        const int K = m.widths[l], O = m.widths[l + 1];
        fused[l] = fuse && layer_fusable(ctx, K, O, woff[l]) && (ctx->ring_uniform || (reinterpret_cast<uintptr_t>(X) & 7) == 0);
        if (l == L - 1 && class_path && !fused[l]) {
            // the class layer: weight, bias and data gradient and the bias gradient of the layer below in one launch
            ClassBwdArgs ca{};
            ca.dz = ws.dz[cur]; ca.h = ws.h[l]; ca.X = X; ca.G = G; ca.ld = ctx->ld; ca.woff = woff[l]; ca.boff = boff[l];
            ca.boff_below = boff[l - 1];
            ca.dzp = l - 1 > 0 ? ws.dz[cur ^ 1] : nullptr;   // read by the data gradient of the layer below, if there is one
            ca.dzpt = ws.dzt[l];
            ca.B = B; ca.Bp = Bp; ca.K = K; ca.C = O;
            ca.loss_part = softmax_in_fwd ? ws.loss_part : nullptr; ca.chunks = (B + 31) / 32; ca.loss = loss;
            const int sgroups = Bp >= 64 ? 4 : 1;   // sample groups per workgroup, 256 / sgroups columns each
            const dim3 cgrid((unsigned)(((i64)K * sgroups + 255) / 256), (unsigned)n);
            if (sgroups == 4) {
                if (O <= 10) hipLaunchKernelGGL((mlp_class_bwd_kernel<10, 4>), cgrid, dim3(256), 0, s, ca);
                else hipLaunchKernelGGL((mlp_class_bwd_kernel<16, 4>), cgrid, dim3(256), 0, s, ca);
            } else {
                if (O <= 10) hipLaunchKernelGGL((mlp_class_bwd_kernel<10, 1>), cgrid, dim3(256), 0, s, ca);
                else hipLaunchKernelGGL((mlp_class_bwd_kernel<16, 1>), cgrid, dim3(256), 0, s, ca);
            }
            st = hip_status(hipGetLastError());
            bias_below_done = true;
            cur ^= 1;
            continue;
        }
        if (fused[l]) {   // only the bias gradient goes to G; the weight gradient is formed inside the mix
            if (!(bias_below_done && l == L - 2))
                hipLaunchKernelGGL(bias_grad_bf16_kernel, dim3((unsigned)((O + 255) / 256), (unsigned)n), dim3(256), 0, s,
                                   ws.dzt[l + 1], O, Bp, G, ctx->ld, boff[l]);
        } else {
            WgradArgs wa{};
            wa.dzt = ws.dzt[l + 1]; wa.at = actt[l]; wa.G = G; wa.ld = ctx->ld; wa.woff = woff[l]; wa.boff = boff[l];
            wa.Bp = Bp; wa.K = K; wa.O = O;
            if (O <= 32) {
                dim3 wgrid((unsigned)((K + 127) / 128), (unsigned)((O + 31) / 32), (unsigned)n);
                hipLaunchKernelGGL(mlp_wgrad_kernel<true>, wgrid, dim3(256), 0, s, wa);
            } else {
                dim3 wgrid((unsigned)((K + 255) / 256), (unsigned)((O + 127) / 128), (unsigned)n);
                hipLaunchKernelGGL(mlp_wgrad_kernel<false>, wgrid, dim3(256), 0, s, wa);
            }
        }
        st = hip_status(hipGetLastError());
        if (l > 0 && st == DPSGD_OK) {
            DgradArgs da{};
            da.dz = ws.dz[cur]; da.X = X; da.ld = ctx->ld; da.woff = woff[l]; da.hprev = ws.h[l];
            da.dzp = ws.dz[cur ^ 1]; da.dzpt = ws.dzt[l];
            da.B = B; da.Bp = Bp; da.K = K; da.O = O;
            da.wb = wb_use[l];
            da.wb_strips = strips_use[l];
            const bool vec = base_ok && (K % 4) == 0 && (O % 8) == 0 && (woff[l] % 4) == 0;
            if (t.mt == 1) st = dgrad_launch<1, 4, 1>(s, n, da, vec);
            else if (t.wm == 1) st = dgrad_launch<1, 4, 2>(s, n, da, vec);
            else st = dgrad_launch<2, 2, 2>(s, n, da, vec);
            cur ^= 1;
        }
    }
    if (st != DPSGD_OK || !fuse) return st;

    // ---- Algorithm 1 steps 4-5, in place: fused layers first, then the remaining column ranges
    const bool cons = consensus != nullptr;
    int64_t nparts = 0;
    bool timing = false;
    if (ctx->opt_time_fused && ctx->ev_pairs < 8192) {   // bracket the fused launches with events
        while ((int64_t)ctx->ev.size() < 2 * (ctx->ev_pairs + 1)) {
            hipEvent_t e = nullptr;
            if (hipEventCreate(&e) != hipSuccess) return DPSGD_EDEVICE;
            ctx->ev.push_back(e);
        }
        timing = true;
        (void)hipEventRecord(ctx->ev[2 * ctx->ev_pairs], s);
    }
    for (int l = 0; l < L && st == DPSGD_OK; ++l) {
        if (!fused[l]) continue;
        if (timing) ctx->ev_launches += 1;
        const int K = m.widths[l], O = m.widths[l + 1];
        i64 np = 0;
        if (ctx->ring_uniform) {
            FusedArgs fa{};
            fa.X = X; fa.ld = ctx->ld; fa.woff = woff[l]; fa.dzt = ws.dzt[l + 1]; fa.at = actt[l];
            fa.n = n; fa.K = K; fa.O = O; fa.Bp = Bp; fa.w = ctx->ring_w; fa.gamma = ctx->gamma;
            fa.partials = ctx->d_partials + nparts;
            dim3 grid((unsigned)(K / 128), (unsigned)(O / 32));
            np = (i64)grid.x * grid.y * 4;
            if (nparts + np > ctx->partials_cap - 256) return DPSGD_EINVAL;
            fa.shadow = wb_emit[l];
            if (rows_kernel[l]) {   // same number of workgroups and of partial sums as the 32 x 32 kernel
                dim3 grid_rows((unsigned)(K / 256), (unsigned)(O / 16));
                // rows of 32 KB (16 KB): a wave's pieces one row (two rows) apart
                const int rs = !ctx->opt_ring_chunks ? 0 : K == 8192 ? 1 : K == 4096 ? 2 : ((K % 1024) == 0 && !fa.shadow) ? 3 : 0;
#define DPSGD_ROWS(CONS, SHADOW)                                                                                              \
    do {                                                                                                                      \
        if (rs == 2) hipLaunchKernelGGL((mlp_fused_ring_rows_kernel<CONS, SHADOW, 2>), grid_rows, dim3(256), 0, s, fa);      \
        else if (rs == 1) hipLaunchKernelGGL((mlp_fused_ring_rows_kernel<CONS, SHADOW, 1>), grid_rows, dim3(256), 0, s, fa); \
        else if (rs == 3) hipLaunchKernelGGL((mlp_fused_ring_rows_kernel<CONS, false, 3>), grid_rows, dim3(256), 0, s, fa);  \
        else hipLaunchKernelGGL((mlp_fused_ring_rows_kernel<CONS, SHADOW, 0>), grid_rows, dim3(256), 0, s, fa);              \
    } while (0)
                if (fa.shadow) {
                    if (cons) DPSGD_ROWS(true, true);
                    else DPSGD_ROWS(false, true);
                } else {
                    if (cons) DPSGD_ROWS(true, false);
                    else DPSGD_ROWS(false, false);
                }
#undef DPSGD_ROWS
            } else if (fa.shadow) {
                if (cons) hipLaunchKernelGGL((mlp_fused_ring_kernel<true, true>), grid, dim3(256), 0, s, fa);
                else hipLaunchKernelGGL((mlp_fused_ring_kernel<false, true>), grid, dim3(256), 0, s, fa);
            } else if (Bp >= 64 && Bp <= 192 && ctx->opt_fused_lds) {   // operands through LDS: 5 KB per 16 minibatch rows (at most 60 KB)
                const size_t shm = (size_t)5 * (Bp / 16) * 1024;
                if (cons) hipLaunchKernelGGL((mlp_fused_ring_lds_kernel<true>), grid, dim3(256), shm, s, fa);
                else hipLaunchKernelGGL((mlp_fused_ring_lds_kernel<false>), grid, dim3(256), shm, s, fa);
            } else {
                if (cons) hipLaunchKernelGGL((mlp_fused_ring_kernel<true, false>), grid, dim3(256), 0, s, fa);
                else hipLaunchKernelGGL((mlp_fused_ring_kernel<false, false>), grid, dim3(256), 0, s, fa);
            }
        } else if (slab_fusion(ctx)) {
            FusedSlabArgs fa{};
            fa.X = X; fa.ld = ctx->ld; fa.woff = woff[l]; fa.dzt = ws.dzt[l + 1]; fa.at = actt[l];
            fa.rowptr = ctx->d_rowptr; fa.colidx = ctx->d_colidx; fa.vals = ctx->d_vals;
            fa.n = n; fa.K = K; fa.O = O; fa.Bp = Bp; fa.gamma = ctx->gamma;
            fa.partials = ctx->d_partials + nparts;
            // column groups of 32 per workgroup: as many as 128 KB of LDS hold for n workers and as divide the inputs
            // (64 KB, two workgroups per CU, where that leaves a group: one fills the slab while the other works on its own)
            int mg = n <= 8 ? 4 : n <= 16 ? 2 : 1;
            while (mg > 1 && (n * mg > 64 || (K % (32 * mg)) != 0)) mg >>= 1;
            const int nw = (mg == 1 && n > 48) ? 16 : 8;   // a full slab has the CU to itself: 16 waves of 4 workers each
            dim3 grid((unsigned)(K / (32 * mg)), (unsigned)(O / 16));
            np = (i64)grid.x * grid.y;
            if (nparts + np > ctx->partials_cap - 256) return DPSGD_EINVAL;
            const size_t slab = (size_t)n * mg * 2048, red = (size_t)256 * nw * (8 * mg + 1);
            const size_t shm = slab > red ? slab : red;
#define DPSGD_SLAB_ONE(CONS, MG, NWV)                                                                                              \
    do {                                                                                                                        \
        auto kern = mlp_fused_slab_kernel<CONS, MG, NWV>;                                                                       \
        if (shm > 64 * 1024 && hipFuncSetAttribute(reinterpret_cast<const void *>(kern),                                        \
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)shm) != hipSuccess)         \
            return DPSGD_EDEVICE;                                                                                               \
        hipLaunchKernelGGL(kern, grid, dim3(64 * NWV), shm, s, fa);                                                             \
    } while (0)
#define DPSGD_SLAB(MG, NWV)                                                                                         \
    do {                                                                                                            \
        if (cons) DPSGD_SLAB_ONE(true, MG, NWV);                                                                    \
        else DPSGD_SLAB_ONE(false, MG, NWV);                                                                        \
    } while (0)
            if (mg == 4) DPSGD_SLAB(4, 8);
            else if (mg == 2) DPSGD_SLAB(2, 8);
            else if (nw == 16) DPSGD_SLAB(1, 16);
            else DPSGD_SLAB(1, 8);
#undef DPSGD_SLAB
#undef DPSGD_SLAB_ONE
        } else {
            FusedTorusColArgs fa{};
            fa.X = X; fa.ld = ctx->ld; fa.woff = woff[l]; fa.dzt = ws.dzt[l + 1]; fa.at = actt[l];
            fa.R = ctx->dim0; fa.C = ctx->dim1; fa.K = K; fa.O = O; fa.Bp = Bp; fa.w = ctx->torus_w; fa.gamma = ctx->gamma;
            fa.partials = ctx->d_partials + nparts;
            // two groups of waves side by side (256-byte row segments) when the inputs divide
            const int kt = ((K % 64) == 0 && fa.C <= 8) ? 2 : 1;
            dim3 grid((unsigned)(K / (32 * kt)), (unsigned)(O / 16));
            np = (i64)grid.x * grid.y * kt;
            if (nparts + np > ctx->partials_cap - 256) return DPSGD_EINVAL;
            const size_t shm = (size_t)2 * fa.C * 2048 * kt;
            if (kt == 2) {
                if (cons) hipLaunchKernelGGL((mlp_fused_torus_cols_kernel<true, 2, 8>), grid, dim3(128u * fa.C), shm, s, fa);
                else hipLaunchKernelGGL((mlp_fused_torus_cols_kernel<false, 2, 8>), grid, dim3(128u * fa.C), shm, s, fa);
            } else if (fa.C <= 8) {
                if (cons) hipLaunchKernelGGL((mlp_fused_torus_cols_kernel<true, 1, 8>), grid, dim3(64u * fa.C), shm, s, fa);
                else hipLaunchKernelGGL((mlp_fused_torus_cols_kernel<false, 1, 8>), grid, dim3(64u * fa.C), shm, s, fa);
            } else {
                if (cons) hipLaunchKernelGGL((mlp_fused_torus_cols_kernel<true, 1, 16>), grid, dim3(64u * fa.C), shm, s, fa);
                else hipLaunchKernelGGL((mlp_fused_torus_cols_kernel<false, 1, 16>), grid, dim3(64u * fa.C), shm, s, fa);
            }
        }
        if (cons) nparts += np;
        st = hip_status(hipGetLastError());
    }
    if (timing) {
        (void)hipEventRecord(ctx->ev[2 * ctx->ev_pairs + 1], s);
        ctx->ev_pairs += 1;
    }
    // maximal runs of columns that no fused kernel owns
    i64 run0 = 0;
    for (int l = 0; l <= L && st == DPSGD_OK; ++l) {
        const bool boundary = (l == L) || fused[l];
        if (!boundary) continue;
        const i64 run1 = (l == L) ? ctx->d : woff[l];
        if (run1 > run0) st = launch_mix_range(ctx, X, G, X, run0, run1 - run0, cons, &nparts);
        if (l < L) run0 = boff[l];
    }
    if (st == DPSGD_OK && cons) st = launch_consensus_finalize(ctx, nparts, consensus);
    if (st == DPSGD_OK) {   // the bf16 copies describe X as this call leaves it
        bool any = false, all = true;
        for (int l = 0; l < L; ++l) {
            any = any || wb_emit[l] != nullptr;
            all = all && (wb_emit[l] == nullptr || fused[l]);
        }
        if (any && all) {
            ctx->shadow_valid = true;
            ctx->shadow_X = X;
            ctx->shadow_model = m;
        }
    }
    return st;
}
}  // namespace

size_t mlp_bf16_workspace_bytes(const dpsgd_ctx *ctx, const dpsgd_model_desc &m) { return carve(ctx, m, nullptr).bytes; }

dpsgd_status launch_grad_mlp_bf16(dpsgd_ctx *ctx, const dpsgd_model_desc &m, const float *X, const void *inputs,
                                  const void *targets, float *G, float *loss)
{
    return run_mlp_bf16(ctx, m, const_cast<float *>(X), inputs, targets, G, loss, false, nullptr);
}

dpsgd_status launch_step_mlp_bf16(dpsgd_ctx *ctx, const dpsgd_model_desc &m, float *X, const void *inputs,
                                  const void *targets, float *G, float *loss, float *consensus)
{
    return run_mlp_bf16(ctx, m, X, inputs, targets, G, loss, true, consensus);
}

}  // namespace dpsgd

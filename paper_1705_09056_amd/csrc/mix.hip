// Gossip-mix + SGD update (Algorithm 1 steps 4-5 fused), node average (step 7) and the
// consensus distance (eq. 10/13 in the proof of Theorem 1) for gfx950.
//
// The work is bound by HBM bandwidth: 12 bytes per (worker, parameter) - X read once, G read
// once, X_next written once - whatever the degree of W.  To read each replica once, a workgroup
// owns a slab of columns for ALL n rows:
//   * ring (Theorem 3's W): each lane owns V consecutive columns and walks the rows keeping
//     x_{i-1}, x_i, x_{i+1} in registers.  The waves of a workgroup split the rows into bands;
//     each band loads its two halo rows before a barrier, so the update may be done in place.
//   * any other W (CSR): the workgroup stages its n x (64 V) slab in LDS, then every wave forms
//     its rows from LDS in CSR order.
// The consensus distance of the OUTPUT is accumulated on the fly per column (sums of deviations
// from a per-lane shift, so that no large numbers cancel), reduced across bands in LDS, across
// lanes with wave shuffles, and across workgroups in a fixed order by a second tiny kernel.
#include <mutex>

#include "dpsgd_internal.h"

namespace dpsgd {
namespace {

typedef long long i64;

template <int V> struct VecT;
template <> struct VecT<1> { typedef float type; };
template <> struct VecT<2> { typedef float type __attribute__((ext_vector_type(2))); };
template <> struct VecT<4> { typedef float type __attribute__((ext_vector_type(4))); };

template <int V> __device__ __forceinline__ typename VecT<V>::type vload(const float *p)
{
    return *reinterpret_cast<const typename VecT<V>::type *>(p);
}
template <int V> __device__ __forceinline__ void vstore(float *p, typename VecT<V>::type v)
{
    *reinterpret_cast<typename VecT<V>::type *>(p) = v;
}
// a * x + y with one rounding, spelled out so that every ring kernel rounds the same way (left to the compiler,
// two kernels may fuse different products of  w x_{i-1} + w x_i + w x_{i+1} - gamma g)
__device__ __forceinline__ float fma_s(float a, float x, float y) { return __builtin_fmaf(a, x, y); }
template <typename T> __device__ __forceinline__ T fma_s(float a, T x, T y) { return __builtin_elementwise_fma((T)(a), x, y); }
// the update of one element or vector: fixed order and roundings
template <typename T> __device__ __forceinline__ T ring_update(float w, T xm, T xc, T xn, float gamma, T g)
{
    T acc = w * xm;
    acc = fma_s(w, xc, acc);
    acc = fma_s(w, xn, acc);
    return fma_s(-gamma, g, acc);
}
template <int V> __device__ __forceinline__ float hsum(typename VecT<V>::type v);
template <> __device__ __forceinline__ float hsum<1>(float v) { return v; }
template <> __device__ __forceinline__ float hsum<2>(VecT<2>::type v) { return v.x + v.y; }
template <> __device__ __forceinline__ float hsum<4>(VecT<4>::type v) { return (v.x + v.y) + (v.z + v.w); }

__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    return v;
}

// Per-column running sums of (x - shift) and (x - shift)^2 over the rows a lane has produced.
template <int V> struct ColStats {
    typedef typename VecT<V>::type vec;
    vec shift, s1, s2;
    float cnt;
    __device__ __forceinline__ void init() { shift = (vec)(0.f); s1 = (vec)(0.f); s2 = (vec)(0.f); cnt = 0.f; }
    __device__ __forceinline__ void add(vec x)
    {
        if (cnt == 0.f) shift = x;
        vec e = x - shift;
        s1 += e;
        s2 += e * e;
        cnt += 1.f;
    }
    // fold `o` (own shift) into this one (keeps this shift)
    __device__ __forceinline__ void merge(vec oshift, vec os1, vec os2, float ocnt)
    {
        if (ocnt == 0.f) return;
        if (cnt == 0.f) { shift = oshift; s1 = os1; s2 = os2; cnt = ocnt; return; }
        vec dlt = oshift - shift;
        s1 += os1 + ocnt * dlt;
        s2 += os2 + 2.f * dlt * os1 + ocnt * dlt * dlt;
        cnt += ocnt;
    }
    // sum over this lane's columns of sum_i (x_i - mean)^2
    __device__ __forceinline__ float m2() const
    {
        if (cnt == 0.f) return 0.f;
        vec r = s2 - s1 * s1 * (1.f / cnt);
        return hsum<V>(r);
    }
};

// Combine the per-band ColStats of one column group through LDS; band 0 ends up with the total.
// lds must hold bands * 64 * (3 V + 1) floats.  Called by every thread of the workgroup.
template <int V>
__device__ __forceinline__ void combine_bands(ColStats<V> &st, float *lds, int band, int lane, int bands)
{
    typedef typename VecT<V>::type vec;
    if (bands == 1) return;
    const int stride = 3 * V + 1;
    float *mine = lds + ((size_t)band * 64 + lane) * stride;
    if (band > 0) {
#pragma unroll
        for (int v = 0; v < V; ++v) {
            mine[v] = ((const float *)&st.shift)[v];
            mine[V + v] = ((const float *)&st.s1)[v];
            mine[2 * V + v] = ((const float *)&st.s2)[v];
        }
        mine[3 * V] = st.cnt;
    }
    __syncthreads();
    if (band == 0) {
        for (int b = 1; b < bands; ++b) {
            const float *o = lds + ((size_t)b * 64 + lane) * stride;
            vec sh, a1, a2;
#pragma unroll
            for (int v = 0; v < V; ++v) {
                ((float *)&sh)[v] = o[v];
                ((float *)&a1)[v] = o[V + v];
                ((float *)&a2)[v] = o[2 * V + v];
            }
            st.merge(sh, a1, a2, o[3 * V]);
        }
    }
}

// ------------------------------------------------------------------------------- ring
// One column group of 64*V columns (group `grp`), walked by a workgroup of 64 * bands threads; wave b owns rows
// [b*rpb, min(n,(b+1)*rpb)).  The group's consensus partial goes to partials[part].
// MOM: heavy-ball variant, the step uses v = mu * Vel + g and Vel is overwritten with it.
template <int V, int U, bool CONS, bool MOM>
__device__ __forceinline__ void ring_walk(const float *Xin, const float *__restrict__ G, float *Xout, int n, i64 ncols, i64 ld,
                                          float w, float gamma, int bands, int rpb, double *__restrict__ partials,
                                          float *__restrict__ Vel, float mu, float *lds, i64 grp, i64 part)
{
    typedef typename VecT<V>::type vec;
    const int lane = threadIdx.x & 63;
    const int band = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const i64 c0 = (grp * 64 + lane) * V;
    const bool active = c0 + V <= ncols;
    const int r0 = band * rpb;
    const int r1 = min(n, r0 + rpb);
    const float *xin = Xin + c0;
    const float *gin = G + c0;
    float *xout = Xout + c0;

    vec xm = (vec)(0.f), xc = (vec)(0.f), xhalo = (vec)(0.f);
    if (active && r0 < r1) {
        xm = vload<V>(xin + (i64)((r0 + n - 1) % n) * ld);
        xc = vload<V>(xin + (i64)r0 * ld);
        xhalo = vload<V>(xin + (i64)(r1 % n) * ld);
    }
    // Every band has fetched the rows its neighbours are about to overwrite.
    if (bands > 1) __syncthreads();

    ColStats<V> st;
    st.init();
    if (active && r0 < r1) {
        // Rows r0 .. r1-2 read their successor from memory in branch-free chunks of U rows (2U
        // loads in flight per lane); the band's last row takes the halo fetched above.
        auto form = [&](vec xn, vec g, float *dst) {
            const vec o = ring_update(w, xm, xc, xn, gamma, g);
            vstore<V>(dst, o);
            if (CONS) st.add(o);
            xm = xc;
            xc = xn;
        };
        int row = r0;
        const int rlast = r1 - 1;
        const float *xp = xin + (i64)(row + 1) * ld;
        const float *gp = gin + (i64)row * ld;
        float *vp = MOM ? Vel + c0 + (i64)row * ld : nullptr;
        float *op = xout + (i64)row * ld;
        // the gradient the step uses: g itself, or the updated velocity (written back)
        auto step_dir = [&](vec g, float *vdst) {
            if (MOM) {
                g = mu * vload<V>(vdst) + g;
                vstore<V>(vdst, g);
            }
            return g;
        };
        for (; row + U <= rlast; row += U) {
            vec xs[U], gs[U], vs[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                gs[u] = __builtin_nontemporal_load(reinterpret_cast<const vec *>(gp + (i64)u * ld));
                if (MOM) vs[u] = vload<V>(vp + (i64)u * ld);
                xs[u] = vload<V>(xp + (i64)u * ld);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (MOM) {
                    gs[u] = mu * vs[u] + gs[u];
                    vstore<V>(vp + (i64)u * ld, gs[u]);
                }
                form(xs[u], gs[u], op + (i64)u * ld);
            }
            xp += (i64)U * ld;
            gp += (i64)U * ld;
            if (MOM) vp += (i64)U * ld;
            op += (i64)U * ld;
        }
        for (; row < rlast; ++row) {
            vec g = step_dir(__builtin_nontemporal_load(reinterpret_cast<const vec *>(gp)), vp);
            vec xn = vload<V>(xp);
            form(xn, g, op);
            xp += ld;
            gp += ld;
            if (MOM) vp += ld;
            op += ld;
        }
        form(xhalo, step_dir(__builtin_nontemporal_load(reinterpret_cast<const vec *>(gp)), vp), op);
    }
    if (CONS) {
        combine_bands<V>(st, lds, band, lane, bands);
        if (band == 0) {
            double v = wave_sum((double)st.m2());
            if (lane == 0) partials[part] = v;
        }
    }
}

// grid.x = column groups of 64*V columns (+ 1 when tail > 0); block = 64 * bands threads.  ncols is a multiple of V.
// tail (V > 1 only, at most V - 1): the columns ncols .. ncols + tail - 1, which the last workgroup walks one per lane
// - the same arithmetic, in the same launch, instead of a launch of their own.
template <int V, int U, bool CONS, bool MOM>
__global__ void __launch_bounds__(512)
mix_ring_kernel(const float *Xin, const float *__restrict__ G, float *Xout, int n, i64 ncols, i64 ld, float w,
                float gamma, int bands, int rpb, double *__restrict__ partials, float *__restrict__ Vel, float mu, int tail)
{
    extern __shared__ float lds[];
    if (V > 1 && tail > 0 && blockIdx.x == gridDim.x - 1) {
        ring_walk<1, U, CONS, MOM>(Xin + ncols, G + ncols, Xout + ncols, n, tail, ld, w, gamma, bands, rpb, partials,
                                   MOM ? Vel + ncols : nullptr, mu, lds, 0, blockIdx.x);
        return;
    }
    ring_walk<V, U, CONS, MOM>(Xin, G, Xout, n, ncols, ld, w, gamma, bands, rpb, partials, Vel, mu, lds, blockIdx.x, blockIdx.x);
}

// The same walk for wide matrices with fat lanes: one wave per workgroup, every lane owns P float4 column groups, U
// rows in flight.  Fewer, fatter waves keep more bytes in flight per memory instruction stream, and WHICH columns a
// wave owns decides how its accesses fall on the HBM channels: with the wave's row footprint cut into chunks of 512
// bytes (half a wave per chunk) that sit 32 KB apart, the walk moves 6.2 TB/s at 64 workers x 29.4 M columns where
// the same walk over 8 KB of consecutive columns moves 5.4 (1 KB chunks 32 or 64 KB apart: 5.9; 512-byte chunks at
// other distances, and 256-byte chunks at any distance: 5.2-5.9).  So the columns are dealt out in super-blocks of
// kFatSuper = 2 P x 8192 floats: workgroup k of a super-block (k < 64) owns the 2 P chunks that start
// k x 128 floats into each 32 KB stripe.
// No row bands (those stay with mix_ring_kernel); MOM is the heavy-ball variant as there.  The shift of the consensus sums is worker 0's ORIGINAL
// value, which the lane keeps anyway for the ring's wrap-around.  Same arithmetic, same order as mix_ring_kernel.
// grid.x = 64 x (ncols / kFatSuper) (whole super-blocks only: no lane is ever idle), block 64; 16-byte aligned rows.
constexpr int kFatChunkLanes = 32;        // lanes per chunk: 512 bytes
constexpr i64 kFatStride = 8192;          // floats between two chunks of a wave: 32 KB
template <int P> constexpr i64 fat_super() { return (i64)P * (64 / kFatChunkLanes) * kFatStride; }

template <int P, int U, bool CONS, bool MOM>
__global__ void __launch_bounds__(64)
mix_ring_fat_kernel(const float *Xin, const float *__restrict__ G, float *Xout, int n, i64 ld, float w, float gamma,
                    double *__restrict__ partials, float *__restrict__ Vel, float mu)
{
    typedef VecT<4>::type vec;
    const int lane = threadIdx.x;
    constexpr i64 kPerSuper = kFatStride / (kFatChunkLanes * 4);   // workgroups per super-block: 64
    constexpr i64 kStep = (64 / kFatChunkLanes) * kFatStride;      // floats between a lane's column groups q and q + 1
    const i64 sb = blockIdx.x / kPerSuper, k = blockIdx.x % kPerSuper;
    const i64 c0 = sb * fat_super<P>() + k * (kFatChunkLanes * 4) + (lane % kFatChunkLanes) * 4 +
                   (i64)(lane / kFatChunkLanes) * kFatStride;
    vec xm[P], xc[P], x0[P], s1[P];
    float s2 = 0.f;
#pragma unroll
    for (int q = 0; q < P; ++q) {
        const i64 c = c0 + (i64)q * kStep;
        xm[q] = vload<4>(Xin + (i64)(n - 1) * ld + c);
        xc[q] = vload<4>(Xin + c);
        x0[q] = xc[q];
        s1[q] = (vec)(0.f);
    }
    auto form = [&](int row, int q, vec xs, vec g) {
        const vec xn = row + 1 < n ? xs : x0[q];   // the ring closes on worker 0's original row
        const vec o = ring_update(w, xm[q], xc[q], xn, gamma, g);
        __builtin_nontemporal_store(o, reinterpret_cast<vec *>(Xout + (i64)row * ld + c0 + (i64)q * kStep));
        if (CONS) {
            const vec e = o - x0[q];
            s1[q] += e;
            s2 += hsum<4>(e * e);
        }
        xm[q] = xc[q];
        xc[q] = xn;
    };
    int row = 0;
    // the direction of the step: the gradient itself, or (MOM) the velocity mu v + g, which is written back
    auto step_dir = [&](int row, int q, vec g, vec v) {
        if (MOM) {
            g = mu * v + g;
            __builtin_nontemporal_store(g, reinterpret_cast<vec *>(Vel + (i64)row * ld + c0 + (i64)q * kStep));
        }
        return g;
    };
    for (; row + U <= n; row += U) {
        vec xs[U][P], gs[U][P], vs[MOM ? U : 1][MOM ? P : 1];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int rn = row + u + 1 < n ? row + u + 1 : n - 1;   // (the last row's successor is x0: clamped, unused)
#pragma unroll
            for (int q = 0; q < P; ++q) {
                const i64 c = c0 + (i64)q * kStep;
                gs[u][q] = __builtin_nontemporal_load(reinterpret_cast<const vec *>(G + (i64)(row + u) * ld + c));
                if (MOM) vs[u][q] = __builtin_nontemporal_load(reinterpret_cast<const vec *>(Vel + (i64)(row + u) * ld + c));
                xs[u][q] = __builtin_nontemporal_load(reinterpret_cast<const vec *>(Xin + (i64)rn * ld + c));
            }
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int q = 0; q < P; ++q) form(row + u, q, xs[u][q], step_dir(row + u, q, gs[u][q], MOM ? vs[u][q] : gs[u][q]));
    }
    for (; row < n; ++row) {
        const int rn = row + 1 < n ? row + 1 : n - 1;
#pragma unroll
        for (int q = 0; q < P; ++q) {
            const i64 c = c0 + (i64)q * kStep;
            const vec g = __builtin_nontemporal_load(reinterpret_cast<const vec *>(G + (i64)row * ld + c));
            const vec v = MOM ? __builtin_nontemporal_load(reinterpret_cast<const vec *>(Vel + (i64)row * ld + c)) : g;
            const vec x = __builtin_nontemporal_load(reinterpret_cast<const vec *>(Xin + (i64)rn * ld + c));
            form(row, q, x, step_dir(row, q, g, v));
        }
    }
    if (CONS) {
        float m2 = s2;
        const float inv_n = 1.0f / (float)n;
#pragma unroll
        for (int q = 0; q < P; ++q) m2 -= hsum<4>(s1[q] * s1[q]) * inv_n;
        const double v = wave_sum((double)m2);
        if (lane == 0) partials[blockIdx.x] = v;
    }
}

// ------------------------------------------------------------------------ CSR via LDS slab
// grid.x = column groups of 64*V columns; block = 64 * RG threads; lane = column vector,
// wave = row group (rows rg, rg+RG, ...).  Dynamic LDS: n * 64 * V floats (+ stats region).
// Vel != NULL (not with SWAPPED): heavy-ball variant, as in the ring kernel.
template <int V, bool CONS, bool SWAPPED>
__global__ void __launch_bounds__(1024)
mix_csr_slab_kernel(const float *Xin, const float *__restrict__ G, float *Xout, int n, i64 ncols, i64 ld,
                    const int *__restrict__ rowptr, const int *__restrict__ colidx, const float *__restrict__ vals,
                    float gamma, int rgroups, double *__restrict__ partials, float *__restrict__ Vel, float mu)
{
    typedef typename VecT<V>::type vec;
    extern __shared__ float lds[];
    vec *slab = reinterpret_cast<vec *>(lds);   // [n][64]
    const int lane = threadIdx.x & 63;
    const int rg = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const i64 c0 = ((i64)blockIdx.x * 64 + lane) * V;
    const bool active = c0 + V <= ncols;
    const float *xin = Xin + c0;
    const float *gin = G + c0;
    float *xout = Xout + c0;

    if (active) {
        auto stage = [&](int row) {
            vec x = vload<V>(xin + (i64)row * ld);
            if (SWAPPED) x = x - gamma * vload<V>(gin + (i64)row * ld);
            return x;
        };
        int row = rg;
        for (; row + 3 * rgroups < n; row += 4 * rgroups) {   // four independent loads in flight
            vec x0 = stage(row), x1 = stage(row + rgroups), x2 = stage(row + 2 * rgroups), x3 = stage(row + 3 * rgroups);
            slab[(size_t)row * 64 + lane] = x0;
            slab[(size_t)(row + rgroups) * 64 + lane] = x1;
            slab[(size_t)(row + 2 * rgroups) * 64 + lane] = x2;
            slab[(size_t)(row + 3 * rgroups) * 64 + lane] = x3;
        }
        for (; row < n; row += rgroups) slab[(size_t)row * 64 + lane] = stage(row);
    }
    __syncthreads();   // the whole slab is in LDS; from here on rows may be overwritten

    ColStats<V> st;
    st.init();
    if (active) {
        auto form = [&](int row, vec g) {
            const int p0 = rowptr[row], p1 = rowptr[row + 1];
            vec acc = (vec)(0.f);
            for (int p = p0; p < p1; ++p) acc = vals[p] * slab[(size_t)colidx[p] * 64 + lane] + acc;
            vec o = SWAPPED ? acc : acc - gamma * g;
            vstore<V>(xout + (i64)row * ld, o);
            if (CONS) st.add(o);
        };
        auto gload = [&](int row) {
            if (SWAPPED) return (vec)(0.f);
            vec g = __builtin_nontemporal_load(reinterpret_cast<const vec *>(gin + (i64)row * ld));
            if (Vel) {
                float *vdst = Vel + c0 + (i64)row * ld;
                g = mu * vload<V>(vdst) + g;
                vstore<V>(vdst, g);
            }
            return g;
        };
        int row = rg;
        for (; row + 3 * rgroups < n; row += 4 * rgroups) {
            vec g0 = gload(row), g1 = gload(row + rgroups), g2 = gload(row + 2 * rgroups), g3 = gload(row + 3 * rgroups);
            form(row, g0);
            form(row + rgroups, g1);
            form(row + 2 * rgroups, g2);
            form(row + 3 * rgroups, g3);
        }
        for (; row < n; row += rgroups) form(row, gload(row));
    }
    if (CONS) {
        __syncthreads();   // slab no longer needed; reuse LDS for the statistics
        combine_bands<V>(st, lds, rg, lane, rgroups);
        if (rg == 0) {
            double v = wave_sum((double)st.m2());
            if (lane == 0) partials[blockIdx.x] = v;
        }
    }
}

// The same for wide matrices, 16-byte accesses, whole super-blocks of columns: every lane owns SP float4 column
// vectors and the workgroup's 64 x SP vectors are 2 SP chunks of 512 bytes that sit 32 KB apart instead of consecutive
// columns - workgroup k of a super-block of 2 SP x 8192 columns owns the chunks that start k x 128 floats into each
// of its 32 KB stripes - which the HBM channels serve faster (see mix_ring_fat_kernel).  Slab: [n][SP][64] float4.
// grid.x = 64 x (ncols / slab_super<SP>()), every lane active.
template <int SP> constexpr i64 slab_super() { return (i64)2 * SP * 8192; }

template <int SP, bool CONS, bool SWAPPED>
__global__ void __launch_bounds__(512)
mix_csr_slab_wide_kernel(const float *Xin, const float *__restrict__ G, float *Xout, int n, i64 ld,
                         const int *__restrict__ rowptr, const int *__restrict__ colidx, const float *__restrict__ vals,
                         float gamma, int rgroups, double *__restrict__ partials, float *__restrict__ Vel, float mu)
{
    typedef VecT<4>::type vec;
    extern __shared__ float lds[];
    vec *slab = reinterpret_cast<vec *>(lds);
    const int lane = threadIdx.x & 63;
    const int rg = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const i64 c0 = (i64)(blockIdx.x / 64) * slab_super<SP>() + (i64)(blockIdx.x % 64) * 128 + (lane % 32) * 4 +
                   (i64)(lane / 32) * 8192;      // column vector q of this lane: c0 + q * 16384
    auto stage = [&](int row, vec (&x)[SP]) {
#pragma unroll
        for (int q = 0; q < SP; ++q) {
            x[q] = __builtin_nontemporal_load(reinterpret_cast<const vec *>(Xin + (i64)row * ld + c0 + q * 16384));
            if (SWAPPED) x[q] = x[q] - gamma * vload<4>(G + (i64)row * ld + c0 + q * 16384);
        }
    };
    auto put = [&](int row, const vec (&x)[SP]) {
#pragma unroll
        for (int q = 0; q < SP; ++q) slab[((size_t)row * SP + q) * 64 + lane] = x[q];
    };
    {
        int row = rg;
        for (; row + rgroups < n; row += 2 * rgroups) {   // two rows of SP vectors in flight
            vec a[SP], b[SP];
            stage(row, a);
            stage(row + rgroups, b);
            put(row, a);
            put(row + rgroups, b);
        }
        for (; row < n; row += rgroups) {
            vec a[SP];
            stage(row, a);
            put(row, a);
        }
    }
    __syncthreads();   // the whole slab is in LDS; from here on rows may be overwritten

    ColStats<4> st[SP];
#pragma unroll
    for (int q = 0; q < SP; ++q) st[q].init();
    auto gload = [&](int row, vec (&g)[SP]) {
#pragma unroll
        for (int q = 0; q < SP; ++q) {
            if (SWAPPED) { g[q] = (vec)(0.f); continue; }
            g[q] = __builtin_nontemporal_load(reinterpret_cast<const vec *>(G + (i64)row * ld + c0 + q * 16384));
            if (Vel) {
                float *vdst = Vel + (i64)row * ld + c0 + q * 16384;
                g[q] = mu * vload<4>(vdst) + g[q];
                vstore<4>(vdst, g[q]);
            }
        }
    };
    auto form = [&](int row, const vec (&g)[SP]) {
        const int p0 = rowptr[row], p1 = rowptr[row + 1];
        vec acc[SP];
#pragma unroll
        for (int q = 0; q < SP; ++q) acc[q] = (vec)(0.f);
        for (int p = p0; p < p1; ++p) {
            const float wv = vals[p];
            const size_t src = (size_t)colidx[p] * SP;
#pragma unroll
            for (int q = 0; q < SP; ++q) acc[q] = wv * slab[(src + q) * 64 + lane] + acc[q];
        }
#pragma unroll
        for (int q = 0; q < SP; ++q) {
            const vec o = SWAPPED ? acc[q] : acc[q] - gamma * g[q];
            __builtin_nontemporal_store(o, reinterpret_cast<vec *>(Xout + (i64)row * ld + c0 + q * 16384));
            if (CONS) st[q].add(o);
        }
    };
    {
        int row = rg;
        for (; row + rgroups < n; row += 2 * rgroups) {
            vec g0[SP], g1[SP];
            gload(row, g0);
            gload(row + rgroups, g1);
            form(row, g0);
            form(row + rgroups, g1);
        }
        for (; row < n; row += rgroups) {
            vec g0[SP];
            gload(row, g0);
            form(row, g0);
        }
    }
    if (CONS) {
        double v = 0.0;
#pragma unroll
        for (int q = 0; q < SP; ++q) {
            __syncthreads();   // the slab (q = 0) or the previous vector's statistics are no longer needed
            combine_bands<4>(st[q], lds, rg, lane, rgroups);
            if (rg == 0) v += wave_sum((double)st[q].m2());
        }
        if (rg == 0 && lane == 0) partials[blockIdx.x] = v;
    }
}

// ------------------------------------------------------------- CSR without a slab (large n)
// One thread per (row, column); neighbours are gathered from global memory.  Out of place only.
template <bool SWAPPED>
__global__ void __launch_bounds__(256)
mix_csr_gather_kernel(const float *__restrict__ Xin, const float *__restrict__ G, float *__restrict__ Xout, int n,
                      i64 ncols, i64 ld, const int *__restrict__ rowptr, const int *__restrict__ colidx,
                      const float *__restrict__ vals, float gamma, float *__restrict__ Vel, float mu)
{
    const i64 c = (i64)blockIdx.x * 256 + threadIdx.x;
    const int row = blockIdx.y;
    if (c >= ncols || row >= n) return;
    float acc = 0.f;
    for (int p = rowptr[row]; p < rowptr[row + 1]; ++p) {
        const i64 j = colidx[p];
        float x = Xin[j * ld + c];
        if (SWAPPED) x -= gamma * G[j * ld + c];
        acc = vals[p] * x + acc;
    }
    if (SWAPPED) {
        Xout[(i64)row * ld + c] = acc;
        return;
    }
    float g = G[(i64)row * ld + c];
    if (Vel) {
        g = mu * Vel[(i64)row * ld + c] + g;
        Vel[(i64)row * ld + c] = g;
    }
    Xout[(i64)row * ld + c] = acc - gamma * g;
}

// ---------------------------------------------------------------- column statistics / mean
// Same slab ownership as the ring kernel (lane = V columns, wave = row band), read only.
// MEAN: writes xbar.  CONS: writes the per-workgroup partial of sum_i ||x_i - xbar||^2.
template <int V, bool MEAN, bool CONS>
__global__ void __launch_bounds__(512)
column_stats_kernel(const float *__restrict__ X, int n, i64 ncols, i64 ld, int bands, int rpb, float inv_n,
                    float *__restrict__ xbar, double *__restrict__ partials)
{
    typedef typename VecT<V>::type vec;
    extern __shared__ float lds[];
    const int lane = threadIdx.x & 63;
    const int band = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const i64 c0 = ((i64)blockIdx.x * 64 + lane) * V;
    const bool active = c0 + V <= ncols;
    const int r0 = band * rpb, r1 = min(n, r0 + rpb);
    ColStats<V> st;
    st.init();
    vec sum = (vec)(0.f);
    if (active) {
        const float *x = X + c0;
#pragma unroll 4
        for (int row = r0; row < r1; ++row) {
            vec v = __builtin_nontemporal_load(reinterpret_cast<const vec *>(x + (i64)row * ld));
            if (MEAN) sum += v;
            if (CONS) st.add(v);
        }
    }
    if (MEAN) {
        vec *acc = reinterpret_cast<vec *>(lds);   // [bands][64]
        if (bands > 1) {
            acc[(size_t)band * 64 + lane] = sum;
            __syncthreads();
            if (band == 0)
                for (int b = 1; b < bands; ++b) sum += acc[(size_t)b * 64 + lane];   // ascending rows
            __syncthreads();
        }
        if (band == 0 && active) vstore<V>(xbar + c0, sum * inv_n);
    }
    if (CONS) {
        combine_bands<V>(st, lds, band, lane, bands);
        if (band == 0) {
            double v = wave_sum((double)st.m2());
            if (lane == 0) partials[blockIdx.x] = v;
        }
    }
}

// The node average of a wide matrix with fat lanes and the chunked column ownership of mix_ring_fat_kernel (one wave
// per workgroup, P float4 column groups per lane, 512-byte chunks 32 KB apart): the same sums in the same order
// (rows ascending), read faster.  grid.x = 64 x (ncols / fat_super<P>()), block 64; 16-byte aligned rows.
template <int P>
__global__ void __launch_bounds__(64)
column_mean_fat_kernel(const float *__restrict__ X, int n, i64 ld, float inv_n, float *__restrict__ xbar)
{
    typedef VecT<4>::type vec;
    const int lane = threadIdx.x;
    constexpr i64 kPerSuper = kFatStride / (kFatChunkLanes * 4);
    constexpr i64 kStep = (64 / kFatChunkLanes) * kFatStride;
    const i64 sb = blockIdx.x / kPerSuper, k = blockIdx.x % kPerSuper;
    const i64 c0 = sb * fat_super<P>() + k * (kFatChunkLanes * 4) + (lane % kFatChunkLanes) * 4 +
                   (i64)(lane / kFatChunkLanes) * kFatStride;
    vec sum[P];
#pragma unroll
    for (int q = 0; q < P; ++q) sum[q] = (vec)(0.f);
    int row = 0;
    for (; row + 2 <= n; row += 2) {   // two rows (2 P loads per lane) in flight
        vec a[P], b[P];
#pragma unroll
        for (int q = 0; q < P; ++q) {
            a[q] = __builtin_nontemporal_load(reinterpret_cast<const vec *>(X + (i64)row * ld + c0 + (i64)q * kStep));
            b[q] = __builtin_nontemporal_load(reinterpret_cast<const vec *>(X + (i64)(row + 1) * ld + c0 + (i64)q * kStep));
        }
#pragma unroll
        for (int q = 0; q < P; ++q) {
            sum[q] += a[q];
            sum[q] += b[q];
        }
    }
    for (; row < n; ++row)
#pragma unroll
        for (int q = 0; q < P; ++q)
            sum[q] += __builtin_nontemporal_load(reinterpret_cast<const vec *>(X + (i64)row * ld + c0 + (i64)q * kStep));
#pragma unroll
    for (int q = 0; q < P; ++q) vstore<4>(xbar + c0 + (i64)q * kStep, sum[q] * inv_n);
}

// Fixed-order sum of the per-workgroup partials in two stages: block b of the first stage sums the
// contiguous slice [b*per, (b+1)*per) into stage1[b]; the second stage (one block) adds those and
// writes consensus = (sum partials) / n.  The order depends only on the launch shape.
__device__ __forceinline__ double block_sum_256(double s, double *sh)
{
    sh[threadIdx.x] = s;
    __syncthreads();
    for (int off = 128; off > 0; off >>= 1) {
        if ((int)threadIdx.x < off) sh[threadIdx.x] += sh[threadIdx.x + off];
        __syncthreads();
    }
    return sh[0];
}

__global__ void __launch_bounds__(256) consensus_stage1_kernel(const double *__restrict__ partials, i64 count, i64 per,
                                                                double *__restrict__ stage1)
{
    __shared__ double sh[256];
    const i64 lo = (i64)blockIdx.x * per, hi = lo + per < count ? lo + per : count;
    double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
    i64 i = lo + threadIdx.x;
    for (; i + 768 < hi; i += 1024) {
        s0 += partials[i];
        s1 += partials[i + 256];
        s2 += partials[i + 512];
        s3 += partials[i + 768];
    }
    for (; i < hi; i += 256) s0 += partials[i];
    const double t = block_sum_256((s0 + s1) + (s2 + s3), sh);
    if (threadIdx.x == 0) stage1[blockIdx.x] = t;
}

__global__ void __launch_bounds__(256) consensus_stage2_kernel(const double *__restrict__ stage1, int count, double inv_n,
                                                                float *__restrict__ out)
{
    __shared__ double sh[256];
    double s = 0.0;
    for (int i = threadIdx.x; i < count; i += 256) s += stage1[i];
    const double t = block_sum_256(s, sh);
    if (threadIdx.x == 0) out[0] = (float)(t * inv_n);
}

// Few partials (up to kSmallCount): both stages in one workgroup, one launch instead of two.
__global__ void __launch_bounds__(256) consensus_small_kernel(const double *__restrict__ partials, int count, double inv_n,
                                                               float *__restrict__ out)
{
    __shared__ double sh[256];
    double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
    int i = threadIdx.x;
    for (; i + 768 < count; i += 1024) {
        s0 += partials[i];
        s1 += partials[i + 256];
        s2 += partials[i + 512];
        s3 += partials[i + 768];
    }
    for (; i < count; i += 256) s0 += partials[i];
    const double t = block_sum_256((s0 + s1) + (s2 + s3), sh);
    if (threadIdx.x == 0) out[0] = (float)(t * inv_n);
}

// --------------------------------------------------------------------------- host helpers
struct Plan {
    int vec;        // floats per lane for the bulk launch
    i64 bulk_cols;  // columns covered by the vector launch (multiple of vec)
    i64 tail_cols;  // remaining columns, handled with vec = 1
};

bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

int pick_vec(const dpsgd_ctx *ctx, std::initializer_list<const void *> ptrs, int cap)
{
    int v = 4;
    if (ctx->opt_mix_vec) v = ctx->opt_mix_vec;
    if (v > cap) v = cap;
    while (v > 1) {
        bool ok = (ctx->ld % v) == 0;
        for (const void *p : ptrs) ok = ok && aligned(p, sizeof(float) * (size_t)v);
        if (ok && ctx->d >= v) break;
        v >>= 1;
    }
    return v;
}

Plan make_plan(const dpsgd_ctx *ctx, int vec)
{
    Plan p;
    p.vec = vec;
    p.bulk_cols = ctx->d - ctx->d % vec;
    p.tail_cols = ctx->d - p.bulk_cols;
    return p;
}

i64 groups_for(i64 cols, int vec) { return (cols + 64LL * vec - 1) / (64LL * vec); }

// Row bands per workgroup: one band when there are already plenty of waves, more when the
// matrix is narrow, so that the chip still sees a few thousand waves.
constexpr int kMaxBands = 8;   // the ring kernel is compiled for at most 8 waves per workgroup

int pick_bands(const dpsgd_ctx *ctx, i64 groups)
{
    int bands = ctx->opt_mix_bands;
    if (bands == 0) {
        bands = 1;
        while (bands < kMaxBands && groups * bands < 8192 && ctx->n / (bands * 2) >= 4) bands *= 2;
    }
    if (bands > kMaxBands) bands = kMaxBands;
    if (bands > ctx->n) bands = ctx->n;
    if (bands < 1) bands = 1;
    return bands;
}

size_t stats_lds_bytes(int bands, int vec) { return bands > 1 ? (size_t)bands * 64 * (3 * vec + 1) * sizeof(float) : 0; }

// tail: columns right after [col0, col0 + ncols) that the same launch walks one per lane (V > 1, tail < V)
template <int V>
dpsgd_status ring_launch(dpsgd_ctx *ctx, const float *Xin, const float *G, float *Xout, i64 col0, i64 ncols,
                         bool cons, double *partials, i64 *nparts, float *Vel = nullptr, float mu = 0.f,
                         bool narrow = false, int tail = 0)
{
    const i64 groups = groups_for(ncols, V);
    const int bands = pick_bands(ctx, groups);
    constexpr int kFatP = 8;              // float4 groups per lane of the fat-lane kernel
    constexpr i64 kFatMinSupers = 64;     // 64 x 64 single-wave workgroups: enough to fill the chip
    if (V == 4 && bands == 1 && !narrow && !ctx->opt_mix_narrow && ctx->opt_mix_bands == 0 && ctx->n >= 3 &&
        ncols / fat_super<kFatP>() >= kFatMinSupers) {
        // wide matrix: whole super-blocks of columns go to the fat-lane kernel, the rest to the kernel below
        const i64 supers = ncols / fat_super<kFatP>(), fat_cols = supers * fat_super<kFatP>();
        const i64 fat_groups = supers * (kFatStride / (kFatChunkLanes * 4));
        if (fat_groups > 0x7fffffffLL) return DPSGD_EUNSUPPORTED;
        float *velc = Vel ? Vel + col0 : nullptr;
#define DPSGD_FAT(U, CONS, MOM)                                                                                          \
    hipLaunchKernelGGL((mix_ring_fat_kernel<kFatP, U, CONS, MOM>), dim3((unsigned)fat_groups), dim3(64), 0, ctx->stream, \
                       Xin + col0, G + col0, Xout + col0, ctx->n, ctx->ld, ctx->ring_w, ctx->gamma, partials, velc, mu)
        if (cons && velc) DPSGD_FAT(1, true, true);
        else if (cons) DPSGD_FAT(1, true, false);
        else if (velc) DPSGD_FAT(1, false, true);
        else DPSGD_FAT(1, false, false);
#undef DPSGD_FAT
        dpsgd_status st = hip_status(hipGetLastError());
        i64 rest = 0;
        if (st == DPSGD_OK && fat_cols < ncols)
            st = ring_launch<V>(ctx, Xin, G, Xout, col0 + fat_cols, ncols - fat_cols, cons, partials + fat_groups, &rest,
                                Vel, mu, true, tail);
        else if (st == DPSGD_OK && tail)
            st = ring_launch<1>(ctx, Xin, G, Xout, col0 + ncols, tail, cons, partials + fat_groups, &rest, Vel, mu);
        *nparts = fat_groups + rest;
        return st;
    }
    const int rpb = (ctx->n + bands - 1) / bands;
    const int used = (ctx->n + rpb - 1) / rpb;   // every launched band owns at least one row
    const i64 wgs = groups + ((V > 1 && tail > 0) ? 1 : 0);
    dim3 grid((unsigned)wgs), block(64u * (unsigned)used);
    if (wgs > 0x7fffffffLL || tail >= V) return DPSGD_EUNSUPPORTED;
    const size_t shm = cons ? stats_lds_bytes(used, V) : 0;
    float *vel = Vel ? Vel + col0 : nullptr;
#define DPSGD_RING(CONS, MOM)                                                                                        \
    hipLaunchKernelGGL((mix_ring_kernel<V, 4, CONS, MOM>), grid, block, shm, ctx->stream, Xin + col0, G + col0,      \
                       Xout + col0, ctx->n, ncols, ctx->ld, ctx->ring_w, ctx->gamma, used, rpb, partials, vel, mu, tail)
    if (cons && vel) DPSGD_RING(true, true);
    else if (cons) DPSGD_RING(true, false);
    else if (vel) DPSGD_RING(false, true);
    else DPSGD_RING(false, false);
#undef DPSGD_RING
    *nparts = wgs;
    return hip_status(hipGetLastError());
}

constexpr size_t kSlabLdsBudget = 64 * 1024;

// Wide part of a slab launch: whole super-blocks with SP float4 per lane.  Returns the columns it took (0: none).
template <int SP, bool SWAPPED>
dpsgd_status slab_wide_launch(dpsgd_ctx *ctx, const float *Xin, const float *G, float *Xout, i64 col0, i64 ncols, bool cons,
                              double *partials, float *vel, float mu, i64 *cols_done, i64 *parts)
{
    const i64 supers = ncols / slab_super<SP>();
    const i64 groups = supers * 64;
    if (groups > 0x7fffffffLL) return DPSGD_EUNSUPPORTED;
    const int rgroups = ctx->n < 8 ? ctx->n : (SP > 1 ? 8 : 4);
    size_t shm = (size_t)ctx->n * 64 * SP * 16;
    if (cons && stats_lds_bytes(rgroups, 4) > shm) shm = stats_lds_bytes(rgroups, 4);
    if (cons) {
        auto k = mix_csr_slab_wide_kernel<SP, true, SWAPPED>;
        if (shm > 64 * 1024 &&
            hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)shm) != hipSuccess)
            return DPSGD_EDEVICE;
        hipLaunchKernelGGL(k, dim3((unsigned)groups), dim3(64u * (unsigned)rgroups), shm, ctx->stream, Xin + col0, G + col0,
                           Xout + col0, ctx->n, ctx->ld, ctx->d_rowptr, ctx->d_colidx, ctx->d_vals, ctx->gamma, rgroups,
                           partials, vel, mu);
    } else {
        auto k = mix_csr_slab_wide_kernel<SP, false, SWAPPED>;
        if (shm > 64 * 1024 &&
            hipFuncSetAttribute(reinterpret_cast<const void *>(k), hipFuncAttributeMaxDynamicSharedMemorySize, (int)shm) != hipSuccess)
            return DPSGD_EDEVICE;
        hipLaunchKernelGGL(k, dim3((unsigned)groups), dim3(64u * (unsigned)rgroups), shm, ctx->stream, Xin + col0, G + col0,
                           Xout + col0, ctx->n, ctx->ld, ctx->d_rowptr, ctx->d_colidx, ctx->d_vals, ctx->gamma, rgroups,
                           partials, vel, mu);
    }
    *cols_done = supers * slab_super<SP>();
    *parts = groups;
    return hip_status(hipGetLastError());
}

constexpr size_t kSlabWideLdsBudget = 128 * 1024;   // one workgroup per CU with two float4 per lane

template <int V, bool SWAPPED>
dpsgd_status slab_launch(dpsgd_ctx *ctx, const float *Xin, const float *G, float *Xout, i64 col0, i64 ncols,
                         bool cons, double *partials, i64 *nparts, float *Vel = nullptr, float mu = 0.f)
{
    float *vel = Vel ? Vel + col0 : nullptr;
    // wide matrices: whole super-blocks of columns with the chunked column ownership, the rest consecutively
    i64 done = 0, parts = 0;
    if (V == 4 && !ctx->opt_mix_narrow) {
        dpsgd_status st = DPSGD_OK;
        if (ncols / slab_super<2>() >= 16 && (size_t)ctx->n * 64 * 2 * 16 <= kSlabWideLdsBudget && ctx->opt_mix_vec != 1)
            st = slab_wide_launch<2, SWAPPED>(ctx, Xin, G, Xout, col0, ncols, cons, partials, vel, mu, &done, &parts);
        else if (ncols / slab_super<1>() >= 32)
            st = slab_wide_launch<1, SWAPPED>(ctx, Xin, G, Xout, col0, ncols, cons, partials, vel, mu, &done, &parts);
        if (st != DPSGD_OK) return st;
    }
    const i64 groups = groups_for(ncols - done, V);
    if (groups > 0x7fffffffLL) return DPSGD_EUNSUPPORTED;
    if (groups > 0) {
        int rgroups = ctx->n < 4 ? ctx->n : 4;
        size_t shm = (size_t)ctx->n * 64 * V * sizeof(float);
        const size_t stats = stats_lds_bytes(rgroups, V);
        if (cons && stats > shm) shm = stats;
        dim3 grid((unsigned)groups), block(64u * (unsigned)rgroups);
        const float *xi = Xin + col0 + done, *gi = G + col0 + done;
        float *xo = Xout + col0 + done, *ve = vel ? vel + done : nullptr;
        if (cons)
            hipLaunchKernelGGL((mix_csr_slab_kernel<V, true, SWAPPED>), grid, block, shm, ctx->stream, xi, gi, xo, ctx->n,
                               ncols - done, ctx->ld, ctx->d_rowptr, ctx->d_colidx, ctx->d_vals, ctx->gamma, rgroups,
                               partials + parts, ve, mu);
        else
            hipLaunchKernelGGL((mix_csr_slab_kernel<V, false, SWAPPED>), grid, block, shm, ctx->stream, xi, gi, xo, ctx->n,
                               ncols - done, ctx->ld, ctx->d_rowptr, ctx->d_colidx, ctx->d_vals, ctx->gamma, rgroups,
                               partials + parts, ve, mu);
    }
    *nparts = parts + groups;
    return hip_status(hipGetLastError());
}

template <int V, bool MEAN, bool CONS>
dpsgd_status stats_launch(dpsgd_ctx *ctx, const float *X, i64 col0, i64 ncols, float *xbar, double *partials,
                          i64 *nparts)
{
    const i64 groups = groups_for(ncols, V);
    if (groups > 0x7fffffffLL) return DPSGD_EUNSUPPORTED;
    const int bands = pick_bands(ctx, groups);
    const int rpb = (ctx->n + bands - 1) / bands;
    const int used = (ctx->n + rpb - 1) / rpb;
    size_t shm = 0;
    if (MEAN && used > 1) shm = (size_t)used * 64 * V * sizeof(float);
    if (CONS && stats_lds_bytes(used, V) > shm) shm = stats_lds_bytes(used, V);
    hipLaunchKernelGGL((column_stats_kernel<V, MEAN, CONS>), dim3((unsigned)groups), dim3(64u * (unsigned)used), shm,
                       ctx->stream, X + col0, ctx->n, ncols, ctx->ld, used, rpb, 1.0f / (float)ctx->n,
                       xbar ? xbar + col0 : nullptr, partials);
    *nparts = groups;
    return hip_status(hipGetLastError());
}

constexpr int kStage1Blocks = 128;   // the partials buffer keeps this many extra slots at its end
constexpr i64 kSmallCount = 8192;    // up to this many partials one workgroup sums them in one launch

dpsgd_status finalize_consensus(dpsgd_ctx *ctx, i64 count, float *consensus)
{
    if (count <= kSmallCount) {
        hipLaunchKernelGGL(consensus_small_kernel, dim3(1), dim3(256), 0, ctx->stream, ctx->d_partials, (int)count,
                           1.0 / (double)ctx->n, consensus);
        return hip_status(hipGetLastError());
    }
    double *stage1 = ctx->d_partials + (ctx->partials_cap - kStage1Blocks);
    i64 per = (count + kStage1Blocks - 1) / kStage1Blocks;
    if (per < 256) per = 256;
    const int blocks = (int)((count + per - 1) / per);
    hipLaunchKernelGGL(consensus_stage1_kernel, dim3((unsigned)blocks), dim3(256), 0, ctx->stream, ctx->d_partials, count,
                       per, stage1);
    hipLaunchKernelGGL(consensus_stage2_kernel, dim3(1), dim3(256), 0, ctx->stream, stage1, blocks,
                       1.0 / (double)ctx->n, consensus);
    return hip_status(hipGetLastError());
}

// sum_i ||x_i - xbar||^2 / n of a matrix already in memory (used when the mix kernel itself
// cannot accumulate it).
dpsgd_status consensus_of(dpsgd_ctx *ctx, const float *X, float *consensus)
{
    const int vec = pick_vec(ctx, {X}, 4);
    const Plan p = make_plan(ctx, vec);
    i64 n1 = 0, n2 = 0;
    dpsgd_status st = DPSGD_OK;
    if (p.bulk_cols) {
        if (vec == 4) st = stats_launch<4, false, true>(ctx, X, 0, p.bulk_cols, nullptr, ctx->d_partials, &n1);
        else if (vec == 2) st = stats_launch<2, false, true>(ctx, X, 0, p.bulk_cols, nullptr, ctx->d_partials, &n1);
        else st = stats_launch<1, false, true>(ctx, X, 0, p.bulk_cols, nullptr, ctx->d_partials, &n1);
    }
    if (st == DPSGD_OK && p.tail_cols)
        st = stats_launch<1, false, true>(ctx, X, p.bulk_cols, p.tail_cols, nullptr, ctx->d_partials + n1, &n2);
    if (st != DPSGD_OK) return st;
    return finalize_consensus(ctx, n1 + n2, consensus);
}

}  // namespace

int64_t mix_partials_needed(const dpsgd_ctx *ctx)
{
    // one partial per workgroup of the widest possible launch (vec = 1) plus the tail launch
    return groups_for(ctx->d, 1) + 8 + kStage1Blocks;
}

dpsgd_status launch_mix(dpsgd_ctx *ctx, const float *Xin, const float *G, float *Xout, float *consensus, bool swapped,
                        float *Vel, float mu)
{
    if (Vel && swapped) return DPSGD_EUNSUPPORTED;
    const bool cons = consensus != nullptr;
    const bool ring = ctx->ring_uniform && !ctx->opt_mix_force_csr && !swapped;
    i64 n1 = 0, n2 = 0;
    dpsgd_status st = DPSGD_OK;

    if (ring) {
        const int vec = pick_vec(ctx, {Xin, G, Xout, Vel ? Vel : Xin}, 4);
        const Plan p = make_plan(ctx, vec);
        // the columns beyond the last whole vector ride along in the bulk launch (its last workgroup)
        const int tail = (int)p.tail_cols;
        if (p.bulk_cols) {
            if (vec == 4) st = ring_launch<4>(ctx, Xin, G, Xout, 0, p.bulk_cols, cons, ctx->d_partials, &n1, Vel, mu, false, tail);
            else if (vec == 2) st = ring_launch<2>(ctx, Xin, G, Xout, 0, p.bulk_cols, cons, ctx->d_partials, &n1, Vel, mu, false, tail);
            else st = ring_launch<1>(ctx, Xin, G, Xout, 0, p.bulk_cols, cons, ctx->d_partials, &n1, Vel, mu);
        }
        if (st == DPSGD_OK && p.tail_cols && (!p.bulk_cols || vec == 1))
            st = ring_launch<1>(ctx, Xin, G, Xout, p.bulk_cols, p.tail_cols, cons, ctx->d_partials + n1, &n2, Vel, mu);
        if (st != DPSGD_OK) return st;
        return cons ? finalize_consensus(ctx, n1 + n2, consensus) : DPSGD_OK;
    }

    // widest vector whose n-row slab fits the LDS budget
    int cap = 4;
    while (cap >= 1 && (size_t)ctx->n * 64 * cap * sizeof(float) > kSlabLdsBudget) cap >>= 1;
    if (cap >= 1) {
        const int vec = pick_vec(ctx, {Xin, G, Xout, Vel ? Vel : Xin}, cap);
        const Plan p = make_plan(ctx, vec);
#define DPSGD_SLAB(V, C0, NC, PART, NP)                                                              \
    (swapped ? slab_launch<V, true>(ctx, Xin, G, Xout, C0, NC, cons, PART, NP)                       \
             : slab_launch<V, false>(ctx, Xin, G, Xout, C0, NC, cons, PART, NP, Vel, mu))
        if (p.bulk_cols) {
            if (vec == 4) st = DPSGD_SLAB(4, 0, p.bulk_cols, ctx->d_partials, &n1);
            else if (vec == 2) st = DPSGD_SLAB(2, 0, p.bulk_cols, ctx->d_partials, &n1);
            else st = DPSGD_SLAB(1, 0, p.bulk_cols, ctx->d_partials, &n1);
        }
        if (st == DPSGD_OK && p.tail_cols) st = DPSGD_SLAB(1, p.bulk_cols, p.tail_cols, ctx->d_partials + n1, &n2);
#undef DPSGD_SLAB
        if (st != DPSGD_OK) return st;
        return cons ? finalize_consensus(ctx, n1 + n2, consensus) : DPSGD_OK;
    }

    // n too large for an LDS slab: gather from global memory, out of place only
    if (Xin == Xout) return DPSGD_EUNSUPPORTED;
    const i64 gx = (ctx->d + 255) / 256;
    if (gx > 0x7fffffffLL || ctx->n > 65535) return DPSGD_EUNSUPPORTED;
    dim3 grid((unsigned)gx, (unsigned)ctx->n);
    if (swapped)
        hipLaunchKernelGGL(mix_csr_gather_kernel<true>, grid, dim3(256), 0, ctx->stream, Xin, G, Xout, ctx->n, ctx->d,
                           ctx->ld, ctx->d_rowptr, ctx->d_colidx, ctx->d_vals, ctx->gamma, nullptr, 0.f);
    else
        hipLaunchKernelGGL(mix_csr_gather_kernel<false>, grid, dim3(256), 0, ctx->stream, Xin, G, Xout, ctx->n,
                           ctx->d, ctx->ld, ctx->d_rowptr, ctx->d_colidx, ctx->d_vals, ctx->gamma, Vel, mu);
    st = hip_status(hipGetLastError());
    if (st != DPSGD_OK) return st;
    return cons ? consensus_of(ctx, Xout, consensus) : DPSGD_OK;
}

// Mix + step restricted to the columns [col0, col0 + ncols), in place or out of place: used when other kernels
// own the remaining columns.  Ring walk for Theorem 3's ring, the LDS-slab kernel for any other W whose n rows
// fit a slab.  Consensus partials are appended at d_partials[*nparts ...] and *nparts advanced.
dpsgd_status launch_mix_range(dpsgd_ctx *ctx, const float *Xin, const float *G, float *Xout, int64_t col0,
                              int64_t ncols, bool cons, int64_t *nparts)
{
    if (ncols <= 0) return DPSGD_OK;
    const bool ring = ctx->ring_uniform && !ctx->opt_mix_force_csr;
    int cap = 4;
    if (!ring) {
        while (cap >= 1 && (size_t)ctx->n * 64 * cap * sizeof(float) > kSlabLdsBudget) cap >>= 1;
        if (cap < 1) return DPSGD_EUNSUPPORTED;
    }
    int vec = cap;
    while (vec > 1) {
        const bool ok = (ctx->ld % vec) == 0 && aligned(Xin + col0, 4u * vec) && aligned(G + col0, 4u * vec) &&
                        aligned(Xout + col0, 4u * vec) && ncols >= vec;
        if (ok) break;
        vec >>= 1;
    }
    const i64 bulk = ncols - ncols % vec, tail = ncols - bulk;
    if (*nparts + groups_for(bulk, vec) + groups_for(tail, 1) + 2 > ctx->partials_cap - kStage1Blocks) return DPSGD_EINVAL;
    i64 n1 = 0, n2 = 0;
    dpsgd_status st = DPSGD_OK;
    double *part = ctx->d_partials + *nparts;
    if (ring) {
        if (bulk) {
            if (vec == 4) st = ring_launch<4>(ctx, Xin, G, Xout, col0, bulk, cons, part, &n1, nullptr, 0.f, false, (int)tail);
            else if (vec == 2) st = ring_launch<2>(ctx, Xin, G, Xout, col0, bulk, cons, part, &n1, nullptr, 0.f, false, (int)tail);
            else st = ring_launch<1>(ctx, Xin, G, Xout, col0, bulk, cons, part, &n1);
        }
        if (st == DPSGD_OK && tail && (!bulk || vec == 1))
            st = ring_launch<1>(ctx, Xin, G, Xout, col0 + bulk, tail, cons, part + n1, &n2);
    } else {
        if (bulk) {
            if (vec == 4) st = slab_launch<4, false>(ctx, Xin, G, Xout, col0, bulk, cons, part, &n1);
            else if (vec == 2) st = slab_launch<2, false>(ctx, Xin, G, Xout, col0, bulk, cons, part, &n1);
            else st = slab_launch<1, false>(ctx, Xin, G, Xout, col0, bulk, cons, part, &n1);
        }
        if (st == DPSGD_OK && tail) st = slab_launch<1, false>(ctx, Xin, G, Xout, col0 + bulk, tail, cons, part + n1, &n2);
    }
    if (cons) *nparts += n1 + n2;
    return st;
}

dpsgd_status launch_consensus_finalize(dpsgd_ctx *ctx, int64_t count, float *consensus)
{
    return finalize_consensus(ctx, count, consensus);
}

dpsgd_status launch_mean(dpsgd_ctx *ctx, const float *X, float *xbar)
{
    const int vec = pick_vec(ctx, {X, xbar}, 4);
    const Plan p = make_plan(ctx, vec);
    i64 np = 0;
    dpsgd_status st = DPSGD_OK;
    constexpr int kMeanP = 4;
    if (vec == 4 && !ctx->opt_mix_narrow && p.bulk_cols / fat_super<kMeanP>() >= 64) {
        // wide matrix: whole super-blocks of columns go to the fat-lane kernel, the rest to the kernel below
        const i64 supers = p.bulk_cols / fat_super<kMeanP>(), fat_cols = supers * fat_super<kMeanP>();
        const i64 groups = supers * (kFatStride / (kFatChunkLanes * 4));
        if (groups > 0x7fffffffLL) return DPSGD_EUNSUPPORTED;
        hipLaunchKernelGGL(column_mean_fat_kernel<kMeanP>, dim3((unsigned)groups), dim3(64), 0, ctx->stream, X, ctx->n, ctx->ld,
                           1.0f / (float)ctx->n, xbar);
        st = hip_status(hipGetLastError());
        if (st == DPSGD_OK && fat_cols < p.bulk_cols)
            st = stats_launch<4, true, false>(ctx, X, fat_cols, p.bulk_cols - fat_cols, xbar, nullptr, &np);
    } else if (p.bulk_cols) {
        if (vec == 4) st = stats_launch<4, true, false>(ctx, X, 0, p.bulk_cols, xbar, nullptr, &np);
        else if (vec == 2) st = stats_launch<2, true, false>(ctx, X, 0, p.bulk_cols, xbar, nullptr, &np);
        else st = stats_launch<1, true, false>(ctx, X, 0, p.bulk_cols, xbar, nullptr, &np);
    }
    if (st == DPSGD_OK && p.tail_cols) st = stats_launch<1, true, false>(ctx, X, p.bulk_cols, p.tail_cols, xbar, nullptr, &np);
    return st;
}

// ------------------------------------------------------------------ allocation-free entry point
// dpsgd_mix_step for callers that cannot allocate: no context, no hipMalloc.  What the ordinary call keeps in
// buffers of its context (per-workgroup partial sums of the consensus distance, the device CSR of a torus) lives
// in one file-scope device array instead.  Every GPU the library runs on holds its own copy of the array, at its own
// address, until the process ends; the address is looked up once per device and only that pointer is ever used.
namespace {

constexpr size_t kStaticCsrBytes = 32 * 1024;                       // rowptr, colidx, vals of a torus with n <= 256
constexpr size_t kStaticPartialBytes = 4 * 1024 * 1024 + 32 * 1024;
constexpr size_t kStaticScratchBytes = kStaticPartialBytes + kStaticCsrBytes;
constexpr int64_t kStaticMaxD = (int64_t)1 << 25;                   // 33 554 432 parameters per worker
constexpr int32_t kStaticMaxTorusN = 256;
constexpr int kStaticMaxDevices = 64;

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

void *g_scratch_ptr[kStaticMaxDevices];   // per device: device address of `scratch`, NULL until looked up
std::mutex g_scratch_mutex;

// Device address of this device's copy of the array (looked up on the first call per device).
dpsgd_status static_scratch(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kStaticMaxDevices) return DPSGD_EDEVICE;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) {
            (void)hipGetLastError();
            return DPSGD_EDEVICE;
        }
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return DPSGD_OK;
}

// CSR of the 2-D torus (both dimensions >= 3, so the five neighbours are distinct): worker i = r * C + c, itself and
// (r +- 1, c), (r, c +- 1) at weight w, columns ascending.  One thread per worker.
__global__ void __launch_bounds__(256) torus_csr_kernel(int R, int C, float w, int *__restrict__ rowptr,
                                                        int *__restrict__ colidx, float *__restrict__ vals)
{
    const int i = blockIdx.x * 256 + threadIdx.x;
    const int n = R * C;
    if (i > n) return;
    rowptr[i] = 5 * i;
    if (i == n) return;
    const int r = i / C, c = i % C;
    int nb[5] = {i, ((r + 1) % R) * C + c, ((r + R - 1) % R) * C + c, r * C + (c + 1) % C, r * C + (c + C - 1) % C};
    for (int a = 1; a < 5; ++a) {   // insertion sort of five
        const int v = nb[a];
        int b = a - 1;
        while (b >= 0 && nb[b] > v) {
            nb[b + 1] = nb[b];
            --b;
        }
        nb[b + 1] = v;
    }
    for (int a = 0; a < 5; ++a) {
        colidx[5 * i + a] = nb[a];
        vals[5 * i + a] = w;
    }
}

bool ranges_overlap(const void *a, const void *b, size_t bytes)
{
    const char *pa = (const char *)a, *pb = (const char *)b;
    return pa < pb + bytes && pb < pa + bytes;
}

}  // namespace
}  // namespace dpsgd

extern "C" dpsgd_status dpsgd_mix_step_static(int32_t n, int64_t d, int64_t ld, const dpsgd_topology *W, float gamma,
                                              const float *X_in, const float *G, float *X_out, float *consensus,
                                              void *hip_stream)
{
    using namespace dpsgd;
    if (n < 1 || d < 1 || !W || !X_in || !G || !X_out || !(gamma == gamma) || gamma - gamma != 0.f) return DPSGD_EINVAL;
    if (ld == 0) ld = d;
    if (ld < d || (double)n * (double)ld > 9.0e18 / 4.0) return DPSGD_EINVAL;
    const size_t bytes = (size_t)n * (size_t)ld * sizeof(float);
    if (ranges_overlap(G, X_out, bytes)) return DPSGD_EINVAL;
    if (X_out != X_in && ranges_overlap(X_in, X_out, bytes)) return DPSGD_EINVAL;
    const bool ring = W->kind == DPSGD_TOPO_RING && n >= 3;
    const bool torus = W->kind == DPSGD_TOPO_TORUS2D && W->dim0 >= 3 && W->dim1 >= 3 && (int64_t)W->dim0 * W->dim1 == n;
    if (W->kind == DPSGD_TOPO_TORUS2D && (W->dim0 < 1 || W->dim1 < 1 || (int64_t)W->dim0 * W->dim1 != n)) return DPSGD_EINVAL;
    // sizes beyond what the fixed array holds, and weight matrices that would need a CSR built on the host
    if (!ring && !torus) return DPSGD_EUNSUPPORTED;
    if (d > kStaticMaxD) return DPSGD_EUNSUPPORTED;
    if (torus && n > kStaticMaxTorusN) return DPSGD_EUNSUPPORTED;

    void *base = nullptr;
    dpsgd_status st = static_scratch(&base);
    if (st != DPSGD_OK) return st;

    dpsgd_ctx ctx;   // a description on the stack: owns nothing, frees nothing
    ctx.n = n;
    ctx.d = d;
    ctx.ld = ld;
    ctx.gamma = gamma;
    ctx.stream = (hipStream_t)hip_stream;
    ctx.topo_kind = W->kind;
    ctx.dim0 = W->dim0;
    ctx.dim1 = W->dim1;
    ctx.d_partials = (double *)base;
    ctx.partials_cap = (int64_t)(kStaticPartialBytes / sizeof(double));
    if (mix_partials_needed(&ctx) > ctx.partials_cap) return DPSGD_EUNSUPPORTED;
    if (ring) {
        ctx.ring_uniform = true;
        ctx.ring_w = (float)(1.0 / 3.0);
    } else {
        ctx.torus_uniform = true;
        ctx.torus_w = (float)(1.0 / 5.0);
        unsigned char *csr = (unsigned char *)base + kStaticPartialBytes;
        ctx.d_rowptr = (int32_t *)csr;
        ctx.d_colidx = (int32_t *)(csr + 2048);              // (256 + 1) * 4 bytes of row pointers fit in front
        ctx.d_vals = (float *)(csr + 2048 + 5 * kStaticMaxTorusN * sizeof(int32_t));
        hipLaunchKernelGGL(torus_csr_kernel, dim3((unsigned)(n / 256 + 1)), dim3(256), 0, ctx.stream, W->dim0, W->dim1,
                           ctx.torus_w, ctx.d_rowptr, ctx.d_colidx, ctx.d_vals);
        if (hipGetLastError() != hipSuccess) return DPSGD_EDEVICE;
    }
    return launch_mix(&ctx, X_in, G, X_out, consensus, false);
}


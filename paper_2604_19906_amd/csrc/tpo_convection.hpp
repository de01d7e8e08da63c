// Volume integral of the convective flux (Eq. 1 of the paper).  Per component c and element e:
// the sum over the three flux directions d of a tensor-product operator on the metric-weighted
// flux of that direction, the differentiation matrix D along direction d and the interpolation
// matrix I along the other two.  Cube axes are called l (fastest), m, n below; direction 0 is l:
//
//   F[c,e] = (I (x) I (x) D) (M.P0) + (I (x) D (x) I) (M.P1) + (D (x) I (x) I) (M.P2),
//
// the three factors of a Kronecker product acting on axes n, m, l in that order.  Written here
// for square D, I (as many nodes as quadrature points per direction).  Sum-factorised and with
// the three terms merged as early as the algebra allows, eight mode products per (c, e) instead
// of nine:
//   axis l:  a0 = D (M.P0),  a1 = I (M.P1),  a2 = I (M.P2)
//   axis m:  b01 = I a0 + D a1,  b2 = I a2
//   axis n:  F = I b01 + D b2
// One lane owns one pencil (as in tpo_pencil.hpp), the matrix entries arrive in SGPRs, the
// intermediate cubes live in LDS (three, then two).  A workgroup handles G units; a unit is
// one (element, component) pair, numbered 3*e + c so that the three components of an element,
// which share M_e, run next to each other and find it in cache.  Loads: each lane reads the n
// consecutive words of M_e and of the three P cubes that belong to its (n,m) pencil; stores
// are coalesced (lanes consecutive along (j,i)).
#pragma once
#include <hip/hip_runtime.h>

#include "tpo_pencil.hpp"
#include "tpo_pencil_mm.hpp"

namespace tpo {

// Workgroups are dealt round-robin to the 8 accelerator dies, each with its own L2.  With
// SAME_DIE the batches of units are renumbered so that three consecutive batches run on ONE die
// one after the other: block b (die b & 7, slot b >> 3) takes batch ((slot / 3) * 8 + die) * 3 +
// slot % 3.  The three components of an element then find M_e in that die's L2 instead of
// fetching it from HBM three times (measured: 12.1 -> 10.1 cubes read per element at n = 11).
// The grid must be convection_grid<SAME_DIE>(number of batches); blocks past the end exit.
template <bool SAME_DIE>
__host__ __device__ inline long long convection_grid(long long nbatch)
{
    return SAME_DIE ? 24 * ((nbatch + 23) / 24) : nbatch;
}
template <bool SAME_DIE>
__device__ __forceinline__ long long convection_batch()
{
    if constexpr (SAME_DIE) {
        const long long die = blockIdx.x & 7, slot = blockIdx.x >> 3;
        return ((slot / 3) * 8 + die) * 3 + slot % 3;
    } else {
        return blockIdx.x;
    }
}

// SPLIT (two LDS cubes per unit, two more barriers) pays once three cubes of a unit pass about
// 20 KB (fp64 n = 11: 0.825 against 0.87 ms; fp32 n = 13: 1.73 against 1.82 ms; fp64 n = 8 with
// 13 KB: 0.61 against 0.60 ms).
template <typename T, int N>
constexpr bool convection_split()
{
    return 3 * PencilShape<T, N, 1>::CUBE * sizeof(T) > 20 * 1024;
}
// Units per workgroup: best lane utilisation with at most 512 threads and 56 KB of LDS.
template <typename T, int N>
constexpr int convection_group()
{
    const long cubes = convection_split<T, N>() ? 2 : 3;
    int best = 1;
    long best_num = 0, best_den = 1;
    for (int g = 1; g <= 64; ++g) {
        const int p = g * N * N;
        const int nt = ((p + 63) / 64) * 64;
        const long lds = cubes * g * PencilShape<T, N, 1>::CUBE * (long)sizeof(T);
        if (g > 1 && (nt > 512 || lds > 56 * 1024)) break;
        if ((long)p * best_den > best_num * nt) {
            best = g;
            best_num = p;
            best_den = nt;
        }
    }
    return best;
}

// HINT bit 0 / 1: non-temporal loads / stores.  XCD: the SAME_DIE renumbering above.
// SPLIT: the third term's axis-l and axis-m products run after the first two terms have been
// merged, in the LDS cube that merge frees: two cubes per unit instead of three (more
// workgroups per CU) for two more barriers.
template <typename T, int N, int G, int HINT, bool XCD, bool SPLIT = false>
__global__ void __launch_bounds__((PencilShape<T, N, G>::NT))
convection_pencil_kernel(const T *__restrict__ Pq, const T *__restrict__ Mq, const T *Dm_,
                         const T *Im_, T *__restrict__ F, long long num_elems)
{
    using Sh = PencilShape<T, N, G>;
    constexpr int P = Sh::P, PA = Sh::PA, PB = Sh::PB, CUBE = Sh::CUBE;
    extern __shared__ __align__(16) unsigned char tpo_lds[];
    T *lds = reinterpret_cast<T *>(tpo_lds);

    const TPO_CONSTANT T *Dm = (const TPO_CONSTANT T *)Dm_;
    const TPO_CONSTANT T *Im = (const TPO_CONSTANT T *)Im_;

    const int tid = threadIdx.x;
    const int g = tid / P;
    const int p = tid - g * P;
    const int hi = p / N;
    const int lo = p - hi * N;
    const long long units = 3 * num_elems;
    const long long nbatch = (units + G - 1) / G;
    const long long batch = convection_batch<XCD>();
    if (XCD && batch >= nbatch) return;                 // whole workgroup: no barrier is skipped
    const long long unit = batch * G + g;
    const bool on = (tid < G * P) && (unit < units);
    const long long e = on ? unit / 3 : 0;
    const int c = on ? (int)(unit - 3 * e) : 0;
    constexpr size_t QC = (size_t)N * N * N;

    T *c0 = lds + (size_t)(g < G ? g : 0) * (SPLIT ? 2 : 3) * CUBE;
    T *c1 = c0 + CUBE;
    T *c2 = SPLIT ? c1 : c1 + CUBE;

    T x[N], y[N], z[N];
    T x2[N];                     // SPLIT: M.P2 of the lane's (n,m) pencil, kept for later

    // axis l: lane (n,m) = (hi,lo) owns the n consecutive words [e][n][m][0..N-1] of M and P
    if (on) {
        T mq[N];
        load_words<(HINT & 1) != 0>(Mq + (size_t)e * QC + (size_t)(p * N), mq);
#pragma unroll
        for (int dir = 0; dir < 3; ++dir) {
            const size_t cube = ((size_t)(c * 3 + dir) * (size_t)num_elems + (size_t)e) * QC;
            load_words<(HINT & 1) != 0>(Pq + cube + (size_t)(p * N), x);
#pragma unroll
            for (int l = 0; l < N; ++l) x[l] *= mq[l];
            if (SPLIT && dir == 2) {
#pragma unroll
                for (int l = 0; l < N; ++l) x2[l] = x[l];
            } else {
                mode_product<T, N, false>(dir == 0 ? Dm : Im, x, y);
                T *dst = dir == 0 ? c0 : (dir == 1 ? c1 : c2);
#pragma unroll
                for (int i = 0; i < N; ++i) dst[hi * PA + lo * PB + i] = y[i];
            }
        }
    }
    __syncthreads();

    // axis m: lane (n,i) = (hi,lo)
    if (on) {
#pragma unroll
        for (int m = 0; m < N; ++m) x[m] = c0[hi * PA + m * PB + lo];
        mode_product<T, N, false>(Im, x, y);
#pragma unroll
        for (int m = 0; m < N; ++m) x[m] = c1[hi * PA + m * PB + lo];
        mode_product<T, N, false>(Dm, x, z);
#pragma unroll
        for (int j = 0; j < N; ++j) c0[hi * PA + j * PB + lo] = y[j] + z[j];
    }
    if constexpr (SPLIT) {
        __syncthreads();                      // every lane has read its pencils of cube 1
        if (on) {                             // axis l of the third term: lane (n,m)
            mode_product<T, N, false>(Im, x2, y);
#pragma unroll
            for (int i = 0; i < N; ++i) c2[hi * PA + lo * PB + i] = y[i];
        }
        __syncthreads();
    }
    if (on) {
#pragma unroll
        for (int m = 0; m < N; ++m) x[m] = c2[hi * PA + m * PB + lo];
        mode_product<T, N, false>(Im, x, y);
#pragma unroll
        for (int j = 0; j < N; ++j) c2[hi * PA + j * PB + lo] = y[j];
    }
    __syncthreads();

    // axis n: lane (j,i) = (hi,lo); stores are consecutive over lanes
    if (on) {
#pragma unroll
        for (int n = 0; n < N; ++n) x[n] = c0[n * PA + hi * PB + lo];
        mode_product<T, N, false>(Im, x, y);
#pragma unroll
        for (int n = 0; n < N; ++n) x[n] = c2[n * PA + hi * PB + lo];
        mode_product<T, N, false>(Dm, x, z);
        const size_t out = ((size_t)c * (size_t)num_elems + (size_t)e) * QC;
#pragma unroll
        for (int k = 0; k < N; ++k) gstore<(HINT & 2) != 0>(F + out + (size_t)(k * P + p), y[k] + z[k]);
    }
}

// fp32 form with the mode products issued as 4x4x1 matrix-core outer products
// (tpo_pencil_mm.hpp): same data movement; the coefficient tables of D and I (both used
// untransposed) stay in registers for the whole kernel.  The matrix instructions run on whole
// wavefronts, outside the `on` branches (their broadcast coefficients come from active lanes
// only); idle lanes carry zeros or stale LDS words and never store.
template <int N, int G, int HINT, bool XCD, bool SPLIT = false>
__global__ void __launch_bounds__((PencilShape<float, N, G>::NT))
convection_mm_kernel(const float *__restrict__ Pq, const float *__restrict__ Mq,
                     const float *__restrict__ Dm, const float *__restrict__ Im,
                     float *__restrict__ F, long long num_elems)
{
    using Sh = PencilShape<float, N, G>;
    using MS = MmShape<N>;
    constexpr int P = Sh::P, PA = Sh::PA, PB = Sh::PB, CUBE = Sh::CUBE, NY = MS::NY;
    extern __shared__ __align__(16) unsigned char tpo_lds[];
    float *lds = reinterpret_cast<float *>(tpo_lds);

    const TPO_CONSTANT float *Dc = (const TPO_CONSTANT float *)Dm;
    const TPO_CONSTANT float *Ic = (const TPO_CONSTANT float *)Im;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int g = tid / P;
    const int p = tid - g * P;
    const int hi = p / N;
    const int lo = p - hi * N;
    const long long units = 3 * num_elems;
    const long long nbatch = (units + G - 1) / G;
    const long long batch = convection_batch<XCD>();
    if (XCD && batch >= nbatch) return;
    const long long unit = batch * G + g;
    const bool on = (tid < G * P) && (unit < units);
    const long long e = on ? unit / 3 : 0;
    const int c = on ? (int)(unit - 3 * e) : 0;
    constexpr size_t QC = (size_t)N * N * N;

    // Lanes past the last pencil read (never write) slot 0; p < P keeps them inside the cube.
    float *c0 = lds + (size_t)(g < G ? g : 0) * (SPLIT ? 2 : 3) * CUBE;
    float *c1 = c0 + CUBE;
    float *c2 = SPLIT ? c1 : c1 + CUBE;

    float tab_d[MS::NTAB], tab_i[MS::NTAB];
#pragma unroll
    for (int t = 0; t < MS::NTAB; ++t) {
        tab_d[t] = mm_coef<N>(Dm, false, t, lane);
        tab_i[t] = mm_coef<N>(Im, false, t, lane);
    }

    float x[N], y[NY], z[NY], mq[N];
    float x2[N];                 // SPLIT: M.P2 of the lane's (n,m) pencil, kept for later

    // axis l: lane (n,m) = (hi,lo)
    if (on) {
        load_words<(HINT & 1) != 0>(Mq + (size_t)e * QC + (size_t)(p * N), mq);
    } else {
#pragma unroll
        for (int l = 0; l < N; ++l) mq[l] = 0.0f;
    }
#pragma unroll
    for (int dir = 0; dir < 3; ++dir) {
        if (on) {
            const size_t cube = ((size_t)(c * 3 + dir) * (size_t)num_elems + (size_t)e) * QC;
            load_words<(HINT & 1) != 0>(Pq + cube + (size_t)(p * N), x);
        } else {
#pragma unroll
            for (int l = 0; l < N; ++l) x[l] = 0.0f;
        }
#pragma unroll
        for (int l = 0; l < N; ++l) x[l] *= mq[l];
        if (SPLIT && dir == 2) {
#pragma unroll
            for (int l = 0; l < N; ++l) x2[l] = x[l];
        } else {
            if (dir == 0) mode_product_mm<N, false>(tab_d, Dc, x, y);
            else mode_product_mm<N, false>(tab_i, Ic, x, y);
            float *dst = dir == 0 ? c0 : (dir == 1 ? c1 : c2);
            if (on) {
#pragma unroll
                for (int i = 0; i < N; ++i) dst[hi * PA + lo * PB + i] = y[i];
            }
        }
    }
    __syncthreads();

    // axis m: lane (n,i) = (hi,lo)
#pragma unroll
    for (int m = 0; m < N; ++m) x[m] = c0[hi * PA + m * PB + lo];
    mode_product_mm<N, false>(tab_i, Ic, x, y);
#pragma unroll
    for (int m = 0; m < N; ++m) x[m] = c1[hi * PA + m * PB + lo];
    mode_product_mm<N, false>(tab_d, Dc, x, z);
    if (on) {
#pragma unroll
        for (int j = 0; j < N; ++j) c0[hi * PA + j * PB + lo] = y[j] + z[j];
    }
    if constexpr (SPLIT) {
        __syncthreads();                      // every lane has read its pencils of cube 1
        mode_product_mm<N, false>(tab_i, Ic, x2, y);       // axis l of the third term: lane (n,m)
        if (on) {
#pragma unroll
            for (int i = 0; i < N; ++i) c2[hi * PA + lo * PB + i] = y[i];
        }
        __syncthreads();
    }
#pragma unroll
    for (int m = 0; m < N; ++m) x[m] = c2[hi * PA + m * PB + lo];
    mode_product_mm<N, false>(tab_i, Ic, x, y);
    if (on) {
#pragma unroll
        for (int j = 0; j < N; ++j) c2[hi * PA + j * PB + lo] = y[j];
    }
    __syncthreads();

    // axis n: lane (j,i) = (hi,lo)
#pragma unroll
    for (int n = 0; n < N; ++n) x[n] = c0[n * PA + hi * PB + lo];
    mode_product_mm<N, false>(tab_i, Ic, x, y);
#pragma unroll
    for (int n = 0; n < N; ++n) x[n] = c2[n * PA + hi * PB + lo];
    mode_product_mm<N, false>(tab_d, Dc, x, z);
    if (on) {
        const size_t out = ((size_t)c * (size_t)num_elems + (size_t)e) * QC;
#pragma unroll
        for (int k = 0; k < N; ++k) gstore<(HINT & 2) != 0>(F + out + (size_t)(k * P + p), y[k] + z[k]);
    }
}

// ---- rectangular form: n_q quadrature points and n_v nodes per direction, n_q != n_v ----------
// Same scheme (vector-FMA pencils, two LDS cubes per unit, the third term's first two products
// after the merge of the first two terms); the lane sets differ per axis: n_q*n_q pencils along
// l, n_q*n_v along m, n_v*n_v along n.

// y[i] = sum_l A[i][l] * x[l], A [NV][NQ] row-major, entries through the scalar data path.
template <typename T, int NV, int NQ>
__device__ __forceinline__ void mode_product_rect(const TPO_CONSTANT T *A, const T (&x)[NQ], T (&y)[NV])
{
    asm volatile("" : "+s"(A));
#pragma unroll
    for (int i = 0; i < NV; ++i) {
        T acc = A[i * NQ] * x[0];
#pragma unroll
        for (int l = 1; l < NQ; ++l) acc = fma_(A[i * NQ + l], x[l], acc);
        y[i] = acc;
    }
}

template <typename T, int NV, int NQ, int G>
struct ConvRectShape {
    static constexpr int NB = NQ > NV ? NQ : NV;
    static constexpr int L = NB * NB;                          // lanes per unit
    static constexpr int NT = ((G * L + 63) / 64) * 64;
    static constexpr int PB = (NV & 1) ? NV : NV + 1;          // row pitch (fastest axis: i)
    static constexpr int PA = ((NB * PB) & 1) ? NB * PB : NB * PB + 1;
    static constexpr int CUBE = NQ * PA;
    static constexpr size_t LDS_BYTES = (size_t)2 * G * CUBE * sizeof(T);
};

template <typename T, int NV, int NQ, int G, int HINT, bool XCD>
__global__ void __launch_bounds__((ConvRectShape<T, NV, NQ, G>::NT))
convection_rect_kernel(const T *__restrict__ Pq, const T *__restrict__ Mq, const T *Dm_,
                       const T *Im_, T *__restrict__ F, long long num_elems)
{
    using Sh = ConvRectShape<T, NV, NQ, G>;
    constexpr int L = Sh::L, PA = Sh::PA, PB = Sh::PB, CUBE = Sh::CUBE;
    extern __shared__ __align__(16) unsigned char tpo_lds[];
    T *lds = reinterpret_cast<T *>(tpo_lds);

    const TPO_CONSTANT T *Dm = (const TPO_CONSTANT T *)Dm_;
    const TPO_CONSTANT T *Im = (const TPO_CONSTANT T *)Im_;

    const int tid = threadIdx.x;
    const int g = tid / L;
    const int p = tid - g * L;
    const long long units = 3 * num_elems;
    const long long nbatch = (units + G - 1) / G;
    const long long batch = convection_batch<XCD>();
    if (XCD && batch >= nbatch) return;                 // whole workgroup: no barrier is skipped
    const long long unit = batch * G + g;
    const bool live = (tid < G * L) && (unit < units);
    const long long e = live ? unit / 3 : 0;
    const int c = live ? (int)(unit - 3 * e) : 0;
    constexpr size_t QC = (size_t)NQ * NQ * NQ, VC = (size_t)NV * NV * NV;
    const bool on_l = live && p < NQ * NQ;              // pencils along l: lane (n,m)
    const bool on_m = live && p < NQ * NV;              // pencils along m: lane (n,i)
    const bool on_n = live && p < NV * NV;              // pencils along n: lane (j,i)

    T *c0 = lds + (size_t)(g < G ? g : 0) * 2 * CUBE;
    T *c1 = c0 + CUBE;

    T xq[NQ], x2[NQ], yv[NV], zv[NV];

    // axis l: lane (n,m) owns the NQ consecutive words [e][n][m][0..NQ-1] of M and P
    if (on_l) {
        const int nn = p / NQ, mm = p - nn * NQ;
        T mq[NQ];
        load_words<(HINT & 1) != 0>(Mq + (size_t)e * QC + (size_t)(p * NQ), mq);
#pragma unroll
        for (int dir = 0; dir < 3; ++dir) {
            const size_t cube = ((size_t)(c * 3 + dir) * (size_t)num_elems + (size_t)e) * QC;
            load_words<(HINT & 1) != 0>(Pq + cube + (size_t)(p * NQ), xq);
#pragma unroll
            for (int l = 0; l < NQ; ++l) xq[l] *= mq[l];
            if (dir == 2) {
#pragma unroll
                for (int l = 0; l < NQ; ++l) x2[l] = xq[l];
            } else {
                mode_product_rect<T, NV, NQ>(dir == 0 ? Dm : Im, xq, yv);
                T *dst = dir == 0 ? c0 : c1;
#pragma unroll
                for (int i = 0; i < NV; ++i) dst[nn * PA + mm * PB + i] = yv[i];
            }
        }
    }
    __syncthreads();

    // axis m, first two terms merged: lane (n,i)
    const int bn = p / NV, bi = p - bn * NV;
    if (on_m) {
#pragma unroll
        for (int m = 0; m < NQ; ++m) xq[m] = c0[bn * PA + m * PB + bi];
        mode_product_rect<T, NV, NQ>(Im, xq, yv);
#pragma unroll
        for (int m = 0; m < NQ; ++m) xq[m] = c1[bn * PA + m * PB + bi];
        mode_product_rect<T, NV, NQ>(Dm, xq, zv);
    }
    __syncthreads();                                    // every pencil of cubes 0 and 1 has been read
    if (on_m) {
#pragma unroll
        for (int j = 0; j < NV; ++j) c0[bn * PA + j * PB + bi] = yv[j] + zv[j];
    }
    // axis l of the third term, into the freed cube 1: lane (n,m)
    if (on_l) {
        const int nn = p / NQ, mm = p - nn * NQ;
        mode_product_rect<T, NV, NQ>(Im, x2, yv);
#pragma unroll
        for (int i = 0; i < NV; ++i) c1[nn * PA + mm * PB + i] = yv[i];
    }
    __syncthreads();
    // axis m of the third term: lane (n,i)
    if (on_m) {
#pragma unroll
        for (int m = 0; m < NQ; ++m) xq[m] = c1[bn * PA + m * PB + bi];
        mode_product_rect<T, NV, NQ>(Im, xq, yv);
#pragma unroll
        for (int j = 0; j < NV; ++j) c1[bn * PA + j * PB + bi] = yv[j];   // the lane's own pencil
    }
    __syncthreads();

    // axis n: lane (j,i); stores are consecutive over lanes
    if (on_n) {
        const int jj = p / NV, ii = p - jj * NV;
#pragma unroll
        for (int n = 0; n < NQ; ++n) xq[n] = c0[n * PA + jj * PB + ii];
        mode_product_rect<T, NV, NQ>(Im, xq, yv);
#pragma unroll
        for (int n = 0; n < NQ; ++n) xq[n] = c1[n * PA + jj * PB + ii];
        mode_product_rect<T, NV, NQ>(Dm, xq, zv);
        const size_t out = ((size_t)c * (size_t)num_elems + (size_t)e) * VC;
#pragma unroll
        for (int k = 0; k < NV; ++k)
            gstore<(HINT & 2) != 0>(F + out + (size_t)(k * NV * NV + p), yv[k] + zv[k]);
    }
}

template <typename T, int NV, int NQ>
constexpr int convection_rect_group()
{
    int best = 1;
    long best_num = 0, best_den = 1;
    for (int g = 1; g <= 64; ++g) {
        const int p = g * ConvRectShape<T, NV, NQ, 1>::L;
        const int nt = ((p + 63) / 64) * 64;
        const long lds = (long)g * (long)ConvRectShape<T, NV, NQ, 1>::LDS_BYTES;
        if (g > 1 && (nt > 512 || lds > 56 * 1024)) break;
        if ((long)p * best_den > best_num * nt) {
            best = g;
            best_num = p;
            best_den = nt;
        }
    }
    return best;
}

template <typename T, int NV, int NQ>
struct ConvectionRectLauncher {
    static constexpr int G = convection_rect_group<T, NV, NQ>();
    using Sh = ConvRectShape<T, NV, NQ, G>;
    static constexpr size_t LDS = Sh::LDS_BYTES;
    static constexpr int HINT = 2;
    static constexpr bool XCD = G % 3 != 0;

    static constexpr auto kernel() { return &convection_rect_kernel<T, NV, NQ, G, HINT, XCD>; }

    static hipError_t launch(const ConvectionArgs &a)
    {
        const long long blocks = convection_grid<XCD>((3 * a.num_elems + G - 1) / G);
        if (blocks <= 0 || blocks > 0x7fffffffLL) return kGridTooLarge;
        drop_stale_error();
        hipLaunchKernelGGL(kernel(), dim3((unsigned)blocks), dim3(Sh::NT), LDS, a.stream,
                           (const T *)a.p, (const T *)a.m, (const T *)a.d_vq, (const T *)a.i_vq,
                           (T *)a.f, a.num_elems);
        return hipGetLastError();
    }

    static hipError_t prepare()
    {
        if (LDS <= 48 * 1024) return hipSuccess;
        return hipFuncSetAttribute((const void *)kernel(),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS);
    }
};

struct ConvectionRectEntry {
    int n_v, n_q;
    ConvectionEntry entry;
};
#define TPO_CONVECTION_RECT_ENTRY(T, NV, NQ)                                              \
    ConvectionRectEntry { NV, NQ, ConvectionEntry { &ConvectionRectLauncher<T, NV, NQ>::launch, \
                                                    &ConvectionRectLauncher<T, NV, NQ>::prepare } }

template <typename T, int N>
struct ConvectionLauncher {
    static constexpr int G = convection_group<T, N>();
    using Sh = PencilShape<T, N, G>;
    static constexpr bool SPLIT = convection_split<T, N>();
    static constexpr size_t LDS = (size_t)(SPLIT ? 2 : 3) * G * Sh::CUBE * sizeof(T);
    // Sweep on MI355X (units per workgroup 1..6 x hints x renumbering; fp64 n = 8, 11, fp32
    // n = 13): non-temporal stores are worth 3 to 8 %, non-temporal loads halve the rate (the
    // per-lane runs share cache lines), more units per workgroup do not pay.
    static constexpr int HINT = 2;
    static constexpr bool XCD = G % 3 != 0;    // with G a multiple of 3 an element stays in one workgroup

    // fp32, n >= 9: the 4x4x1 matrix-core form (the vector-FMA form is bound by FMA issue there,
    // as for the inverse-Helmholtz operator).
    static constexpr bool MM = sizeof(T) == 4 && N >= 9;

    static constexpr auto kernel()
    {
        if constexpr (MM) return &convection_mm_kernel<N, G, HINT, XCD, SPLIT>;
        else return &convection_pencil_kernel<T, N, G, HINT, XCD, SPLIT>;
    }

    static hipError_t launch(const ConvectionArgs &a)
    {
        const long long blocks = convection_grid<XCD>((3 * a.num_elems + G - 1) / G);
        if (blocks <= 0 || blocks > 0x7fffffffLL) return kGridTooLarge;
        drop_stale_error();
        hipLaunchKernelGGL(kernel(), dim3((unsigned)blocks), dim3(Sh::NT), LDS, a.stream,
                           (const T *)a.p, (const T *)a.m, (const T *)a.d_vq, (const T *)a.i_vq,
                           (T *)a.f, a.num_elems);
        return hipGetLastError();
    }

    static hipError_t prepare()
    {
        if (LDS <= 48 * 1024) return hipSuccess;
        return hipFuncSetAttribute((const void *)kernel(),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS);
    }
};

#define TPO_CONVECTION_ENTRY(T, N) \
    ConvectionEntry { &ConvectionLauncher<T, N>::launch, &ConvectionLauncher<T, N>::prepare }

}  // namespace tpo

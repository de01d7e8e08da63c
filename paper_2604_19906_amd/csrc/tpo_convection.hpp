// Volume integral of the convective flux (Eq. 1 of the paper, printed in index form for the
// paper's DSL):
//
//   F[c,e,k,j,i] = sum_l sum_m sum_n (  D[i,l] I[j,m] I[k,n] M[e,n,m,l] P[c,0,e,n,m,l]
//                                     + I[i,l] D[j,m] I[k,n] M[e,n,m,l] P[c,1,e,n,m,l]
//                                     + I[i,l] I[j,m] D[k,n] M[e,n,m,l] P[c,2,e,n,m,l] )
//
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

namespace tpo {

// Units per workgroup: best lane utilisation with at most 512 threads and 48 KB of LDS.
template <typename T, int N>
constexpr int convection_group()
{
    int best = 1;
    long best_num = 0, best_den = 1;
    for (int g = 1; g <= 64; ++g) {
        const int p = g * N * N;
        const int nt = ((p + 63) / 64) * 64;
        const long lds = 3L * g * PencilShape<T, N, 1>::CUBE * (long)sizeof(T);
        if (nt > 512 || lds > 48 * 1024) break;
        if ((long)p * best_den > best_num * nt) {
            best = g;
            best_num = p;
            best_den = nt;
        }
    }
    return best;
}

template <typename T, int N, int G, int HINT>
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
    const long long unit = (long long)blockIdx.x * G + g;
    const bool on = (tid < G * P) && (unit < units);
    const long long e = on ? unit / 3 : 0;
    const int c = on ? (int)(unit - 3 * e) : 0;
    constexpr size_t QC = (size_t)N * N * N;

    T *c0 = lds + (size_t)(g < G ? g : 0) * 3 * CUBE;
    T *c1 = c0 + CUBE;
    T *c2 = c1 + CUBE;

    T x[N], y[N], z[N];

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
            mode_product<T, N, false>(dir == 0 ? Dm : Im, x, y);
            T *dst = dir == 0 ? c0 : (dir == 1 ? c1 : c2);
#pragma unroll
            for (int i = 0; i < N; ++i) dst[hi * PA + lo * PB + i] = y[i];
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

template <typename T, int N>
struct ConvectionLauncher {
    static constexpr int G = convection_group<T, N>();
    using Sh = PencilShape<T, N, G>;
    static constexpr size_t LDS = (size_t)3 * G * Sh::CUBE * sizeof(T);
    static constexpr int HINT = 0;

    static constexpr auto kernel() { return &convection_pencil_kernel<T, N, G, HINT>; }

    static hipError_t launch(const ConvectionArgs &a)
    {
        const long long blocks = (3 * a.num_elems + G - 1) / G;
        if (blocks <= 0 || blocks > 0x7fffffffLL) return hipErrorInvalidValue;
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

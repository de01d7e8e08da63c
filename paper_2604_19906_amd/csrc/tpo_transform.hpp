// One half of the operator on its own: the three-dimensional transform
//   forward   t[i,j,k] = sum_l sum_m sum_q  S_x[l,i] * S_y[m,j] * S_z[q,k] * u[l,m,q]
//   backward  t[i,j,k] = sum_l sum_m sum_q  S_x[i,l] * S_y[j,m] * S_z[k,q] * u[l,m,q]
// evaluated as three one-dimensional mode products (the forward one is the worked example of
// reduction lifting in Sec. 5.2 of the paper).  Same building blocks as the pencil kernels
// (tpo_pencil.hpp): one pencil per lane, matrix entries in SGPRs, the cube re-distributed
// through LDS between axes.  Order: axis 2 first, on the n consecutive words each lane loads
// straight from global memory (lane (a,b)), then axis 1, then axis 0, whose outputs leave as
// coalesced stores (lanes consecutive along (b,c)).  Two barriers.
#pragma once
#include <hip/hip_runtime.h>

#include "tpo_pencil.hpp"

namespace tpo {

template <typename T, int N, int G, int HINT, bool XCD, bool FWD>
__global__ void __launch_bounds__((PencilShape<T, N, G>::NT))
transform_pencil_kernel(const T *u, const T *Sx_, const T *Sy_, const T *Sz_, T *t,
                        long long num_elems)
{
    using Sh = PencilShape<T, N, G>;
    constexpr int P = Sh::P, PA = Sh::PA, PB = Sh::PB, CUBE = Sh::CUBE;
    extern __shared__ __align__(16) unsigned char tpo_lds[];
    T *cube_all = reinterpret_cast<T *>(tpo_lds);

    const TPO_CONSTANT T *Sx = (const TPO_CONSTANT T *)Sx_;
    const TPO_CONSTANT T *Sy = (const TPO_CONSTANT T *)Sy_;
    const TPO_CONSTANT T *Sz = (const TPO_CONSTANT T *)Sz_;

    const int tid = threadIdx.x;
    const int g = tid / P;
    const int p = tid - g * P;
    const int hi = p / N;
    const int lo = p - hi * N;
    const long long nbatch = (num_elems + G - 1) / G;
    const long long batch = pencil_batch<XCD>(nbatch);
    if (XCD && batch >= nbatch) return;                 // whole workgroup: no barrier is skipped
    const long long e = batch * G + g;
    const bool on = (tid < G * P) && (e < num_elems);
    T *cube = cube_all + (g < G ? g : 0) * CUBE;
    const size_t base = (size_t)(on ? e : 0) * (size_t)(N * N * N);

    T x[N], y[N];

    // axis 2: lane (a,b) = (hi,lo) owns u[a][b][0..n-1], contiguous in memory
    if (on) {
        load_words<(HINT & 1) != 0>(u + base + (size_t)(p * N), x);
        mode_product<T, N, FWD>(Sz, x, y);
#pragma unroll
        for (int k = 0; k < N; ++k) cube[hi * PA + lo * PB + k] = y[k];
    }
    __syncthreads();

    // axis 1: lane (a,c) = (hi,lo)
    if (on) {
#pragma unroll
        for (int m = 0; m < N; ++m) x[m] = cube[hi * PA + m * PB + lo];
        mode_product<T, N, FWD>(Sy, x, y);
#pragma unroll
        for (int j = 0; j < N; ++j) cube[hi * PA + j * PB + lo] = y[j];
    }
    __syncthreads();

    // axis 0: lane (b,c) = (hi,lo); stores are consecutive over lanes
    if (on) {
#pragma unroll
        for (int l = 0; l < N; ++l) x[l] = cube[l * PA + hi * PB + lo];
        mode_product<T, N, FWD>(Sx, x, y);
#pragma unroll
        for (int i = 0; i < N; ++i) gstore<(HINT & 2) != 0>(t + base + (size_t)(i * P + p), y[i]);
    }
}

// Elements per workgroup and die renumbering as for the separable-diagonal operator kernels
// (same traffic: one field in, one out); cached loads, since each lane's n-word run shares its
// cache lines with its neighbours' runs.
template <typename T, int N, bool FWD>
struct TransformLauncher {
    using Tune = PencilSepTune<T, N>;
    static constexpr int G = Tune::G;
    using Sh = PencilShape<T, N, G>;
    static constexpr size_t LDS = Sh::LDS_BYTES / 2;
    static constexpr int HINT = Tune::HINT & 2;

    static constexpr auto kernel() { return &transform_pencil_kernel<T, N, G, HINT, Tune::XCD, FWD>; }

    static hipError_t launch(const TransformArgs &a)
    {
        const long long blocks = pencil_grid<Tune::XCD>((a.num_elems + G - 1) / G);
        if (blocks <= 0 || blocks > 0x7fffffffLL) return kGridTooLarge;
        drop_stale_error();
        hipLaunchKernelGGL(kernel(), dim3((unsigned)blocks), dim3(Sh::NT), LDS, a.stream,
                           (const T *)a.u, (const T *)a.sx, (const T *)a.sy, (const T *)a.sz,
                           (T *)a.t, a.num_elems);
        return hipGetLastError();
    }

    static hipError_t prepare()
    {
        if (LDS <= 48 * 1024) return hipSuccess;
        return hipFuncSetAttribute((const void *)kernel(),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS);
    }
};

#define TPO_TRANSFORM_ENTRY(T, N)                                                          \
    TransformEntry { &TransformLauncher<T, N, true>::launch, &TransformLauncher<T, N, false>::launch, \
                     &TransformLauncher<T, N, true>::prepare, &TransformLauncher<T, N, false>::prepare }

}  // namespace tpo

// Kernel of the inverse-Helmholtz operator for anisotropic elements: nx, ny, nz points along
// axes 0, 1, 2, all runtime values in 1 .. 16.  It stands behind tpo_ihelm_apply_aniso for the
// shapes that are not cubic (cubic shapes go to the tuned families).
//
// Same scheme as the pencil kernels: a workgroup takes g whole elements, the cube lives in LDS,
// every lane owns one pencil per mode product, the matrix entries arrive in SGPRs.  What makes
// it work for runtime sizes is that a mode product only needs the size of ITS axis at compile
// time (for the unrolled FMAs and the batched scalar loads of the matrix); the other two sizes
// only enter pencil counts and strides, which may be runtime values.  So every product is a
// uniform switch over the size of its axis, and the kernel is compiled once per size class
// (largest of the three sizes at most 4, 8, 12 or 16: the class bounds the registers).
//
// Order of the products, as in the pencil kernels: axis 0 first, on words read coalesced from
// u_e (for a fixed index along axis 0 the lanes of that pass are consecutive words), axis 1,
// then axis 2 forward, the scale and axis 2 backward on the lane's registers (each lane asked
// for the nz consecutive words of D_e it needs when the kernel started), axis 1, and axis 0
// last, stored coalesced to v_e.  Four barriers, no index arithmetic per word.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "tpo_internal.h"
#include "tpo_pencil.hpp"

namespace tpo {

namespace {

constexpr int ANISO_MAX_NT = 256;
// Non-temporal stores of v_e, workgroups renumbered per die: the best or within 2 % of the best
// of a sweep over eight shapes on MI355X (hint bits x renumbering x elements per workgroup x LDS
// floor).  Non-temporal loads of u_e as well measured the same rate on average with 5 % more
// HBM reads (the 32-byte pieces two rows of a pass share are then fetched twice).
constexpr int ANISO_HINT = 2;
constexpr bool ANISO_XCD = true;

// f(integral_constant<int, n>) for the runtime n in 1 .. MAXN (uniform over the workgroup).
template <int MAXN, typename F>
__device__ __forceinline__ void dispatch_size(int n, F &&f)
{
#define TPO_SIZE_CASE(K)                                                       \
    case K:                                                                    \
        if constexpr (K <= MAXN) f(std::integral_constant<int, K>{});          \
        break;
    switch (n) {
        TPO_SIZE_CASE(1) TPO_SIZE_CASE(2) TPO_SIZE_CASE(3) TPO_SIZE_CASE(4)
        TPO_SIZE_CASE(5) TPO_SIZE_CASE(6) TPO_SIZE_CASE(7) TPO_SIZE_CASE(8)
        TPO_SIZE_CASE(9) TPO_SIZE_CASE(10) TPO_SIZE_CASE(11) TPO_SIZE_CASE(12)
        TPO_SIZE_CASE(13) TPO_SIZE_CASE(14) TPO_SIZE_CASE(15) TPO_SIZE_CASE(16)
    default: break;
    }
#undef TPO_SIZE_CASE
}

// LDS pitches: odd row pitch and odd plane pitch (in words) against bank conflicts.
__host__ __device__ inline int aniso_pz(int nz) { return nz | 1; }
__host__ __device__ inline int aniso_pyz(int ny, int nz) { return (ny * aniso_pz(nz)) | 1; }

// HINT bits as in the pencil kernels: 1 non-temporal loads of u_e, 2 non-temporal stores of v_e,
// 4 non-temporal loads of D_e.  XCD: workgroups renumbered per accelerator die (the grid must be
// pencil_grid<XCD>(number of groups)).
template <typename T, int MAXN, int HINT, bool XCD>
__global__ void __launch_bounds__(ANISO_MAX_NT)
ihelm_aniso_kernel(const T *u, const T *Sx_, const T *Sy_, const T *Sz_, const T *__restrict__ D,
                   T *v, int nx, int ny, int nz, int g, long long num_elems, long long groups)
{
    extern __shared__ __align__(16) unsigned char tpo_lds[];
    T *cube = reinterpret_cast<T *>(tpo_lds);
    const TPO_CONSTANT T *Sx = (const TPO_CONSTANT T *)Sx_;
    const TPO_CONSTANT T *Sy = (const TPO_CONSTANT T *)Sy_;
    const TPO_CONSTANT T *Sz = (const TPO_CONSTANT T *)Sz_;

    const int tid = threadIdx.x;
    const long long batch = pencil_batch<XCD>(groups);
    if (batch >= groups) return;                           // padding workgroup of the renumbering
    const long long e0 = batch * g;
    const long long left = num_elems - e0;
    const int here = left < g ? (int)left : g;             // elements of this workgroup
    const int pz = aniso_pz(nz), pyz = aniso_pyz(ny, nz);
    const int cube_words = nx * pyz;
    const int face = ny * nz;
    const size_t total = (size_t)nx * face;

    // the lane's place in a pass with `pencils` pencils per element: element ge, pencil p
    auto place = [&](int pencils, int &ge, int &p) {
        ge = tid / pencils;
        p = tid - ge * pencils;
        return ge < here;
    };

    int ge2, p2;
    const bool act2 = place(nx * ny, ge2, p2);              // lane (a, b): a pencil along axis 2
    const int a2 = p2 / ny, b2 = p2 - a2 * ny;
    T *row2 = cube + ge2 * cube_words + a2 * pyz + b2 * pz;

    // D_e in the layout of the axis-2 pass, asked for before anything else
    T dreg[MAXN];
    if (act2)
        dispatch_size<MAXN>(nz, [&](auto nc) {
            constexpr int N = decltype(nc)::value;
            T t[N];
            load_words<(HINT & 4) != 0, T, N>(D + (size_t)(e0 + ge2) * total + (size_t)p2 * nz, t);
#pragma unroll
            for (int k = 0; k < N; ++k) dreg[k] = t[k];
        });

    int ge1, p1;
    const bool act1 = place(nx * nz, ge1, p1);              // lane (a, c): a pencil along axis 1
    const int a1 = p1 / nz, c1 = p1 - a1 * nz;
    T *col1 = cube + ge1 * cube_words + a1 * pyz + c1;

    int ge0, p0;
    const bool act0 = place(face, ge0, p0);                 // lane (b, c): a pencil along axis 0
    const int b0 = p0 / nz, c0 = p0 - b0 * nz;
    T *col0 = cube + ge0 * cube_words + b0 * pz + c0;
    const size_t base0 = (size_t)(e0 + ge0) * total + p0;

    // forward, axis 0, from global memory
    if (act0)
        dispatch_size<MAXN>(nx, [&](auto nc) {
            constexpr int N = decltype(nc)::value;
            T x[N], y[N];
#pragma unroll
            for (int l = 0; l < N; ++l) x[l] = gload<(HINT & 1) != 0>(u + base0 + (size_t)l * face);
            mode_product<T, N, true>(Sx, x, y);
#pragma unroll
            for (int i = 0; i < N; ++i) col0[i * pyz] = y[i];
        });
    __syncthreads();
    // forward, axis 1, in place
    if (act1)
        dispatch_size<MAXN>(ny, [&](auto nc) {
            constexpr int N = decltype(nc)::value;
            T x[N], y[N];
#pragma unroll
            for (int m = 0; m < N; ++m) x[m] = col1[m * pz];
            mode_product<T, N, true>(Sy, x, y);
#pragma unroll
            for (int m = 0; m < N; ++m) col1[m * pz] = y[m];
        });
    __syncthreads();
    // axis 2: forward, scale by D_e, backward, in place
    if (act2)
        dispatch_size<MAXN>(nz, [&](auto nc) {
            constexpr int N = decltype(nc)::value;
            T x[N], y[N];
#pragma unroll
            for (int k = 0; k < N; ++k) x[k] = row2[k];
            mode_product<T, N, true>(Sz, x, y);
#pragma unroll
            for (int k = 0; k < N; ++k) y[k] *= dreg[k];
            mode_product<T, N, false>(Sz, y, x);
#pragma unroll
            for (int k = 0; k < N; ++k) row2[k] = x[k];
        });
    __syncthreads();
    // backward, axis 1, in place
    if (act1)
        dispatch_size<MAXN>(ny, [&](auto nc) {
            constexpr int N = decltype(nc)::value;
            T x[N], y[N];
#pragma unroll
            for (int m = 0; m < N; ++m) x[m] = col1[m * pz];
            mode_product<T, N, false>(Sy, x, y);
#pragma unroll
            for (int m = 0; m < N; ++m) col1[m * pz] = y[m];
        });
    __syncthreads();
    // backward, axis 0, to global memory
    if (act0)
        dispatch_size<MAXN>(nx, [&](auto nc) {
            constexpr int N = decltype(nc)::value;
            T x[N], y[N];
#pragma unroll
            for (int l = 0; l < N; ++l) x[l] = col0[l * pyz];
            mode_product<T, N, false>(Sx, x, y);
#pragma unroll
            for (int i = 0; i < N; ++i) gstore<(HINT & 2) != 0>(v + base0 + (size_t)i * face, y[i]);
        });
}

// Elements per workgroup: the g with the best lane utilisation in the pass with the most
// pencils, among those with at most 256 lanes and at most 40 KB of LDS.
template <typename T>
void aniso_shape(const AnisoArgs &a, int &g, int &nt, size_t &lds)
{
    int maxp = a.ny * a.nz;
    if (a.nx * a.nz > maxp) maxp = a.nx * a.nz;
    if (a.nx * a.ny > maxp) maxp = a.nx * a.ny;
    const size_t cube_bytes = (size_t)a.nx * aniso_pyz(a.ny, a.nz) * sizeof(T);
    g = 1;
    long best_num = 0, best_den = 1;
    for (int c = 1; c <= 256; ++c) {
        const int lanes = c * maxp;
        const int rounded = ((lanes + 63) / 64) * 64;
        if (rounded > ANISO_MAX_NT || c * cube_bytes > 40 * 1024) break;
        if ((long)lanes * best_den >= best_num * rounded) {   // ties: the larger workgroup
            g = c;
            best_num = lanes;
            best_den = rounded;
        }
    }
    nt = ((g * maxp + 63) / 64) * 64;                              // at most 256
    lds = g * cube_bytes;                                          // at most 40 KB (34 KB for g = 1)
}

template <typename T, int MAXN>
hipError_t launch_bound(const AnisoArgs &a)
{
    int g, nt;
    size_t lds;
    aniso_shape<T>(a, g, nt, lds);
    const long long groups = (a.num_elems + g - 1) / g;
    drop_stale_error();
    hipLaunchKernelGGL((ihelm_aniso_kernel<T, MAXN, ANISO_HINT, ANISO_XCD>),
                       dim3((unsigned)pencil_grid<ANISO_XCD>(groups)), dim3(nt), lds, a.stream,
                       (const T *)a.u, (const T *)a.sx, (const T *)a.sy, (const T *)a.sz,
                       (const T *)a.d, (T *)a.v, a.nx, a.ny, a.nz, g, a.num_elems, groups);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_generic(const AnisoArgs &a)
{
    if (a.num_elems <= 0 || a.num_elems > 0x7fffffffLL) return kGridTooLarge;
    int n = a.nx > a.ny ? a.nx : a.ny;
    if (a.nz > n) n = a.nz;
    if (n <= 4) return launch_bound<T, 4>(a);
    if (n <= 8) return launch_bound<T, 8>(a);
    if (n <= 12) return launch_bound<T, 12>(a);
    return launch_bound<T, 16>(a);
}

}  // namespace

hipError_t launch_ihelm_generic(const AnisoArgs &a, int dtype)
{
    return dtype == TPO_F64 ? launch_generic<double>(a) : launch_generic<float>(a);
}

}  // namespace tpo

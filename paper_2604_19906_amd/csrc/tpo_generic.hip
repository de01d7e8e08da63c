// Generic kernel of the inverse-Helmholtz operator for anisotropic elements: nx, ny, nz points
// along axes 0, 1, 2, all runtime values in 1 .. 16.  The fallback behind
// tpo_ihelm_apply_aniso for shapes that have no tuned instantiation (cubic shapes go to the
// tuned families).  Same scheme as the pencil kernels, with runtime sizes: one workgroup of 256
// lanes at most per element (the largest pencil count of the three axes, rounded up to whole
// wavefronts), the cube in LDS, one pencil per lane for each mode product, matrix entries
// through the scalar data path (their addresses are uniform), loops unrolled to a compile-time
// bound (4, 8, 12 or 16, the smallest that covers the three sizes) with uniform guards so that
// the pencil stays in registers.
#include <hip/hip_runtime.h>

#include "tpo_internal.h"

namespace tpo {

#define TPO_CONSTANT_G __attribute__((address_space(4)))

namespace {

constexpr int MAX_NT = 256;

__device__ __forceinline__ double gfma(double a, double b, double c) { return __builtin_fma(a, b, c); }
__device__ __forceinline__ float gfma(float a, float b, float c) { return __builtin_fmaf(a, b, c); }

// y[i] = sum_l M(i,l) x[l], i, l < n;  M(i,l) = S[l*n+i] when transposed, else S[i*n+l].
template <typename T, int MAXN>
__device__ __forceinline__ void product_rt(const TPO_CONSTANT_G T *S, bool transposed, int n,
                                           const T (&x)[MAXN], T (&y)[MAXN])
{
#pragma unroll
    for (int i = 0; i < MAXN; ++i) {
        T acc = T(0);
        if (i < n) {
#pragma unroll
            for (int l = 0; l < MAXN; ++l)
                if (l < n) acc = gfma(transposed ? S[l * n + i] : S[i * n + l], x[l], acc);
        }
        y[i] = acc;
    }
}

template <typename T, int MAXN>
__global__ void __launch_bounds__(MAX_NT)
ihelm_generic_kernel(const T *u, const T *Sx_, const T *Sy_, const T *Sz_, const T *__restrict__ D,
                     T *v, int nx, int ny, int nz, long long num_elems)
{
    extern __shared__ __align__(16) unsigned char tpo_lds[];
    T *cube = reinterpret_cast<T *>(tpo_lds);
    const TPO_CONSTANT_G T *Sx = (const TPO_CONSTANT_G T *)Sx_;
    const TPO_CONSTANT_G T *Sy = (const TPO_CONSTANT_G T *)Sy_;
    const TPO_CONSTANT_G T *Sz = (const TPO_CONSTANT_G T *)Sz_;

    const int tid = threadIdx.x;
    const int NT = blockDim.x;
    const long long e = blockIdx.x;
    if (e >= num_elems) return;
    const int total = nx * ny * nz;
    const size_t base = (size_t)e * (size_t)total;

    for (int i = tid; i < total; i += NT) cube[i] = u[base + i];
    __syncthreads();

    T x[MAXN], y[MAXN];
    // one mode product along `axis` on the cube in LDS, in place (a lane rewrites its own pencil)
    auto along = [&](int axis, const TPO_CONSTANT_G T *S, bool transposed) {
        const int n = axis == 0 ? nx : (axis == 1 ? ny : nz);
        const int pencils = total / n;
        if (tid < pencils) {
            int start, stride;
            if (axis == 0) { start = tid; stride = ny * nz; }
            else if (axis == 1) { const int a = tid / nz; start = a * ny * nz + (tid - a * nz); stride = nz; }
            else { start = tid * nz; stride = 1; }
#pragma unroll
            for (int l = 0; l < MAXN; ++l) x[l] = l < n ? cube[start + l * stride] : T(0);
            product_rt<T, MAXN>(S, transposed, n, x, y);
#pragma unroll
            for (int i = 0; i < MAXN; ++i)
                if (i < n) cube[start + i * stride] = y[i];
        }
        __syncthreads();
    };

    along(0, Sx, true);
    along(1, Sy, true);
    // axis 2: forward, scale by D_e (each lane reads the nz consecutive words of its pencil),
    // backward, all on the lane's registers
    {
        const int pencils = nx * ny;
        if (tid < pencils) {
            const int start = tid * nz;
#pragma unroll
            for (int l = 0; l < MAXN; ++l) x[l] = l < nz ? cube[start + l] : T(0);
            product_rt<T, MAXN>(Sz, true, nz, x, y);
#pragma unroll
            for (int k = 0; k < MAXN; ++k) x[k] = k < nz ? y[k] * D[base + start + k] : T(0);
            product_rt<T, MAXN>(Sz, false, nz, x, y);
#pragma unroll
            for (int k = 0; k < MAXN; ++k)
                if (k < nz) cube[start + k] = y[k];
        }
        __syncthreads();
    }
    along(1, Sy, false);
    along(0, Sx, false);

    for (int i = tid; i < total; i += NT) v[base + i] = cube[i];
}

template <typename T, int MAXN>
hipError_t launch_bound(const AnisoArgs &a)
{
    const size_t lds = (size_t)a.nx * a.ny * a.nz * sizeof(T);     // at most 32 KB
    int pencils = a.ny * a.nz;
    if (a.nx * a.nz > pencils) pencils = a.nx * a.nz;
    if (a.nx * a.ny > pencils) pencils = a.nx * a.ny;
    const int nt = ((pencils + 63) / 64) * 64;                     // at most 256
    hipLaunchKernelGGL((ihelm_generic_kernel<T, MAXN>), dim3((unsigned)a.num_elems), dim3(nt), lds,
                       a.stream, (const T *)a.u, (const T *)a.sx, (const T *)a.sy,
                       (const T *)a.sz, (const T *)a.d, (T *)a.v, a.nx, a.ny, a.nz, a.num_elems);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_generic(const AnisoArgs &a)
{
    if (a.num_elems <= 0 || a.num_elems > 0x7fffffffLL) return hipErrorInvalidValue;
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

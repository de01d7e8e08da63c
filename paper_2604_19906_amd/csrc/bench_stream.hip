// Measurement aid (libtpo_bench.so, not the operator library): the plain streaming kernel v[i] = u[i] * D[i] over flat arrays.  It moves
// exactly the operator's algorithmic traffic (two reads, one write per word) with no other
// work, so its time is the streaming ceiling the operator is compared with, and the HBM
// counters it reads calibrate those read for the operator's kernels.
#include <hip/hip_runtime.h>

#include <cstdint>

#include "tpo_bench.h"
#include "tpo_internal.h"

namespace {

// One 16-byte access per lane and array, non-temporal, one wavefront per workgroup: the launch
// shape that measured fastest for a plain stream on MI355X (64 lanes 6675 GB/s, 256 lanes
// 6471, 512 lanes 6076 on 2 GiB fields).
constexpr int kStreamLanes = 64;

template <typename V>
__global__ void __launch_bounds__(kStreamLanes)
stream_scale_kernel(const V *__restrict__ u, const V *__restrict__ d, V *__restrict__ v,
                    size_t nvec)
{
    const size_t i = (size_t)blockIdx.x * kStreamLanes + threadIdx.x;
    if (i < nvec) {
        const V a = __builtin_nontemporal_load(u + i);
        const V b = __builtin_nontemporal_load(d + i);
        __builtin_nontemporal_store(a * b, v + i);
    }
}

typedef double double2_ __attribute__((ext_vector_type(2)));
typedef float float4_ __attribute__((ext_vector_type(4)));

template <typename T, typename V>
hipError_t launch(const void *u, const void *d, void *v, long long count, hipStream_t s)
{
    constexpr int W = sizeof(V) / sizeof(T);
    const size_t nvec = (size_t)count / W;
    const size_t tail = (size_t)count - nvec * W;
    if (nvec) {
        const size_t blocks = (nvec + kStreamLanes - 1) / kStreamLanes;
        if (blocks > 0x7fffffffULL) return tpo::kGridTooLarge;
        tpo::drop_stale_error();
        hipLaunchKernelGGL(stream_scale_kernel<V>, dim3((unsigned)blocks), dim3(kStreamLanes), 0, s,
                           (const V *)u, (const V *)d, (V *)v, nvec);
    }
    if (tail) {
        tpo::drop_stale_error();
        hipLaunchKernelGGL(stream_scale_kernel<T>, dim3(1), dim3(kStreamLanes), 0, s,
                           (const T *)u + nvec * W, (const T *)d + nvec * W,
                           (T *)v + nvec * W, tail);
    }
    return hipGetLastError();
}

}  // namespace

extern "C" int tpo_stream_scale(const void *u, const void *D, void *v, long long count,
                                int dtype, void *stream)
{
    if (dtype != TPO_F64 && dtype != TPO_F32) return TPO_ERR_INVALID_ARG;
    if (count < 0) return TPO_ERR_INVALID_ARG;
    if (count == 0) return TPO_OK;
    if (!u || !D || !v) return TPO_ERR_INVALID_ARG;
    // 16-byte vectors need 16-byte aligned arrays
    if (((uintptr_t)u | (uintptr_t)D | (uintptr_t)v) % 16) return TPO_ERR_INVALID_ARG;
    const hipError_t e = (dtype == TPO_F64)
                             ? launch<double, double2_>(u, D, v, count, (hipStream_t)stream)
                             : launch<float, float4_>(u, D, v, count, (hipStream_t)stream);
    if (e != hipSuccess) {
        (void)hipGetLastError();
        return e == tpo::kGridTooLarge ? TPO_ERR_UNSUPPORTED : TPO_ERR_DEVICE;
    }
    return TPO_OK;
}

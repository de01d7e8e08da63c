// Internal interfaces of libtpo (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>

#include "tpo.h"

namespace tpo {

// Returned by a launcher whose grid would pass the 2^31-1 workgroups of a HIP launch; the entry
// points report it as TPO_ERR_UNSUPPORTED (the arguments are valid, the batch is too large
// for one launch).
constexpr hipError_t kGridTooLarge = hipErrorInvalidConfiguration;

// Called right before a kernel launch: drops an error that an earlier runtime call of this
// thread (the caller's, e.g. an event query that returned "not ready") left recorded, so that
// the hipGetLastError() after the launch reports this launch only.
inline void drop_stale_error() { (void)hipGetLastError(); }

struct ApplyArgs {
    const void *u, *sx, *sy, *sz, *d;
    void *v;
    long long num_elems;
    hipStream_t stream;
    // separable diagonal (tpo_ihelm_apply_sep): d is null and these are set
    const void *lam_x = nullptr, *lam_y = nullptr, *lam_z = nullptr, *mu = nullptr;
};

// One kernel instantiation for a fixed (n, dtype): how to launch it and how to prepare it
// once per device (e.g. raise its dynamic-LDS limit).
struct KernelEntry {
    hipError_t (*launch)(const ApplyArgs &);
    hipError_t (*launch_sep)(const ApplyArgs &);   // null: no separable-diagonal form
    hipError_t (*prepare)();
};

// The transform halves on their own (tpo_transform_apply).
struct TransformArgs {
    const void *u, *sx, *sy, *sz;
    void *t;
    long long num_elems;
    hipStream_t stream;
};
struct TransformEntry {
    hipError_t (*launch_forward)(const TransformArgs &);
    hipError_t (*launch_backward)(const TransformArgs &);
    hipError_t (*prepare_forward)();
    hipError_t (*prepare_backward)();
};
const TransformEntry *transform_entry(int n, int dtype);

// The convection volume term (tpo_convection_apply).
struct ConvectionArgs {
    const void *p, *m, *d_vq, *i_vq;
    void *f;
    long long num_elems;
    hipStream_t stream;
};
struct ConvectionEntry {
    hipError_t (*launch)(const ConvectionArgs &);
    hipError_t (*prepare)();
};
// n_v == n_q: every n in 1..TPO_MAX_N; n_v != n_q: the instantiated over-integration shapes.
const ConvectionEntry *convection_entry(int n_v, int n_q, int dtype);
int convection_rect_count(int dtype);
const ConvectionEntry *convection_rect_at(int k, int dtype);

// Anisotropic elements (tpo_ihelm_apply_aniso): the generic runtime-size kernel.
struct AnisoArgs {
    const void *u, *sx, *sy, *sz, *d;
    void *v;
    int nx, ny, nz;
    long long num_elems;
    hipStream_t stream;
};
hipError_t launch_ihelm_generic(const AnisoArgs &a, int dtype);

// dtype index: 0 = f64, 1 = f32.  n in 1..TPO_MAX_N.  Returns nullptr when the family has
// no kernel for that shape.
const KernelEntry *pencil_entry(int n, int dtype);
const KernelEntry *mfma_entry(int n, int dtype);
const KernelEntry *pencil_mm_entry(int n, int dtype);   // fp32 only

// Pure host validation shared by the entry points; touches no HIP state.
int validate_apply(const void *u, const void *sx, const void *sy, const void *sz,
                   const void *d, const void *v, int n, long long num_elems, int dtype,
                   int variant);
int validate_convection(const void *p, const void *m, const void *d_vq, const void *i_vq,
                        const void *f, int n_v, int n_q, long long num_elems, int dtype,
                        bool has_kernel);   // has_kernel: a kernel exists for (n_v, n_q, dtype)
int validate_apply_aniso(const void *u, const void *sx, const void *sy, const void *sz,
                         const void *d, const void *v, int nx, int ny, int nz, long long num_elems,
                         int dtype);
int validate_transform(const void *u, const void *sx, const void *sy, const void *sz,
                       const void *t, int n, long long num_elems, int dtype, int direction);
int validate_apply_sep(const void *u, const void *sx, const void *sy, const void *sz,
                       const void *lam_x, const void *lam_y, const void *lam_z, const void *mu,
                       const void *v, int n, long long num_elems, int dtype, int variant);

}  // namespace tpo

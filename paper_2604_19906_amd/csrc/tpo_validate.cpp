// Host-only argument validation for the C ABI (no HIP call is made here, so it runs on a
// machine without a GPU).
#include <cstddef>
#include <cstdint>

#include "tpo.h"

namespace tpo {

static bool overlaps(const void *a, size_t abytes, const void *b, size_t bbytes)
{
    const uintptr_t a0 = (uintptr_t)a, a1 = a0 + abytes;
    const uintptr_t b0 = (uintptr_t)b, b1 = b0 + bbytes;
    return a0 < b1 && b0 < a1;
}

int validate_apply(const void *u, const void *sx, const void *sy, const void *sz,
                   const void *d, const void *v, int n, long long num_elems, int dtype,
                   int variant)
{
    if (dtype != TPO_F64 && dtype != TPO_F32) return TPO_ERR_INVALID_ARG;
    if (variant != TPO_VARIANT_AUTO && variant != TPO_VARIANT_PENCIL &&
        variant != TPO_VARIANT_MFMA && variant != TPO_VARIANT_PENCIL_MM)
        return TPO_ERR_INVALID_ARG;
    if (n < 1 || num_elems < 0) return TPO_ERR_INVALID_ARG;
    if (n > TPO_MAX_N) return TPO_ERR_UNSUPPORTED;
    if (num_elems == 0) return TPO_OK;
    if (!u || !sx || !sy || !sz || !d || !v) return TPO_ERR_INVALID_ARG;
    const size_t w = (dtype == TPO_F64) ? 8 : 4;
    const void *ptrs[6] = {u, sx, sy, sz, d, v};
    for (const void *p : ptrs)
        if ((uintptr_t)p % w) return TPO_ERR_INVALID_ARG;
    // E * n^3 * w must fit in size_t with room to spare (n <= 16, so n^3*w <= 32768)
    if ((unsigned long long)num_elems > (~(size_t)0 >> 16)) return TPO_ERR_INVALID_ARG;
    const size_t field = (size_t)num_elems * n * n * n * w;
    const size_t mat = (size_t)n * n * w;
    if (v != u && overlaps(v, field, u, field)) return TPO_ERR_ALIAS;
    if (overlaps(v, field, d, field)) return TPO_ERR_ALIAS;
    if (overlaps(v, field, sx, mat) || overlaps(v, field, sy, mat) ||
        overlaps(v, field, sz, mat))
        return TPO_ERR_ALIAS;
    return TPO_OK;
}

int validate_convection(const void *p, const void *m, const void *d_vq, const void *i_vq,
                        const void *f, int n_v, int n_q, long long num_elems, int dtype,
                        bool has_kernel)
{
    if (dtype != TPO_F64 && dtype != TPO_F32) return TPO_ERR_INVALID_ARG;
    if (n_v < 1 || n_q < 1 || num_elems < 0) return TPO_ERR_INVALID_ARG;
    if (n_v > TPO_MAX_N || n_q > TPO_MAX_N || !has_kernel) return TPO_ERR_UNSUPPORTED;
    if (num_elems == 0) return TPO_OK;
    if (!p || !m || !d_vq || !i_vq || !f) return TPO_ERR_INVALID_ARG;
    const size_t w = (dtype == TPO_F64) ? 8 : 4;
    const void *ptrs[5] = {p, m, d_vq, i_vq, f};
    for (const void *q : ptrs)
        if ((uintptr_t)q % w) return TPO_ERR_INVALID_ARG;
    if ((unsigned long long)num_elems > (~(size_t)0 >> 20)) return TPO_ERR_INVALID_ARG;
    const size_t qcube = (size_t)num_elems * n_q * n_q * n_q * w;
    const size_t vcube = (size_t)num_elems * n_v * n_v * n_v * w;
    const size_t mat = (size_t)n_v * n_q * w;
    if (overlaps(f, 3 * vcube, p, 9 * qcube) || overlaps(f, 3 * vcube, m, qcube) ||
        overlaps(f, 3 * vcube, d_vq, mat) || overlaps(f, 3 * vcube, i_vq, mat))
        return TPO_ERR_ALIAS;
    return TPO_OK;
}

int validate_apply_aniso(const void *u, const void *sx, const void *sy, const void *sz,
                         const void *d, const void *v, int nx, int ny, int nz, long long num_elems,
                         int dtype)
{
    if (dtype != TPO_F64 && dtype != TPO_F32) return TPO_ERR_INVALID_ARG;
    if (nx < 1 || ny < 1 || nz < 1 || num_elems < 0) return TPO_ERR_INVALID_ARG;
    if (nx > TPO_MAX_N || ny > TPO_MAX_N || nz > TPO_MAX_N) return TPO_ERR_UNSUPPORTED;
    if (num_elems == 0) return TPO_OK;
    if (!u || !sx || !sy || !sz || !d || !v) return TPO_ERR_INVALID_ARG;
    const size_t w = (dtype == TPO_F64) ? 8 : 4;
    const void *ptrs[6] = {u, sx, sy, sz, d, v};
    for (const void *p : ptrs)
        if ((uintptr_t)p % w) return TPO_ERR_INVALID_ARG;
    if ((unsigned long long)num_elems > (~(size_t)0 >> 16)) return TPO_ERR_INVALID_ARG;
    const size_t field = (size_t)num_elems * nx * ny * nz * w;
    if (v != u && overlaps(v, field, u, field)) return TPO_ERR_ALIAS;
    if (overlaps(v, field, d, field)) return TPO_ERR_ALIAS;
    if (overlaps(v, field, sx, (size_t)nx * nx * w) || overlaps(v, field, sy, (size_t)ny * ny * w) ||
        overlaps(v, field, sz, (size_t)nz * nz * w))
        return TPO_ERR_ALIAS;
    return TPO_OK;
}

int validate_transform(const void *u, const void *sx, const void *sy, const void *sz,
                       const void *t, int n, long long num_elems, int dtype, int direction)
{
    if (dtype != TPO_F64 && dtype != TPO_F32) return TPO_ERR_INVALID_ARG;
    if (direction != TPO_FORWARD && direction != TPO_BACKWARD) return TPO_ERR_INVALID_ARG;
    if (n < 1 || num_elems < 0) return TPO_ERR_INVALID_ARG;
    if (n > TPO_MAX_N) return TPO_ERR_UNSUPPORTED;
    if (num_elems == 0) return TPO_OK;
    if (!u || !sx || !sy || !sz || !t) return TPO_ERR_INVALID_ARG;
    const size_t w = (dtype == TPO_F64) ? 8 : 4;
    const void *ptrs[5] = {u, sx, sy, sz, t};
    for (const void *p : ptrs)
        if ((uintptr_t)p % w) return TPO_ERR_INVALID_ARG;
    if ((unsigned long long)num_elems > (~(size_t)0 >> 16)) return TPO_ERR_INVALID_ARG;
    const size_t field = (size_t)num_elems * n * n * n * w;
    const size_t mat = (size_t)n * n * w;
    if (t != u && overlaps(t, field, u, field)) return TPO_ERR_ALIAS;
    if (overlaps(t, field, sx, mat) || overlaps(t, field, sy, mat) ||
        overlaps(t, field, sz, mat))
        return TPO_ERR_ALIAS;
    return TPO_OK;
}

int validate_apply_sep(const void *u, const void *sx, const void *sy, const void *sz,
                       const void *lam_x, const void *lam_y, const void *lam_z, const void *mu,
                       const void *v, int n, long long num_elems, int dtype, int variant)
{
    if (dtype != TPO_F64 && dtype != TPO_F32) return TPO_ERR_INVALID_ARG;
    if (variant != TPO_VARIANT_AUTO && variant != TPO_VARIANT_PENCIL &&
        variant != TPO_VARIANT_MFMA && variant != TPO_VARIANT_PENCIL_MM)
        return TPO_ERR_INVALID_ARG;
    if (n < 1 || num_elems < 0) return TPO_ERR_INVALID_ARG;
    if (n > TPO_MAX_N) return TPO_ERR_UNSUPPORTED;
    if (num_elems == 0) return TPO_OK;
    if (!u || !sx || !sy || !sz || !lam_x || !lam_y || !lam_z || !mu || !v)
        return TPO_ERR_INVALID_ARG;
    const size_t w = (dtype == TPO_F64) ? 8 : 4;
    const void *ptrs[9] = {u, sx, sy, sz, lam_x, lam_y, lam_z, mu, v};
    for (const void *p : ptrs)
        if ((uintptr_t)p % w) return TPO_ERR_INVALID_ARG;
    if ((unsigned long long)num_elems > (~(size_t)0 >> 16)) return TPO_ERR_INVALID_ARG;
    const size_t field = (size_t)num_elems * n * n * n * w;
    const size_t mat = (size_t)n * n * w;
    const size_t vec = (size_t)n * w;
    if (v != u && overlaps(v, field, u, field)) return TPO_ERR_ALIAS;
    if (overlaps(v, field, sx, mat) || overlaps(v, field, sy, mat) ||
        overlaps(v, field, sz, mat))
        return TPO_ERR_ALIAS;
    if (overlaps(v, field, lam_x, vec) || overlaps(v, field, lam_y, vec) ||
        overlaps(v, field, lam_z, vec) || overlaps(v, field, mu, (size_t)num_elems * w))
        return TPO_ERR_ALIAS;
    return TPO_OK;
}

}  // namespace tpo

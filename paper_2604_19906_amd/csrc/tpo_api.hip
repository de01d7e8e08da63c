// C-ABI entry points of libtpo: per-device reference counting, validation, choice of the
// kernel family for (n, dtype) and the single kernel launch on the caller's stream.
#include <hip/hip_runtime.h>

#include <cstring>
#include <mutex>

#include "tpo.h"
#include "tpo_internal.h"

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_mu;
int g_refs[kMaxDevices] = {0};

// Family chosen by TPO_VARIANT_AUTO, from measurements on MI355X.
int auto_variant(int n, int dtype, bool shared_s, long long num_elems)
{
    // Measured on MI355X at the sizes of the named workloads (ms per launch, pencil / MFMA):
    // fp64 n=8 0.25 / 0.27, n=11 1.46 / 1.69, fp32 n=13 5.99 / 6.09: pencil.
    // fp64 n=16: pencil 1.16-1.23; MFMA 1.13-1.17 when one matrix is shared by the three
    // directions (A operands held once: 134 instead of 156 VGPRs), 1.21 with three distinct
    // matrices.  With a shared matrix the matrix-core kernel leads at every batch size (us per
    // launch, pencil / MFMA: E = 1024 26.2 / 22.1, 2048 46.2 / 36.4, 4096 80.9 / 77.1, 8192 148.5 /
    // 145.4, 12288 236 / 220, 16384 311 / 292), so the choice does not depend on num_elems.
    (void)num_elems;
    if (dtype == TPO_F64 && n == 16 && shared_s) return TPO_VARIANT_MFMA;
    // fp32: with 4x4x1 matrix-core products the pencil kernel leaves the vector-FMA bound
    // (n=13, E=1048576: 5.5 against 6.0 ms).  All three families on 1 GiB fields, every n, each at
    // its best setting (GB/s, vector-FMA pencil / 4x4x1 pencil / MFMA tiles): n=8 6079/5853/4790,
    // n=9 5497/5484/3849, n=11 4939/5040/4440, n=12 4492/4934/4488, n=13 4559/5114/4197,
    // n=14 3748/3990/4071, n=15 3873/4361/4607, n=16 4012/4878/5599: vector FMA up to n=7, the
    // 4x4x1 kernels for n=8..13 (n=8 with non-temporal u loads and stores: 6181/6401), the
    // 16-wide tiles once n fills them (n >= 14).
    if (dtype == TPO_F32 && n >= 14) return TPO_VARIANT_MFMA;
    if (dtype == TPO_F32 && n >= 8) return TPO_VARIANT_PENCIL_MM;
    return TPO_VARIANT_PENCIL;
}

const tpo::KernelEntry *lookup(int n, int dtype, int variant)
{
    if (variant == TPO_VARIANT_PENCIL) return tpo::pencil_entry(n, dtype);
    if (variant == TPO_VARIANT_MFMA) return tpo::mfma_entry(n, dtype);
    if (variant == TPO_VARIANT_PENCIL_MM) return tpo::pencil_mm_entry(n, dtype);
    return nullptr;
}

// Status of an entry point from what its launcher returned.
int launch_status(hipError_t err)
{
    if (err == hipSuccess) return TPO_OK;
    (void)hipGetLastError();
    return err == tpo::kGridTooLarge ? TPO_ERR_UNSUPPORTED : TPO_ERR_DEVICE;
}

// True when tpo_create has succeeded (and not been undone) on the calling thread's device.
bool created_on_current_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return false;
    }
    std::lock_guard<std::mutex> lock(g_mu);
    return g_refs[dev] > 0;
}

}  // namespace

extern "C" {

int tpo_create(void)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return TPO_ERR_DEVICE;
    }
    hipDeviceProp_t prop;
    if (hipGetDeviceProperties(&prop, dev) != hipSuccess) {
        (void)hipGetLastError();
        return TPO_ERR_DEVICE;
    }
    if (std::strncmp(prop.gcnArchName, "gfx950", 6) != 0) return TPO_ERR_DEVICE;
    std::lock_guard<std::mutex> lock(g_mu);
    if (g_refs[dev] == 0) {
        for (int dt = 0; dt < 2; ++dt)
            for (int n = 1; n <= TPO_MAX_N; ++n)
                for (int var : {TPO_VARIANT_PENCIL, TPO_VARIANT_MFMA, TPO_VARIANT_PENCIL_MM}) {
                    const tpo::KernelEntry *k = lookup(n, dt, var);
                    if (k && k->prepare && k->prepare() != hipSuccess) {
                        (void)hipGetLastError();
                        return TPO_ERR_DEVICE;
                    }
                }
        for (int n = 1; n <= TPO_MAX_N; ++n)
            for (const tpo::ConvectionEntry *k :
                 {tpo::convection_entry(n, n, TPO_F64), tpo::convection_entry(n, n, TPO_F32)})
                if (k && k->prepare() != hipSuccess) {
                    (void)hipGetLastError();
                    return TPO_ERR_DEVICE;
                }
        for (int dt = 0; dt < 2; ++dt)
            for (int i = 0; i < tpo::convection_rect_count(dt); ++i) {
                const tpo::ConvectionEntry *k = tpo::convection_rect_at(i, dt);
                if (k && k->prepare() != hipSuccess) {
                    (void)hipGetLastError();
                    return TPO_ERR_DEVICE;
                }
            }
        for (int dt = 0; dt < 2; ++dt)
            for (int n = 1; n <= TPO_MAX_N; ++n) {
                const tpo::TransformEntry *k = tpo::transform_entry(n, dt);
                if (k && (k->prepare_forward() != hipSuccess || k->prepare_backward() != hipSuccess)) {
                    (void)hipGetLastError();
                    return TPO_ERR_DEVICE;
                }
            }
    }
    ++g_refs[dev];
    return TPO_OK;
}

int tpo_destroy(void)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        (void)hipGetLastError();
        return TPO_ERR_NOT_INITIALIZED;
    }
    std::lock_guard<std::mutex> lock(g_mu);
    if (g_refs[dev] <= 0) return TPO_ERR_NOT_INITIALIZED;
    --g_refs[dev];
    return TPO_OK;
}

int tpo_ihelm_variant_for_batch(int n, int dtype, int shared_s, long long num_elems)
{
    if (dtype != TPO_F64 && dtype != TPO_F32) return TPO_ERR_INVALID_ARG;
    if (n < 1 || num_elems < 0) return TPO_ERR_INVALID_ARG;
    if (n > TPO_MAX_N) return TPO_ERR_UNSUPPORTED;
    int var = auto_variant(n, dtype, shared_s != 0, num_elems);
    if (!lookup(n, dtype, var)) var = TPO_VARIANT_PENCIL;
    return var;
}

int tpo_ihelm_variant_for(int n, int dtype, int shared_s)
{
    return tpo_ihelm_variant_for_batch(n, dtype, shared_s, 1LL << 40);
}

int tpo_ihelm_has_variant(int n, int dtype, int variant)
{
    if (dtype != TPO_F64 && dtype != TPO_F32) return 0;
    if (n < 1 || n > TPO_MAX_N) return 0;
    if (variant == TPO_VARIANT_AUTO) variant = tpo_ihelm_variant_for(n, dtype, 0);
    return lookup(n, dtype, variant) != nullptr;
}

int tpo_ihelm_apply_variant(const void *u, const void *S_x, const void *S_y, const void *S_z,
                            const void *D, void *v, int n, long long num_elems, int dtype,
                            void *stream, int variant)
{
    const int rc = tpo::validate_apply(u, S_x, S_y, S_z, D, v, n, num_elems, dtype, variant);
    if (rc != TPO_OK) return rc;
    if (variant == TPO_VARIANT_AUTO)
        variant = tpo_ihelm_variant_for_batch(n, dtype, S_x == S_y && S_y == S_z, num_elems);
    const tpo::KernelEntry *k = lookup(n, dtype, variant);
    if (!k) return TPO_ERR_UNSUPPORTED;
    if (num_elems == 0) return TPO_OK;

    if (!created_on_current_device()) return TPO_ERR_NOT_INITIALIZED;
    tpo::ApplyArgs a{u, S_x, S_y, S_z, D, v, num_elems, (hipStream_t)stream};
    return launch_status(k->launch(a));
}

int tpo_convection_has_shape(int n_v, int n_q, int dtype)
{
    if (dtype != TPO_F64 && dtype != TPO_F32) return 0;
    if (n_v < 1 || n_q < 1 || n_v > TPO_MAX_N || n_q > TPO_MAX_N) return 0;
    return tpo::convection_entry(n_v, n_q, dtype) != nullptr;
}

int tpo_convection_apply(const void *P, const void *M, const void *D_vq, const void *I_vq, void *F,
                         int n_v, int n_q, long long num_elems, int dtype, void *stream)
{
    const tpo::ConvectionEntry *k =
        tpo_convection_has_shape(n_v, n_q, dtype) ? tpo::convection_entry(n_v, n_q, dtype) : nullptr;
    const int rc = tpo::validate_convection(P, M, D_vq, I_vq, F, n_v, n_q, num_elems, dtype,
                                            k != nullptr);
    if (rc != TPO_OK) return rc;
    if (!k) return TPO_ERR_UNSUPPORTED;
    if (num_elems == 0) return TPO_OK;

    if (!created_on_current_device()) return TPO_ERR_NOT_INITIALIZED;
    tpo::ConvectionArgs a{P, M, D_vq, I_vq, F, num_elems, (hipStream_t)stream};
    return launch_status(k->launch(a));
}

int tpo_transform_apply(const void *u, const void *S_x, const void *S_y, const void *S_z, void *t,
                        int n, long long num_elems, int dtype, int direction, void *stream)
{
    const int rc = tpo::validate_transform(u, S_x, S_y, S_z, t, n, num_elems, dtype, direction);
    if (rc != TPO_OK) return rc;
    const tpo::TransformEntry *k = tpo::transform_entry(n, dtype);
    if (!k) return TPO_ERR_UNSUPPORTED;
    if (num_elems == 0) return TPO_OK;

    if (!created_on_current_device()) return TPO_ERR_NOT_INITIALIZED;
    tpo::TransformArgs a{u, S_x, S_y, S_z, t, num_elems, (hipStream_t)stream};
    return launch_status(direction == TPO_FORWARD ? k->launch_forward(a) : k->launch_backward(a));
}

int tpo_ihelm_sep_variant_for_batch(int n, int dtype, int shared_s, long long num_elems)
{
    if (dtype != TPO_F64 && dtype != TPO_F32) return TPO_ERR_INVALID_ARG;
    if (n < 1 || num_elems < 0) return TPO_ERR_INVALID_ARG;
    if (n > TPO_MAX_N) return TPO_ERR_UNSUPPORTED;
    // Every family has the separable form, and the D form's choice holds for it too.  Measured
    // on MI355X (ms per launch, best pencil family / matrix-core tiles): fp64 n=16, E=65536, one
    // shared matrix 1.112 / 1.052; fp32, E=262144: n=14 2.038 / 2.029, n=15 2.323 / 2.203,
    // n=16 2.407 / 2.070.
    int var = auto_variant(n, dtype, shared_s != 0, num_elems);
    const tpo::KernelEntry *k = lookup(n, dtype, var);
    if (!k || !k->launch_sep)
        var = (dtype == TPO_F32 && n >= 8) ? TPO_VARIANT_PENCIL_MM : TPO_VARIANT_PENCIL;
    return var;
}

int tpo_ihelm_sep_variant_for(int n, int dtype)
{
    return tpo_ihelm_sep_variant_for_batch(n, dtype, 0, 1LL << 40);
}

int tpo_ihelm_sep_has_variant(int n, int dtype, int variant)
{
    if (dtype != TPO_F64 && dtype != TPO_F32) return 0;
    if (n < 1 || n > TPO_MAX_N) return 0;
    if (variant == TPO_VARIANT_AUTO) variant = tpo_ihelm_sep_variant_for(n, dtype);
    const tpo::KernelEntry *k = lookup(n, dtype, variant);
    return k != nullptr && k->launch_sep != nullptr;
}

int tpo_ihelm_apply_sep_variant(const void *u, const void *S_x, const void *S_y, const void *S_z,
                                const void *lam_x, const void *lam_y, const void *lam_z,
                                const void *mu, void *v, int n, long long num_elems, int dtype,
                                void *stream, int variant)
{
    const int rc = tpo::validate_apply_sep(u, S_x, S_y, S_z, lam_x, lam_y, lam_z, mu, v, n,
                                           num_elems, dtype, variant);
    if (rc != TPO_OK) return rc;
    if (variant == TPO_VARIANT_AUTO)
        variant = tpo_ihelm_sep_variant_for_batch(n, dtype, S_x == S_y && S_y == S_z, num_elems);
    const tpo::KernelEntry *k = lookup(n, dtype, variant);
    if (!k || !k->launch_sep) return TPO_ERR_UNSUPPORTED;
    if (num_elems == 0) return TPO_OK;

    if (!created_on_current_device()) return TPO_ERR_NOT_INITIALIZED;
    tpo::ApplyArgs a{u, S_x, S_y, S_z, nullptr, v, num_elems, (hipStream_t)stream,
                     lam_x, lam_y, lam_z, mu};
    return launch_status(k->launch_sep(a));
}

int tpo_ihelm_apply_sep(const void *u, const void *S_x, const void *S_y, const void *S_z,
                        const void *lam_x, const void *lam_y, const void *lam_z, const void *mu,
                        void *v, int n, long long num_elems, int dtype, void *stream)
{
    return tpo_ihelm_apply_sep_variant(u, S_x, S_y, S_z, lam_x, lam_y, lam_z, mu, v, n, num_elems,
                                       dtype, stream, TPO_VARIANT_AUTO);
}

int tpo_ihelm_apply_aniso(const void *u, const void *S_x, const void *S_y, const void *S_z,
                          const void *D, void *v, int n_x, int n_y, int n_z, long long num_elems,
                          int dtype, void *stream)
{
    if (n_x == n_y && n_y == n_z)       // cubic: the tuned kernels
        return tpo_ihelm_apply_variant(u, S_x, S_y, S_z, D, v, n_x, num_elems, dtype, stream,
                                       TPO_VARIANT_AUTO);
    const int rc = tpo::validate_apply_aniso(u, S_x, S_y, S_z, D, v, n_x, n_y, n_z, num_elems, dtype);
    if (rc != TPO_OK) return rc;
    if (num_elems == 0) return TPO_OK;
    if (!created_on_current_device()) return TPO_ERR_NOT_INITIALIZED;
    tpo::AnisoArgs a{u, S_x, S_y, S_z, D, v, n_x, n_y, n_z, num_elems, (hipStream_t)stream};
    return launch_status(tpo::launch_ihelm_generic(a, dtype));
}

int tpo_ihelm_apply(const void *u, const void *S_x, const void *S_y, const void *S_z,
                    const void *D, void *v, int n, long long num_elems, int dtype,
                    void *stream)
{
    return tpo_ihelm_apply_variant(u, S_x, S_y, S_z, D, v, n, num_elems, dtype, stream,
                                   TPO_VARIANT_AUTO);
}

const char *tpo_status_string(int status)
{
    switch (status) {
    case TPO_OK: return "ok";
    case TPO_ERR_INVALID_ARG: return "invalid argument";
    case TPO_ERR_UNSUPPORTED: return "unsupported n or kernel variant";
    case TPO_ERR_NOT_INITIALIZED: return "tpo_create has not been called on this device";
    case TPO_ERR_DEVICE: return "no gfx950 device or HIP launch failure";
    case TPO_ERR_ALIAS: return "output overlaps an input (only v == u is allowed)";
    default: return "unknown status";
    }
}

}  // extern "C"

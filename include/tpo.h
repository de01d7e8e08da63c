/*
 * tpo.h -- C ABI of the MI355X (gfx950) batched inverse-Helmholtz tensor-product operator.
 *
 * The operator is the `inv_helm` spectral-element kernel evaluated in the paper (Table 1,
 * Table 2): per element a forward three-dimensional transform made of one-dimensional mode
 * products (Sec. 2.2: tensor-product operators are applied "successively as one-dimensional
 * transformations"; Sec. 5.2 gives the forward triple sum and its lifted, sum-factorised
 * form), a pointwise scale by a per-element diagonal, and the backward transform:
 *
 *   t[i,j,k] = sum_l sum_m sum_q  S_x[l,i] * S_y[m,j] * S_z[q,k] * u_e[l,m,q]
 *   g[i,j,k] = D_e[i,j,k] * t[i,j,k]
 *   v_e[i,j,k] = sum_l sum_m sum_q  S_x[i,l] * S_y[j,m] * S_z[k,q] * g[l,m,q]
 *
 * i.e. v_e = (S_x (x) S_y (x) S_z) diag(D_e) (S_x (x) S_y (x) S_z)^T u_e on the row-major
 * flattening of the n*n*n cube.  Elements are independent (Sec. 6.1).
 *
 * Plain C types only; no exception crosses this boundary; every function returns a
 * tpo_status_t (as int) unless stated otherwise.
 */
#ifndef TPO_H
#define TPO_H

#ifdef __cplusplus
extern "C" {
#endif

/* Element type of u, S_*, D and v.  The arithmetic runs in the same type. */
typedef enum { TPO_F64 = 0, TPO_F32 = 1 } tpo_dtype_t;

typedef enum {
    TPO_OK = 0,
    TPO_ERR_INVALID_ARG = -1,      /* NULL pointer with num_elems > 0, n < 1, num_elems < 0,
                                      unknown dtype or variant, misaligned pointer */
    TPO_ERR_UNSUPPORTED = -2,      /* n > TPO_MAX_N, a variant that has no kernel for (n, dtype), or a
                                      batch that needs more than 2^31-1 workgroups in one launch */
    TPO_ERR_NOT_INITIALIZED = -3,  /* tpo_create has not succeeded on the current device */
    TPO_ERR_DEVICE = -4,           /* no gfx950 device, or THIS launch was rejected by HIP (an error
                                      left recorded by the caller's earlier HIP calls is dropped
                                      before the launch and never reported here) */
    TPO_ERR_ALIAS = -5             /* v overlaps an input other than "v == u exactly" */
} tpo_status_t;

/* Kernel families (the choice per (n, dtype) is the library's unless forced). */
typedef enum {
    TPO_VARIANT_AUTO = 0,    /* the library's measured choice for (n, dtype) */
    TPO_VARIANT_PENCIL = 1,  /* register-blocked vector FMAs, one pencil per lane */
    TPO_VARIANT_MFMA = 2,    /* matrix-core tiles (v_mfma_f64_16x16x4 / v_mfma_f32_16x16x4) */
    TPO_VARIANT_PENCIL_MM = 3 /* fp32 only: the pencil kernel's data movement, its FMAs issued four
                                 at a time as 4x4x1 matrix-core outer products
                                 (v_mfma_f32_4x4x1 with A broadcast) */
} tpo_variant_t;

/* Which half of the operator tpo_transform_apply evaluates. */
typedef enum {
    TPO_FORWARD = 0,   /* t = (S_x (x) S_y (x) S_z)^T u: sums over the FIRST index of each matrix */
    TPO_BACKWARD = 1   /* t = (S_x (x) S_y (x) S_z) u:   sums over the SECOND index */
} tpo_direction_t;

#define TPO_MAX_N 16         /* points per direction supported: 1 .. TPO_MAX_N */

/*
 * tpo_create -- bind the library to the calling thread's current HIP device.
 * Checks that the device is gfx950 and prepares the kernel table (raises the dynamic
 * LDS limit of the kernels that need it).  Reference counted per device: every successful
 * call must be matched by one tpo_destroy.  Allocates no device memory.
 * Errors: TPO_ERR_DEVICE when there is no usable gfx950 device.
 */
int tpo_create(void);

/* tpo_destroy -- drop one reference on the current device.
 * Errors: TPO_ERR_NOT_INITIALIZED when there is none to drop. */
int tpo_destroy(void);

/*
 * tpo_ihelm_apply -- enqueue v_e = (S_x(x)S_y(x)S_z) [ D_e .* ((S_x(x)S_y(x)S_z)^T u_e) ]
 * for e = 0 .. num_elems-1 (operator above; Sec. 2.2 and Sec. 5.2 of the paper).
 *
 *   u, D   DEVICE pointers, read only, [num_elems][n][n][n] C-contiguous (axis 2 fastest)
 *   v      DEVICE pointer, written, same shape.  v == u (exactly) is allowed: every u_e is
 *          read on chip before v_e is written.  Any other overlap of v with u, D or an S
 *          is rejected with TPO_ERR_ALIAS.
 *   S_x, S_y, S_z
 *          DEVICE pointers, read only, [n][n] row-major (S[a*n+b]), shared by all elements;
 *          S_x pairs with cube axis 0 (slowest), S_y with axis 1, S_z with axis 2 (fastest).
 *          The forward transform applies the transpose of each stored matrix (it sums over
 *          the first index), the backward transform the matrix itself.  The three pointers
 *          may be equal.
 *   n      points per direction (polynomial degree + 1), 1 .. TPO_MAX_N
 *   num_elems  number of elements E >= 0; 0 is a no-op returning TPO_OK
 *   dtype  tpo_dtype_t of every array; arithmetic is done in that type
 *   stream hipStream_t passed as void* (NULL = the default stream)
 *
 * Alignment: every pointer must be aligned to its element size (8 or 4 bytes); nothing more
 * is assumed (odd n makes individual elements only word aligned).
 * Ownership: the caller owns all buffers before, during and after the call; the library
 * allocates nothing, keeps no pointer after the kernel has run, and never synchronises: the
 * call enqueues one kernel on `stream` and returns.  Re-entrant after tpo_create.
 * Errors (checked on the host, in this order, before any HIP call): TPO_ERR_INVALID_ARG,
 * TPO_ERR_UNSUPPORTED, TPO_ERR_ALIAS, then TPO_ERR_NOT_INITIALIZED, then TPO_ERR_DEVICE if
 * HIP rejects the launch.
 */
int tpo_ihelm_apply(const void *u, const void *S_x, const void *S_y, const void *S_z,
                    const void *D, void *v, int n, long long num_elems, int dtype,
                    void *stream);

/*
 * tpo_ihelm_apply_variant -- the same operation with the kernel family forced
 * (tpo_variant_t), for A/B measurements and for testing each family on its own.
 * TPO_VARIANT_AUTO makes it identical to tpo_ihelm_apply.
 * Extra error: TPO_ERR_UNSUPPORTED when the family has no kernel for (n, dtype).
 */
int tpo_ihelm_apply_variant(const void *u, const void *S_x, const void *S_y, const void *S_z,
                            const void *D, void *v, int n, long long num_elems, int dtype,
                            void *stream, int variant);

/* tpo_ihelm_variant_for -- which family TPO_VARIANT_AUTO selects for (n, dtype) on a large
 * batch (the choice can depend on the batch size: see tpo_ihelm_variant_for_batch).
 * shared_s != 0 asks about calls that pass ONE matrix for all three directions (S_x, S_y and
 * S_z are the same pointer), 0 about calls with distinct pointers; the choice can differ
 * because the matrix-core kernels hold a shared matrix once.
 * Returns TPO_VARIANT_PENCIL, TPO_VARIANT_MFMA or TPO_VARIANT_PENCIL_MM, or TPO_ERR_UNSUPPORTED /
 * TPO_ERR_INVALID_ARG.
 * Pure host function; needs no device. */
int tpo_ihelm_variant_for(int n, int dtype, int shared_s);

/* tpo_ihelm_variant_for_batch -- the family TPO_VARIANT_AUTO selects for a call with
 * num_elems elements (the paper times 8192 elements per call, Sec. 6.1; with a few thousand
 * workgroups per launch another family can be ahead of the large-batch choice; with the
 * kernels as they stand the answer is the same for every num_elems).  Arguments,
 * return values and errors as tpo_ihelm_variant_for; num_elems < 0 is TPO_ERR_INVALID_ARG.
 * Pure host function; needs no device. */
int tpo_ihelm_variant_for_batch(int n, int dtype, int shared_s, long long num_elems);

/* tpo_ihelm_has_variant -- 1 if `variant` has a kernel for (n, dtype), else 0
 * (TPO_VARIANT_AUTO always has one for supported n). */
int tpo_ihelm_has_variant(int n, int dtype, int variant);

/*
 * tpo_ihelm_apply_sep -- the same operator for diagonals of separable (fast-diagonalisation)
 * form, which is how the evaluated workloads build D_e:
 *
 *     D_e[i,j,k] = 1 / (lam_x[i] + lam_y[j] + lam_z[k] + mu[e])
 *
 * The kernel evaluates D_e where it is used instead of reading it: one of the three HBM streams
 * of tpo_ihelm_apply disappears (2*n^3 instead of 3*n^3 words per element), at the price of n^3
 * divisions per element.  This is the operator's share of the buffer sharing that the paper
 * credits for part of inv_helm's speed (Sec. 6.2): an array that can be recomputed from 3n + 1
 * numbers is not materialised.
 *
 *   lam_x, lam_y, lam_z   DEVICE pointers, read only, [n] each (may be equal); lam_x pairs with
 *                         cube axis 0, like S_x
 *   mu                    DEVICE pointer, read only, [num_elems]
 *   every other argument  as in tpo_ihelm_apply
 *
 * Arithmetic: the denominator is summed left to right, ((lam_x[i] + lam_y[j]) + lam_z[k]) + mu[e],
 * in `dtype`; its reciprocal is the hardware reciprocal, in fp64 refined by two Newton steps:
 * within 2 ulp (fp64) / 1 ulp (fp32) of the IEEE quotient for normal denominators, so the result
 * agrees with tpo_ihelm_apply on an IEEE-divided D_e to a few ulp, not bit for bit.  A zero
 * denominator gives Inf/NaN; it is not checked.
 * Errors: as tpo_ihelm_apply (v must not overlap lam_* or mu either); TPO_ERR_UNSUPPORTED
 * from the _variant form when the family has no kernel for (n, dtype).
 */
int tpo_ihelm_apply_sep(const void *u, const void *S_x, const void *S_y, const void *S_z,
                        const void *lam_x, const void *lam_y, const void *lam_z, const void *mu,
                        void *v, int n, long long num_elems, int dtype, void *stream);

/* The same with the kernel family forced, and the queries that go with it: which family
 * TPO_VARIANT_AUTO selects (tpo_ihelm_sep_variant_for: three distinct matrix pointers, large
 * batch; tpo_ihelm_sep_variant_for_batch: for shared_s and num_elems as in
 * tpo_ihelm_variant_for_batch), and whether a family has a separable form for (n, dtype). */
int tpo_ihelm_apply_sep_variant(const void *u, const void *S_x, const void *S_y, const void *S_z,
                                const void *lam_x, const void *lam_y, const void *lam_z,
                                const void *mu, void *v, int n, long long num_elems, int dtype,
                                void *stream, int variant);
int tpo_ihelm_sep_variant_for(int n, int dtype);
int tpo_ihelm_sep_variant_for_batch(int n, int dtype, int shared_s, long long num_elems);
int tpo_ihelm_sep_has_variant(int n, int dtype, int variant);

/*
 * tpo_ihelm_apply_aniso -- the operator of tpo_ihelm_apply on anisotropic elements: n_x, n_y, n_z
 * points along cube axes 0, 1, 2 (each 1 .. TPO_MAX_N).  u, D, v are
 * [num_elems][n_x][n_y][n_z] C-contiguous, S_x is [n_x][n_x], S_y [n_y][n_y], S_z [n_z][n_z].
 * With n_x == n_y == n_z the call is tpo_ihelm_apply; every other shape runs one kernel with
 * runtime sizes whose mode products are compiled for every size of their own axis (measured
 * 3.8 - 6.1 TB/s of algorithmic traffic, against 5.0 - 5.8 of the tuned cubic kernels).
 * Everything else (alignment, aliasing, ownership, stream, error order) as in tpo_ihelm_apply.
 */
int tpo_ihelm_apply_aniso(const void *u, const void *S_x, const void *S_y, const void *S_z,
                          const void *D, void *v, int n_x, int n_y, int n_z, long long num_elems,
                          int dtype, void *stream);

/*
 * tpo_transform_apply -- one half of the operator on its own, for e = 0 .. num_elems-1:
 *
 *   TPO_FORWARD   t_e[i,j,k] = sum_l sum_m sum_q  S_x[l,i] * S_y[m,j] * S_z[q,k] * u_e[l,m,q]
 *   TPO_BACKWARD  t_e[i,j,k] = sum_l sum_m sum_q  S_x[i,l] * S_y[j,m] * S_z[k,q] * u_e[l,m,q]
 *
 * The forward transform is the worked example of reduction lifting in Sec. 5.2 of the paper
 * (the triple sum evaluated as three one-dimensional sums); tpo_ihelm_apply is forward, scale by
 * D_e, backward.  Arguments, layout, alignment, ownership and stream semantics as in
 * tpo_ihelm_apply; t == u exactly is allowed, any other overlap of t with u or an S is
 * TPO_ERR_ALIAS; direction other than TPO_FORWARD / TPO_BACKWARD is TPO_ERR_INVALID_ARG.
 */
int tpo_transform_apply(const void *u, const void *S_x, const void *S_y, const void *S_z, void *t,
                        int n, long long num_elems, int dtype, int direction, void *stream);

/*
 * tpo_convection_apply -- volume integral of the convective flux, Eq. 1 of the paper (the
 * `convection` kernel of its Tables 1 and 2).  Per velocity component c and element e it is the
 * sum over the three flux directions d of a tensor-product operator applied to the
 * metric-weighted flux of that direction: the differentiation matrix acts along direction d, the
 * interpolation matrix along the other two.  With the cube axes numbered from the fastest one
 * (axis 0 = last array index, direction d = 0 is xi):
 *
 *   F[c,e] = sum_{d=0,1,2}  ( A(d,2) (x) A(d,1) (x) A(d,0) )  ( M[e] .* P[c,d,e] ),
 *   A(d,a) = D_vq if a == d, else I_vq,
 *
 * each factor A[x,q] contracting the quadrature index q of its axis.
 *
 *   P      DEVICE pointer, read only, [3][3][num_elems][n_q][n_q][n_q] C-contiguous: velocity
 *          component c, flux direction (xi, eta, zeta), element, quadrature point (last index fastest)
 *   M      DEVICE pointer, read only, [num_elems][n_q][n_q][n_q]: metric factor per quadrature point
 *   D_vq, I_vq
 *          DEVICE pointers, read only, [n_v][n_q] row-major: differentiation and interpolation
 *          from the n_q quadrature points to the n_v nodes of one direction
 *   F      DEVICE pointer, written, [3][num_elems][n_v][n_v][n_v]; must not overlap any input
 *   n_v, n_q  1 .. TPO_MAX_N.  Kernels exist for n_v == n_q (every n) and for the over-integration
 *          shapes n_q in {n_v + 1, n_v + 2, ceil(3 n_v / 2)} with n_v in 2 .. 12 and n_q <= 16;
 *          any other pair returns TPO_ERR_UNSUPPORTED (tpo_convection_has_shape tells)
 *   num_elems, dtype, stream, alignment, ownership, error order: as in tpo_ihelm_apply.
 */
int tpo_convection_apply(const void *P, const void *M, const void *D_vq, const void *I_vq, void *F,
                         int n_v, int n_q, long long num_elems, int dtype, void *stream);

/* tpo_convection_has_shape -- 1 if tpo_convection_apply has a kernel for (n_v, n_q, dtype),
 * else 0.  Pure host function. */
int tpo_convection_has_shape(int n_v, int n_q, int dtype);

/* tpo_status_string -- static, NUL-terminated description of a status; never freed. */
const char *tpo_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* TPO_H */

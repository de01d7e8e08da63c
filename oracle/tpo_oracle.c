/*
 * CPU oracle for the batched inverse-Helmholtz tensor-product operator.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the operator
 * computes.  It is linked by nothing in the product library; only the tests, the smoke
 * check and the benchmark's CPU-baseline leg call it.  It shares no code with the GPU path.
 *
 * Operator (per element e, independent of every other element; Sec. 2.2 describes such
 * tensor-product operators as successive one-dimensional transformations, Sec. 6.1 states
 * the per-element parallelism):
 *
 *   forward   t[i,j,k] = sum_l sum_m sum_q  Sx[l,i] * Sy[m,j] * Sz[q,k] * u[l,m,q]
 *   scale     g[i,j,k] = D[i,j,k] * t[i,j,k]
 *   backward  v[i,j,k] = sum_l sum_m sum_q  Sx[i,l] * Sy[j,m] * Sz[k,q] * g[l,m,q]
 *
 * i.e. v = (Sx (x) Sy (x) Sz) diag(D) (Sx (x) Sy (x) Sz)^T u on the row-major flattening of
 * the cube.  The forward half is the worked example of Sec. 5.2 ("reduction lifting"): the
 * matrix written S^T there is the transpose of the array passed in, so the forward sums
 * run over the FIRST index of the row-major array and the backward sums over the SECOND.
 * Indices run 0..p inclusive in the paper, so n = p + 1 points per direction.
 *
 * Layout: u, D, v are [E][n][n][n] C-contiguous (axis 2 fastest); Sx, Sy, Sz are [n][n]
 * row-major and pair with axis 0, 1, 2.
 *
 * All arithmetic is IEEE double, accumulated left to right, no blocking, no reordering
 * beyond what the two forms below state.  Compile with -ffp-contract=off so that no
 * multiply-add is fused.
 *
 * Pins (tests/test_oracle_pins.py): explicit n^3 x n^3 Kronecker matrix, exact rational
 * evaluation on tiny inputs, orthogonal-S identity, eigenvector property with three
 * distinct non-symmetric matrices, dense Helmholtz solve, linearity, self-adjointness;
 * for the separable-diagonal form the dense Helmholtz solve with three different operators
 * and the entry-by-entry definition of D.
 */
#include <stddef.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define TPO_ORACLE_MAX_N 64

/* One mode product along one axis of an n x n x n cube.
 *   axis 0: out[i,b,c] = sum_l M(l,i) * in[l,b,c]
 *   axis 1: out[a,j,c] = sum_m M(m,j) * in[a,m,c]
 *   axis 2: out[a,b,k] = sum_q M(q,k) * in[a,b,q]
 * where M(r,o) = S[r*n+o] when transposed != 0 (the forward transform, which applies the
 * transpose of the stored matrix) and M(r,o) = S[o*n+r] otherwise (the backward one). */
static void mode_product(const double *S, int transposed, int axis, int n,
                         const double *in, double *out)
{
    for (int a = 0; a < n; ++a)
        for (int b = 0; b < n; ++b)
            for (int c = 0; c < n; ++c) {
                double acc = 0.0;
                for (int r = 0; r < n; ++r) {
                    int o = (axis == 0) ? a : (axis == 1) ? b : c;
                    double m = transposed ? S[r * n + o] : S[o * n + r];
                    size_t src = (axis == 0) ? ((size_t)r * n + b) * n + c
                               : (axis == 1) ? ((size_t)a * n + r) * n + c
                                             : ((size_t)a * n + b) * n + r;
                    acc = acc + m * in[src];
                }
                out[((size_t)a * n + b) * n + c] = acc;
            }
}

/* Lifted (sum-factorised) form, Sec. 5.2: the innermost sum (fastest axis) is taken first,
 * then the middle one, then the outermost, for the forward and for the backward half.
 * Returns 0, or -1 on a bad argument or failed allocation.  nthreads <= 0 means "all". */
int tpo_oracle_ihelm_lifted(const double *u, const double *Sx, const double *Sy,
                            const double *Sz, const double *D, double *v, int n,
                            long long num_elems, int nthreads)
{
    if (n < 1 || n > TPO_ORACLE_MAX_N || num_elems < 0) return -1;
    if (num_elems == 0) return 0;
    if (!u || !Sx || !Sy || !Sz || !D || !v) return -1;
    const size_t cube = (size_t)n * n * n;
    int failed = 0;
#ifdef _OPENMP
    if (nthreads <= 0) nthreads = omp_get_max_threads();
#else
    nthreads = 1;
#endif
#pragma omp parallel num_threads(nthreads)
    {
        double *p = (double *)malloc(cube * sizeof(double));
        double *q = (double *)malloc(cube * sizeof(double));
        if (!p || !q) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        if (!failed) {
#pragma omp for schedule(static)
            for (long long e = 0; e < num_elems; ++e) {
                const double *ue = u + (size_t)e * cube;
                const double *De = D + (size_t)e * cube;
                double *ve = v + (size_t)e * cube;
                mode_product(Sz, 1, 2, n, ue, p);
                mode_product(Sy, 1, 1, n, p, q);
                mode_product(Sx, 1, 0, n, q, p);
                for (size_t x = 0; x < cube; ++x) q[x] = De[x] * p[x];
                mode_product(Sz, 0, 2, n, q, p);
                mode_product(Sy, 0, 1, n, p, q);
                mode_product(Sx, 0, 0, n, q, ve);
            }
        }
        free(p);
        free(q);
    }
    return failed ? -1 : 0;
}

/* Unlifted form: the six-deep sums exactly as the definition writes them, O(n^6) per
 * element.  Serves as the slow cross-check of the lifted form (Sec. 5.2 states the two are
 * the same sum rearranged by distributivity). */
int tpo_oracle_ihelm_direct(const double *u, const double *Sx, const double *Sy,
                            const double *Sz, const double *D, double *v, int n,
                            long long num_elems)
{
    if (n < 1 || n > TPO_ORACLE_MAX_N || num_elems < 0) return -1;
    if (num_elems == 0) return 0;
    if (!u || !Sx || !Sy || !Sz || !D || !v) return -1;
    const size_t cube = (size_t)n * n * n;
    double *g = (double *)malloc(cube * sizeof(double));
    if (!g) return -1;
    for (long long e = 0; e < num_elems; ++e) {
        const double *ue = u + (size_t)e * cube;
        const double *De = D + (size_t)e * cube;
        double *ve = v + (size_t)e * cube;
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < n; ++j)
                for (int k = 0; k < n; ++k) {
                    double t = 0.0;
                    for (int l = 0; l < n; ++l)
                        for (int m = 0; m < n; ++m)
                            for (int q = 0; q < n; ++q)
                                t = t + Sx[l * n + i] * Sy[m * n + j] * Sz[q * n + k]
                                        * ue[((size_t)l * n + m) * n + q];
                    size_t x = ((size_t)i * n + j) * n + k;
                    g[x] = De[x] * t;
                }
        for (int i = 0; i < n; ++i)
            for (int j = 0; j < n; ++j)
                for (int k = 0; k < n; ++k) {
                    double s = 0.0;
                    for (int l = 0; l < n; ++l)
                        for (int m = 0; m < n; ++m)
                            for (int q = 0; q < n; ++q)
                                s = s + Sx[i * n + l] * Sy[j * n + m] * Sz[k * n + q]
                                        * g[((size_t)l * n + m) * n + q];
                    ve[((size_t)i * n + j) * n + k] = s;
                }
    }
    free(g);
    return 0;
}

/* Separable (fast-diagonalisation) diagonal: the operator above with
 *     D[i,j,k] = 1 / (lam_x[i] + lam_y[j] + lam_z[k] + mu[e])
 * written out per element and handed to the lifted form.  With S_d the eigenvectors and lam_d
 * the eigenvalues of three symmetric one-dimensional operators A_d, v solves the separable
 * Helmholtz problem (A_x (x) I (x) I + I (x) A_y (x) I + I (x) I (x) A_z + mu I) v = u, which
 * is what pins this function (tests/test_oracle_pins.py).  The denominator is summed left to
 * right.  Returns 0 or -1 like the functions above. */
int tpo_oracle_ihelm_sep(const double *u, const double *Sx, const double *Sy, const double *Sz,
                         const double *lam_x, const double *lam_y, const double *lam_z,
                         const double *mu, double *v, int n, long long num_elems, int nthreads)
{
    if (n < 1 || n > TPO_ORACLE_MAX_N || num_elems < 0) return -1;
    if (num_elems == 0) return 0;
    if (!u || !Sx || !Sy || !Sz || !lam_x || !lam_y || !lam_z || !mu || !v) return -1;
    const size_t cube = (size_t)n * n * n;
    /* blocks of elements, so that the materialised D stays small whatever num_elems is */
    const long long block = 1024;
    double *D = (double *)malloc((size_t)block * cube * sizeof(double));
    if (!D) return -1;
    int rc = 0;
    for (long long e0 = 0; e0 < num_elems && rc == 0; e0 += block) {
        const long long ne = (num_elems - e0 < block) ? num_elems - e0 : block;
        for (long long e = 0; e < ne; ++e)
            for (int i = 0; i < n; ++i)
                for (int j = 0; j < n; ++j)
                    for (int k = 0; k < n; ++k)
                        D[(size_t)e * cube + ((size_t)i * n + j) * n + k] =
                            1.0 / (((lam_x[i] + lam_y[j]) + lam_z[k]) + mu[e0 + e]);
        rc = tpo_oracle_ihelm_lifted(u + (size_t)e0 * cube, Sx, Sy, Sz, D, v + (size_t)e0 * cube,
                                     n, ne, nthreads);
    }
    free(D);
    return rc;
}

/* Forward half only (the paper's worked example), lifted form: t = (Sx^T (x) Sy^T (x) Sz^T) u. */
int tpo_oracle_forward_lifted(const double *u, const double *Sx, const double *Sy,
                              const double *Sz, double *t, int n, long long num_elems)
{
    if (n < 1 || n > TPO_ORACLE_MAX_N || num_elems < 0) return -1;
    if (num_elems == 0) return 0;
    if (!u || !Sx || !Sy || !Sz || !t) return -1;
    const size_t cube = (size_t)n * n * n;
    double *p = (double *)malloc(cube * sizeof(double));
    double *q = (double *)malloc(cube * sizeof(double));
    if (!p || !q) { free(p); free(q); return -1; }
    for (long long e = 0; e < num_elems; ++e) {
        mode_product(Sz, 1, 2, n, u + (size_t)e * cube, p);
        mode_product(Sy, 1, 1, n, p, q);
        mode_product(Sx, 1, 0, n, q, t + (size_t)e * cube);
    }
    free(p);
    free(q);
    return 0;
}

/* Backward half only, lifted form in the same axis order: v = (Sx (x) Sy (x) Sz) g, i.e. the
 * forward sums of Sec. 5.2 with each matrix used untransposed. */
int tpo_oracle_backward_lifted(const double *g, const double *Sx, const double *Sy,
                               const double *Sz, double *v, int n, long long num_elems)
{
    if (n < 1 || n > TPO_ORACLE_MAX_N || num_elems < 0) return -1;
    if (num_elems == 0) return 0;
    if (!g || !Sx || !Sy || !Sz || !v) return -1;
    const size_t cube = (size_t)n * n * n;
    double *p = (double *)malloc(cube * sizeof(double));
    double *q = (double *)malloc(cube * sizeof(double));
    if (!p || !q) { free(p); free(q); return -1; }
    for (long long e = 0; e < num_elems; ++e) {
        mode_product(Sz, 0, 2, n, g + (size_t)e * cube, p);
        mode_product(Sy, 0, 1, n, p, q);
        mode_product(Sx, 0, 0, n, q, v + (size_t)e * cube);
    }
    free(p);
    free(q);
    return 0;
}

/* ------------------------------------------------------------------------------------------
 * Anisotropic elements: nx, ny, nz points along axes 0, 1, 2 (u, D, v are [E][nx][ny][nz]; Sx is
 * [nx][nx], Sy [ny][ny], Sz [nz][nz]).  Same operator, written on its own so that it does not
 * lean on the cubic routine above: each half as three successive one-dimensional sums, axis 2
 * first (Sec. 5.2), then the plain six-deep sums as a cross-check for small sizes. */
static void aniso_product(const double *S, int transposed, int axis, const int dims[3],
                          const double *in, double *out)
{
    const int n = dims[axis];
    for (int a = 0; a < dims[0]; ++a)
        for (int b = 0; b < dims[1]; ++b)
            for (int c = 0; c < dims[2]; ++c) {
                const int o = (axis == 0) ? a : (axis == 1) ? b : c;
                double acc = 0.0;
                for (int r = 0; r < n; ++r) {
                    const int ia = (axis == 0) ? r : a, ib = (axis == 1) ? r : b, ic = (axis == 2) ? r : c;
                    const double m = transposed ? S[r * n + o] : S[o * n + r];
                    acc = acc + m * in[((size_t)ia * dims[1] + ib) * dims[2] + ic];
                }
                out[((size_t)a * dims[1] + b) * dims[2] + c] = acc;
            }
}

int tpo_oracle_ihelm_aniso(const double *u, const double *Sx, const double *Sy, const double *Sz,
                           const double *D, double *v, int nx, int ny, int nz,
                           long long num_elems, int direct)
{
    if (nx < 1 || ny < 1 || nz < 1 || nx > TPO_ORACLE_MAX_N || ny > TPO_ORACLE_MAX_N ||
        nz > TPO_ORACLE_MAX_N || num_elems < 0)
        return -1;
    if (num_elems == 0) return 0;
    if (!u || !Sx || !Sy || !Sz || !D || !v) return -1;
    const int dims[3] = {nx, ny, nz};
    const size_t cube = (size_t)nx * ny * nz;
    double *p = (double *)malloc(cube * sizeof(double));
    double *q = (double *)malloc(cube * sizeof(double));
    if (!p || !q) { free(p); free(q); return -1; }
    for (long long e = 0; e < num_elems; ++e) {
        const double *ue = u + (size_t)e * cube, *De = D + (size_t)e * cube;
        double *ve = v + (size_t)e * cube;
        if (!direct) {
            aniso_product(Sz, 1, 2, dims, ue, p);
            aniso_product(Sy, 1, 1, dims, p, q);
            aniso_product(Sx, 1, 0, dims, q, p);
            for (size_t x = 0; x < cube; ++x) q[x] = De[x] * p[x];
            aniso_product(Sz, 0, 2, dims, q, p);
            aniso_product(Sy, 0, 1, dims, p, q);
            aniso_product(Sx, 0, 0, dims, q, ve);
            continue;
        }
        for (int i = 0; i < nx; ++i)
            for (int j = 0; j < ny; ++j)
                for (int k = 0; k < nz; ++k) {
                    double t = 0.0;
                    for (int l = 0; l < nx; ++l)
                        for (int m = 0; m < ny; ++m)
                            for (int r = 0; r < nz; ++r)
                                t = t + Sx[l * nx + i] * Sy[m * ny + j] * Sz[r * nz + k]
                                        * ue[((size_t)l * ny + m) * nz + r];
                    const size_t x = ((size_t)i * ny + j) * nz + k;
                    p[x] = De[x] * t;
                }
        for (int i = 0; i < nx; ++i)
            for (int j = 0; j < ny; ++j)
                for (int k = 0; k < nz; ++k) {
                    double acc = 0.0;
                    for (int l = 0; l < nx; ++l)
                        for (int m = 0; m < ny; ++m)
                            for (int r = 0; r < nz; ++r)
                                acc = acc + Sx[i * nx + l] * Sy[j * ny + m] * Sz[k * nz + r]
                                            * p[((size_t)l * ny + m) * nz + r];
                    ve[((size_t)i * ny + j) * nz + k] = acc;
                }
    }
    free(p);
    free(q);
    return 0;
}

/* ------------------------------------------------------------------------------------------
 * Volume integral of the convective flux (Eq. 1 of the paper).  Per component c and element e
 * it is the sum over the three flux directions d of a tensor-product operator applied to the
 * metric-weighted flux of that direction, with the differentiation matrix along direction d and
 * the interpolation matrix along the other two:
 *
 *   F[c,e] = sum_{d=0,1,2}  ( A(d,2) (x) A(d,1) (x) A(d,0) )  ( M[e] .* P[c,d,e] ),
 *   A(d,a) = Dm if a == d, else Im.
 *
 * Cube axes are numbered from the FASTEST one: axis 0 is the last array index.  Written out,
 *   term_d[x2,x1,x0] = sum_{q2,q1,q0} A(d,2)[x2,q2] A(d,1)[x1,q1] A(d,0)[x0,q0] (M.*P_d)[q2,q1,q0].
 *
 * Dm, Im: [nv][nq] row-major (differentiation and interpolation from the nq quadrature points
 * to the nv nodes of one direction); M: [E][nq][nq][nq]; P: [3][3][E][nq][nq][nq] (component c,
 * direction d, element); F: [3][E][nv][nv][nv].
 *
 * _direct: each direction's six-deep sum on its own, the three results added in the order
 * d = 0, 1, 2.  _lifted: each term as three successive one-dimensional products (Sec. 2.2),
 * fastest axis first, the three terms added at the end. */
int tpo_oracle_convection_direct(const double *P, const double *M, const double *Dm,
                                 const double *Im, double *F, int nv, int nq, long long num_elems)
{
    if (nv < 1 || nq < 1 || nv > TPO_ORACLE_MAX_N || nq > TPO_ORACLE_MAX_N || num_elems < 0) return -1;
    if (num_elems == 0) return 0;
    if (!P || !M || !Dm || !Im || !F) return -1;
    const size_t qc = (size_t)nq * nq * nq, vc = (size_t)nv * nv * nv;
    for (int c = 0; c < 3; ++c)
        for (long long e = 0; e < num_elems; ++e) {
            const double *Me = M + (size_t)e * qc;
            double *Fe = F + ((size_t)c * num_elems + e) * vc;
            for (size_t x = 0; x < vc; ++x) Fe[x] = 0.0;
            for (int d = 0; d < 3; ++d) {
                const double *Pd = P + (((size_t)c * 3 + d) * num_elems + e) * qc;
                const double *A[3];                    /* operator along axis 0, 1, 2 */
                for (int a = 0; a < 3; ++a) A[a] = (a == d) ? Dm : Im;
                for (int x2 = 0; x2 < nv; ++x2)
                    for (int x1 = 0; x1 < nv; ++x1)
                        for (int x0 = 0; x0 < nv; ++x0) {
                            double term = 0.0;
                            for (int q2 = 0; q2 < nq; ++q2)
                                for (int q1 = 0; q1 < nq; ++q1)
                                    for (int q0 = 0; q0 < nq; ++q0) {
                                        const size_t q = ((size_t)q2 * nq + q1) * nq + q0;
                                        term = term + A[2][x2 * nq + q2] * A[1][x1 * nq + q1]
                                                      * A[0][x0 * nq + q0] * (Me[q] * Pd[q]);
                                    }
                            Fe[((size_t)x2 * nv + x1) * nv + x0] += term;
                        }
            }
        }
    return 0;
}

/* out[k,j,i] = sum_{n,m,l} A2[k,n] A1[j,m] A0[i,l] in[n,m,l], one axis at a time (fastest first);
 * tmp1, tmp2 hold nq*nq*nv and nq*nv*nv words. */
static void three_products(const double *A2, const double *A1, const double *A0, int nv, int nq,
                           const double *in, double *tmp1, double *tmp2, double *out)
{
    for (int n = 0; n < nq; ++n)
        for (int m = 0; m < nq; ++m)
            for (int i = 0; i < nv; ++i) {
                double acc = 0.0;
                for (int l = 0; l < nq; ++l) acc = acc + A0[i * nq + l] * in[((size_t)n * nq + m) * nq + l];
                tmp1[((size_t)n * nq + m) * nv + i] = acc;
            }
    for (int n = 0; n < nq; ++n)
        for (int j = 0; j < nv; ++j)
            for (int i = 0; i < nv; ++i) {
                double acc = 0.0;
                for (int m = 0; m < nq; ++m) acc = acc + A1[j * nq + m] * tmp1[((size_t)n * nq + m) * nv + i];
                tmp2[((size_t)n * nv + j) * nv + i] = acc;
            }
    for (int k = 0; k < nv; ++k)
        for (int j = 0; j < nv; ++j)
            for (int i = 0; i < nv; ++i) {
                double acc = 0.0;
                for (int n = 0; n < nq; ++n) acc = acc + A2[k * nq + n] * tmp2[((size_t)n * nv + j) * nv + i];
                out[((size_t)k * nv + j) * nv + i] = acc;
            }
}

int tpo_oracle_convection_lifted(const double *P, const double *M, const double *Dm,
                                 const double *Im, double *F, int nv, int nq, long long num_elems,
                                 int nthreads)
{
    if (nv < 1 || nq < 1 || nv > TPO_ORACLE_MAX_N || nq > TPO_ORACLE_MAX_N || num_elems < 0) return -1;
    if (num_elems == 0) return 0;
    if (!P || !M || !Dm || !Im || !F) return -1;
    const size_t qc = (size_t)nq * nq * nq, vc = (size_t)nv * nv * nv;
    const int big = nv > nq ? nv : nq;
    const size_t wc = (size_t)big * big * big;
    int failed = 0;
#ifdef _OPENMP
    if (nthreads <= 0) nthreads = omp_get_max_threads();
#else
    nthreads = 1;
#endif
#pragma omp parallel num_threads(nthreads)
    {
        double *w = (double *)malloc(6 * wc * sizeof(double));
        if (!w) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp barrier
        if (!failed) {
            double *in = w, *t1 = w + wc, *t2 = w + 2 * wc, *o0 = w + 3 * wc, *o1 = w + 4 * wc,
                   *o2 = w + 5 * wc;
#pragma omp for schedule(static) collapse(2)
            for (int c = 0; c < 3; ++c)
                for (long long e = 0; e < num_elems; ++e) {
                    const double *Me = M + (size_t)e * qc;
                    double *outs[3] = {o0, o1, o2};
                    for (int dir = 0; dir < 3; ++dir) {
                        const double *Pd = P + (((size_t)c * 3 + dir) * num_elems + e) * qc;
                        for (size_t x = 0; x < qc; ++x) in[x] = Me[x] * Pd[x];
                        three_products(dir == 2 ? Dm : Im, dir == 1 ? Dm : Im, dir == 0 ? Dm : Im,
                                       nv, nq, in, t1, t2, outs[dir]);
                    }
                    double *Fe = F + ((size_t)c * num_elems + e) * vc;
                    for (size_t x = 0; x < vc; ++x) Fe[x] = (o0[x] + o1[x]) + o2[x];
                }
        }
        free(w);
    }
    return failed ? -1 : 0;
}

int tpo_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

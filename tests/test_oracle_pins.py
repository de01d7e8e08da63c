"""Pins for the CPU oracle: each test checks ``oracle/`` against something the mathematics
fixes without calling the oracle's own formula again.

The paper prints no numeric example for this kernel (Table 2 holds times only), so every pin
is mathematical: the explicit Kronecker matrix, exact rational arithmetic on tiny inputs,
the orthogonal-S identity, the eigenvector property, a dense Helmholtz solve, linearity and
self-adjointness.  The last test plants the plausible mistakes (swapped axes, transposed
matrix, D indexed in the wrong order) into the *call* and shows the pins would catch them.
"""
from fractions import Fraction
from itertools import product

import numpy as np
import pytest

import oracle
from paper_2604_19906_amd import workloads as wl


def rand_inputs(n, e, seed, orthogonal=False):
    rng = np.random.default_rng(seed)
    if orthogonal:
        s = [wl.orthogonal_matrix(n, rng) for _ in range(3)]
    else:
        s = [rng.standard_normal((n, n)) for _ in range(3)]
    u = rng.uniform(-1, 1, (e, n, n, n))
    d = rng.uniform(0.05, 3.0, (e, n, n, n))
    return u, s[0], s[1], s[2], d


def kron_apply(u, sx, sy, sz, d):
    """Definition written with the explicit n^3 x n^3 matrix (row-major vec of the cube)."""
    e, n = u.shape[0], u.shape[1]
    m = np.kron(np.kron(sx, sy), sz)
    uf = u.reshape(e, -1)
    t = uf @ m                      # row e: (M^T u_e)^T
    g = d.reshape(e, -1) * t
    return (g @ m.T).reshape(e, n, n, n)


# --- p1: explicit Kronecker matrix ---------------------------------------------------------
@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 6])
def test_kronecker_small_n(n):
    u, sx, sy, sz, d = rand_inputs(n, 5, 1000 + n)
    ref = kron_apply(u, sx, sy, sz, d)
    got = oracle.ihelm_apply(u, sx, sy, sz, d)
    assert oracle.max_rel_err_per_element(got, ref) < 1e-13
    got_direct = oracle.ihelm_apply_direct(u, sx, sy, sz, d)
    assert oracle.max_rel_err_per_element(got_direct, ref) < 1e-13


def test_kronecker_config0_all_elements():
    w = wl.CONFIGS[0]
    u, sx, sy, sz, d = wl.make_inputs(w)
    ref = kron_apply(u, sx, sy, sz, d)
    got = oracle.ihelm_apply(u, sx, sy, sz, d)
    assert got.shape == (1000, 7, 7, 7)
    assert oracle.max_rel_err_per_element(got, ref) < 1e-13


def test_kronecker_three_distinct_matrices_n13():
    # the shape of the fp32 configuration, on a few elements
    w = wl.custom(13, 3, "f32", key=4, distinct_s=True)
    u, sx, sy, sz, d = wl.make_inputs(w)
    assert u.dtype == np.float32
    args = [a.astype(np.float64) for a in (u, sx, sy, sz, d)]
    ref = kron_apply(*args)
    got = oracle.ihelm_apply(u, sx, sy, sz, d)      # promoted inside
    assert oracle.max_rel_err_per_element(got, ref) < 1e-13


# --- exact rational arithmetic on a tiny case (brute force, no floating point) -------------
def test_exact_rational_n2():
    n = 2
    fr = Fraction
    sx = [[fr(1, 2), fr(-3, 4)], [fr(5, 8), fr(2)]]
    sy = [[fr(3), fr(1, 4)], [fr(-1, 2), fr(7, 8)]]
    sz = [[fr(-2), fr(3, 2)], [fr(1, 8), fr(-5, 4)]]
    u = [[[fr(a * 4 + b * 2 + c - 3, 2) for c in range(n)] for b in range(n)] for a in range(n)]
    d = [[[fr(1, 1 + a + 2 * b + 4 * c) for c in range(n)] for b in range(n)] for a in range(n)]
    idx = list(product(range(n), repeat=3))
    t = {}
    for (i, j, k) in idx:
        t[i, j, k] = sum(sx[l][i] * sy[m][j] * sz[q][k] * u[l][m][q] for (l, m, q) in idx)
    g = {x: d[x[0]][x[1]][x[2]] * t[x] for x in idx}
    v = {}
    for (i, j, k) in idx:
        v[i, j, k] = sum(sx[i][l] * sy[j][m] * sz[k][q] * g[l, m, q] for (l, m, q) in idx)
    # all inputs are dyadic or small fractions; convert exactly where possible
    f = lambda a: np.array(a, dtype=object).astype(np.float64)
    un, dn = f(u)[None], f(d)[None]
    got = oracle.ihelm_apply(un, f(sx), f(sy), f(sz), dn)[0]
    got_d = oracle.ihelm_apply_direct(un, f(sx), f(sy), f(sz), dn)[0]
    for x in idx:
        exact = float(v[x])
        assert got[x] == pytest.approx(exact, rel=1e-14, abs=1e-14)
        assert got_d[x] == pytest.approx(exact, rel=1e-14, abs=1e-14)


def test_n1_scalar_closed_form():
    # n = 1: every matrix is a scalar, v = sx^2 sy^2 sz^2 D u
    u = np.array([0.5, -2.0, 3.0]).reshape(3, 1, 1, 1)
    d = np.array([2.0, 0.25, 1.5]).reshape(3, 1, 1, 1)
    sx, sy, sz = np.array([[3.0]]), np.array([[-0.5]]), np.array([[2.0]])
    got = oracle.ihelm_apply(u, sx, sy, sz, d)
    assert np.allclose(got.ravel(), 9.0 * 0.25 * 4.0 * d.ravel() * u.ravel(), rtol=1e-15)


# --- p2: orthogonal S and constant D give a multiple of the identity -----------------------
@pytest.mark.parametrize("n", [2, 7, 8, 11, 16])
def test_orthogonal_identity(n):
    u, sx, sy, sz, _ = rand_inputs(n, 4, 2000 + n, orthogonal=True)
    one = np.ones_like(u)
    assert oracle.max_rel_err_per_element(oracle.ihelm_apply(u, sx, sy, sz, one), u) < 1e-13
    c = 0.375
    got = oracle.ihelm_apply(u, sx, sy, sz, c * one)
    assert oracle.max_rel_err_per_element(got, c * u) < 1e-13


# --- p3: linearity in u and in D; no leakage between elements -------------------------------
def test_linearity_and_element_independence():
    n = 6
    u, sx, sy, sz, d = rand_inputs(n, 6, 3000)
    rng = np.random.default_rng(7)
    y = rng.standard_normal(u.shape)
    d2 = rng.uniform(0.1, 1.0, d.shape)
    al, be = 1.75, -0.625
    a = lambda uu, dd: oracle.ihelm_apply(uu, sx, sy, sz, dd)
    lhs = a(al * u + be * y, d)
    rhs = al * a(u, d) + be * a(y, d)
    assert oracle.max_rel_err_per_element(lhs, rhs) < 1e-13
    lhs = a(u, al * d + be * d2)
    rhs = al * a(u, d) + be * a(u, d2)
    assert oracle.max_rel_err_per_element(lhs, rhs) < 1e-12
    # p9: a permuted / subset batch gives the permuted / subset result bit for bit
    perm = np.array([4, 0, 5, 2])
    full = a(u, d)
    part = a(u[perm], d[perm])
    assert np.array_equal(part, full[perm])
    assert np.array_equal(a(u, d, ), oracle.ihelm_apply(u, sx, sy, sz, d, nthreads=1))


# --- p4: unlifted six-deep sums equal the lifted form (Sec. 5.2) ----------------------------
@pytest.mark.parametrize("n", [3, 7, 8])
def test_direct_equals_lifted(n):
    u, sx, sy, sz, d = rand_inputs(n, 2, 4000 + n)
    a = oracle.ihelm_apply(u, sx, sy, sz, d)
    b = oracle.ihelm_apply_direct(u, sx, sy, sz, d)
    assert oracle.max_rel_err_per_element(a, b) < 1e-13


# --- p5: eigenvector property, three distinct non-symmetric orthogonal matrices ------------
@pytest.mark.parametrize("n", [3, 5, 11])
def test_eigenvector_property(n):
    _, sx, sy, sz, d = rand_inputs(n, 1, 5000 + n, orthogonal=True)
    assert not np.allclose(sx, sx.T)
    picks = [(0, 1, 2), (n - 1, 0, 1), (1, n - 1, n - 2), (2, 2, 0)]
    u = np.stack([np.einsum("i,j,k->ijk", sx[:, a], sy[:, b], sz[:, c]) for a, b, c in picks])
    dd = np.repeat(d, len(picks), axis=0)
    v = oracle.ihelm_apply(u, sx, sy, sz, dd)
    for e, (a, b, c) in enumerate(picks):
        assert np.allclose(v[e], d[0, a, b, c] * u[e], rtol=0, atol=1e-13)


# --- p6: rank-1 closed form of the forward half ---------------------------------------------
def test_forward_rank_one():
    n = 5
    rng = np.random.default_rng(6000)
    sx, sy, sz = (rng.standard_normal((n, n)) for _ in range(3))
    a, b, c = (rng.standard_normal(n) for _ in range(3))
    u = np.einsum("i,j,k->ijk", a, b, c)[None]
    t = oracle.forward(u, sx, sy, sz)[0]
    ref = np.einsum("i,j,k->ijk", sx.T @ a, sy.T @ b, sz.T @ c)
    assert np.allclose(t, ref, rtol=0, atol=1e-13 * np.abs(ref).max())
    # each axis on its own: identity on the other two
    eye = np.eye(n)
    x = rng.standard_normal((1, n, n, n))
    assert np.allclose(oracle.forward(x, sx, eye, eye)[0], np.einsum("li,lbc->ibc", sx, x[0]))
    assert np.allclose(oracle.forward(x, eye, sy, eye)[0], np.einsum("mj,amc->ajc", sy, x[0]))
    assert np.allclose(oracle.forward(x, eye, eye, sz)[0], np.einsum("qk,abq->abk", sz, x[0]))


# --- p7: self-adjoint and positive definite for D > 0 ---------------------------------------
def test_symmetric_positive():
    n = 4
    u, sx, sy, sz, d = rand_inputs(n, 1, 7000)
    rng = np.random.default_rng(7001)
    y = rng.standard_normal(u.shape)
    au = oracle.ihelm_apply(u, sx, sy, sz, d)
    ay = oracle.ihelm_apply(y, sx, sy, sz, d)
    assert np.vdot(y, au) == pytest.approx(np.vdot(ay, u), rel=1e-12)
    assert np.vdot(u, au) > 0


# --- p8: it is the inverse of a Helmholtz operator (fast diagonalisation) -------------------
@pytest.mark.parametrize("n", [2, 3, 4])
def test_inverse_helmholtz_dense_solve(n):
    rng = np.random.default_rng(8000 + n)
    s = [wl.orthogonal_matrix(n, rng) for _ in range(3)]
    lam = [rng.uniform(0.1, 10, n) for _ in range(3)]
    mu = 0.37
    k = [s[a] @ np.diag(lam[a]) @ s[a].T for a in range(3)]
    eye = np.eye(n)
    h = (np.kron(np.kron(k[0], eye), eye) + np.kron(np.kron(eye, k[1]), eye)
         + np.kron(np.kron(eye, eye), k[2]) + mu * np.eye(n ** 3))
    u = rng.uniform(-1, 1, (1, n, n, n))
    d = 1.0 / (lam[0][:, None, None] + lam[1][None, :, None] + lam[2][None, None, :] + mu)
    v = oracle.ihelm_apply(u, s[0], s[1], s[2], d[None])
    ref = np.linalg.solve(h, u.ravel()).reshape(n, n, n)
    assert np.allclose(v[0], ref, rtol=0, atol=1e-12 * np.abs(ref).max())


def test_workload_diagonal_matches_helmholtz_recipe():
    # the generator's D is the fast-diagonalisation diagonal of its own lam and mu
    w = wl.custom(4, 3, "f64", key=9)
    u, sx, sy, sz, d = wl.make_inputs(w)
    lx, ly, lz = wl.eigenvalues(w)
    mu = wl.shifts(w)
    for e in range(3):
        assert d[e, 1, 2, 3] == pytest.approx(1.0 / (lx[1] + ly[2] + lz[3] + mu[e]), rel=1e-15)
    assert d.min() > 1 / 31.0 and d.max() < 1 / 0.3


# --- p6b: the two halves on their own ---------------------------------------------------------
@pytest.mark.parametrize("n", [1, 2, 3, 5])
def test_transform_halves_against_kronecker(n):
    u, sx, sy, sz, _ = rand_inputs(n, 3, 6100 + n)
    m = np.kron(np.kron(sx, sy), sz)
    uf = u.reshape(3, -1)
    fwd = (uf @ m).reshape(u.shape)          # rows: (M^T u_e)^T
    bwd = (uf @ m.T).reshape(u.shape)        # rows: (M u_e)^T
    assert np.allclose(oracle.forward(u, sx, sy, sz), fwd, rtol=0, atol=1e-13 * np.abs(fwd).max())
    assert np.allclose(oracle.backward(u, sx, sy, sz), bwd, rtol=0, atol=1e-13 * np.abs(bwd).max())
    # with three different non-symmetric matrices the two halves differ: a transposed matrix
    # or swapped roles cannot pass both
    if n > 1:
        assert oracle.max_rel_err_per_element(oracle.backward(u, sx, sy, sz), fwd) > 1e-2


def test_transform_halves_compose_to_the_operator():
    n = 4
    u, sx, sy, sz, d = rand_inputs(n, 5, 6200)
    whole = oracle.ihelm_apply(u, sx, sy, sz, d)
    parts = oracle.backward(d * oracle.forward(u, sx, sy, sz), sx, sy, sz)
    assert np.array_equal(whole, parts)       # same routine, same order of operations
    q = [wl.orthogonal_matrix(n, np.random.default_rng(6300 + a)) for a in range(3)]
    back = oracle.backward(oracle.forward(u, *q), *q)
    assert np.allclose(back, u, rtol=0, atol=1e-14)


# --- p6c: anisotropic elements ----------------------------------------------------------------
@pytest.mark.parametrize("dims", [(1, 2, 3), (2, 3, 4), (4, 2, 3), (3, 3, 2), (5, 1, 4)])
def test_aniso_against_kronecker(dims):
    nx, ny, nz = dims
    rng = np.random.default_rng(6400 + 100 * nx + 10 * ny + nz)
    sx, sy, sz = (rng.standard_normal((n, n)) for n in dims)
    u = rng.uniform(-1, 1, (3, nx, ny, nz))
    d = rng.uniform(0.05, 3.0, u.shape)
    m = np.kron(np.kron(sx, sy), sz)                 # axis 0 <-> S_x (slowest), axis 2 <-> S_z
    ref = ((d.reshape(3, -1) * (u.reshape(3, -1) @ m)) @ m.T).reshape(u.shape)
    for direct in (False, True):
        got = oracle.ihelm_apply_aniso(u, sx, sy, sz, d, direct=direct)
        assert np.allclose(got, ref, rtol=0, atol=1e-12 * np.abs(ref).max())
    # matrices handed to the wrong axes must not pass: shapes forbid most swaps, equal sizes not
    if nx == ny:
        assert oracle.max_rel_err_per_element(oracle.ihelm_apply_aniso(u, sy, sx, sz, d), ref) > 1e-2


def test_aniso_reduces_to_the_cubic_operator():
    u, sx, sy, sz, d = rand_inputs(4, 3, 6500)
    assert np.array_equal(oracle.ihelm_apply_aniso(u, sx, sy, sz, d), oracle.ihelm_apply(u, sx, sy, sz, d))
    with pytest.raises(ValueError):
        oracle.ihelm_apply_aniso(u, sx, sy[:3, :3], sz, d)


# --- p9: separable-diagonal form --------------------------------------------------------------
def helmholtz_matrix(s, lam, mu):
    """Dense (A_x (x) I (x) I + I (x) A_y (x) I + I (x) I (x) A_z + mu I), A_d = S_d diag(lam_d) S_d^T."""
    n = s[0].shape[0]
    k = [s[a] @ np.diag(lam[a]) @ s[a].T for a in range(3)]
    eye = np.eye(n)
    return (np.kron(np.kron(k[0], eye), eye) + np.kron(np.kron(eye, k[1]), eye)
            + np.kron(np.kron(eye, eye), k[2]) + mu * np.eye(n ** 3))


@pytest.mark.parametrize("n", [1, 2, 3, 4, 5])
def test_sep_dense_helmholtz_solve(n):
    # three different operators, different eigenvalues per direction, a different shift per
    # element: a swapped lam_x/lam_z, a missing mu or mu indexed by the wrong element fails
    rng = np.random.default_rng(8100 + n)
    s = [wl.orthogonal_matrix(n, rng) for _ in range(3)]
    lam = [rng.uniform(0.1, 10, n) for _ in range(3)]
    mu = rng.uniform(0, 1, 3)
    u = rng.uniform(-1, 1, (3, n, n, n))
    v = oracle.ihelm_apply_sep(u, s[0], s[1], s[2], lam[0], lam[1], lam[2], mu)
    for e in range(3):
        ref = np.linalg.solve(helmholtz_matrix(s, lam, mu[e]), u[e].ravel()).reshape(n, n, n)
        assert np.allclose(v[e], ref, rtol=0, atol=1e-12 * np.abs(ref).max())


def test_sep_is_the_d_form_with_the_definition_of_d():
    # entry by entry: D[e,i,j,k] = 1 / (lam_x[i] + lam_y[j] + lam_z[k] + mu[e]), built here with
    # explicit loops, given to the D form; 1100 elements cross the oracle's block of 1024
    n, e = 3, 1100
    rng = np.random.default_rng(8200)
    s = [rng.standard_normal((n, n)) for _ in range(3)]
    lam = [rng.uniform(0.1, 10, n) for _ in range(3)]
    mu = rng.uniform(0, 1, e)
    u = rng.uniform(-1, 1, (e, n, n, n))
    d = np.empty((e, n, n, n))
    for ee in range(e):
        for i, j, k in product(range(n), repeat=3):
            d[ee, i, j, k] = 1.0 / (lam[0][i] + lam[1][j] + lam[2][k] + mu[ee])
    got = oracle.ihelm_apply_sep(u, s[0], s[1], s[2], lam[0], lam[1], lam[2], mu)
    ref = oracle.ihelm_apply(u, s[0], s[1], s[2], d)
    assert np.array_equal(got, ref)


def test_sep_planted_mistakes():
    n = 4
    rng = np.random.default_rng(8300)
    s = [wl.orthogonal_matrix(n, rng) for _ in range(3)]
    lam = [rng.uniform(0.1, 10, n) for _ in range(3)]
    mu = rng.uniform(0, 1, 2)
    u = rng.uniform(-1, 1, (2, n, n, n))
    ref = np.stack([np.linalg.solve(helmholtz_matrix(s, lam, mu[e]), u[e].ravel()).reshape(n, n, n)
                    for e in range(2)])
    err = lambda got: oracle.max_rel_err_per_element(got, ref)
    assert err(oracle.ihelm_apply_sep(u, *s, *lam, mu)) < 1e-12
    assert err(oracle.ihelm_apply_sep(u, *s, lam[2], lam[1], lam[0], mu)) > 1e-3   # lam_x <-> lam_z
    assert err(oracle.ihelm_apply_sep(u, *s, *lam, mu[::-1])) > 1e-4               # wrong element's mu
    assert err(oracle.ihelm_apply_sep(u, *s, *lam, np.zeros(2))) > 1e-4            # dropped mu


def test_sep_argument_checks():
    n = 3
    rng = np.random.default_rng(8400)
    s = rng.standard_normal((n, n))
    lam = rng.uniform(1, 2, n)
    u = rng.uniform(-1, 1, (2, n, n, n))
    with pytest.raises(ValueError):
        oracle.ihelm_apply_sep(u, s, s, s, lam[:2], lam, lam, np.zeros(2))
    with pytest.raises(ValueError):
        oracle.ihelm_apply_sep(u, s, s, s, lam, lam, lam, np.zeros(3))
    assert oracle.ihelm_apply_sep(u[:0], s, s, s, lam, lam, lam, np.zeros(0)).shape == (0, n, n, n)


# --- planted mistakes are caught -------------------------------------------------------------
def test_pins_detect_planted_mistakes():
    n = 4
    u, sx, sy, sz, d = rand_inputs(n, 2, 9000, orthogonal=True)
    ref = kron_apply(u, sx, sy, sz, d)
    err = lambda got: oracle.max_rel_err_per_element(got, ref)
    assert err(oracle.ihelm_apply(u, sx, sy, sz, d)) < 1e-13
    # axes paired with the wrong matrices
    assert err(oracle.ihelm_apply(u, sz, sy, sx, d)) > 1e-2
    assert err(oracle.ihelm_apply(u, sy, sx, sz, d)) > 1e-2
    # transposed matrices (forward/backward roles swapped)
    assert err(oracle.ihelm_apply(u, sx.T, sy.T, sz.T, d)) > 1e-2
    # D indexed with axes reversed; cube read with axes reversed
    assert err(oracle.ihelm_apply(u, sx, sy, sz, d.transpose(0, 3, 2, 1))) > 1e-2
    assert err(oracle.ihelm_apply(u.transpose(0, 3, 2, 1), sx, sy, sz, d)) > 1e-2
    # a dropped diagonal
    assert err(oracle.ihelm_apply(u, sx, sy, sz, np.ones_like(d))) > 1e-2


def test_error_metric():
    a = np.zeros((2, 2, 2, 2))
    b = np.zeros((2, 2, 2, 2))
    b[0] = 2.0
    a[0] = 2.0
    a[0, 0, 0, 0] = 2.5
    b[1, 0, 0, 0] = 4.0
    a[1, 0, 0, 0] = 4.0
    assert oracle.max_rel_err_per_element(a, b) == pytest.approx(0.25)
    assert oracle.max_rel_err_per_element(b, b) == 0.0
    assert oracle.max_rel_err_per_element(a[:0], b[:0]) == 0.0


def test_oracle_argument_checks():
    u, sx, sy, sz, d = rand_inputs(3, 2, 1)
    with pytest.raises(ValueError):
        oracle.ihelm_apply(u, sx[:2], sy, sz, d)
    with pytest.raises(ValueError):
        oracle.ihelm_apply(u, sx, sy, sz, d[:1])
    assert oracle.ihelm_apply(u[:0], sx, sy, sz, d[:0]).shape == (0, 3, 3, 3)


def test_golden_regression(repo_root):
    import os
    path = os.path.join(repo_root, "tests", "golden", "ihelm_f64_n3_E2.txt")
    want = np.array([float.fromhex(l) for l in open(path) if not l.startswith("#")])
    w = wl.custom(3, 2, "f64", key=77)
    got = oracle.ihelm_apply(*wl.make_inputs(w))
    assert np.array_equal(got.ravel(), want)

"""Pins for the oracle's convection volume term (Eq. 1 of the paper): the explicit Kronecker
matrices, exact derivatives of polynomials, the equivalent NumPy index expression, the six-deep
sums, and planted mistakes.  The paper prints no numbers for this kernel either."""
import numpy as np
import pytest

import oracle


def rand_case(nv, nq, e, seed):
    rng = np.random.default_rng(seed)
    return (rng.uniform(-1, 1, (3, 3, e, nq, nq, nq)), rng.uniform(0.5, 2.0, (e, nq, nq, nq)),
            rng.standard_normal((nv, nq)), rng.standard_normal((nv, nq)))


def kron_reference(p, m, d, i):
    """Eq. 1 with its three operators written out as (nv^3 x nq^3) matrices acting on the
    row-major flattening [n,m,l] -> [k,j,i]: the first factor of each Kronecker product pairs
    with the slowest axis."""
    ops = [np.kron(np.kron(i, i), d), np.kron(np.kron(i, d), i), np.kron(np.kron(d, i), i)]
    nv = d.shape[0]
    e = m.shape[0]
    f = np.zeros((3, e, nv, nv, nv))
    for c in range(3):
        for ee in range(e):
            acc = np.zeros(nv ** 3)
            for t in range(3):
                acc += ops[t] @ (m[ee] * p[c, t, ee]).ravel()
            f[c, ee] = acc.reshape(nv, nv, nv)
    return f


@pytest.mark.parametrize("nv,nq", [(1, 1), (2, 2), (3, 3), (4, 4), (2, 3), (4, 3), (3, 5)])
def test_convection_kronecker(nv, nq):
    p, m, d, i = rand_case(nv, nq, 2, 100 * nv + nq)
    ref = kron_reference(p, m, d, i)
    for direct in (False, True):
        got = oracle.convection_apply(p, m, d, i, direct=direct)
        assert np.allclose(got, ref, rtol=0, atol=1e-12 * np.abs(ref).max())


def test_convection_matches_the_index_expression():
    # the paper's index form, spelled with einsum: F[c,e,k,j,i] over P[c,dir,e,n,m,l]
    p, m, d, i = rand_case(4, 5, 3, 77)
    mp = m[None, None] * p
    ref = (np.einsum("il,jm,kn,cenml->cekji", d, i, i, mp[:, 0])
           + np.einsum("il,jm,kn,cenml->cekji", i, d, i, mp[:, 1])
           + np.einsum("il,jm,kn,cenml->cekji", i, i, d, mp[:, 2]))
    got = oracle.convection_apply(p, m, d, i)
    assert np.allclose(got, ref, rtol=0, atol=1e-13 * np.abs(ref).max())


def diff_matrix(x):
    """Differentiation matrix of the Lagrange basis on nodes x (barycentric form)."""
    n = len(x)
    w = np.array([1.0 / np.prod([x[a] - x[b] for b in range(n) if b != a]) for a in range(n)])
    d = np.zeros((n, n))
    for a in range(n):
        for b in range(n):
            if a != b:
                d[a, b] = w[b] / w[a] / (x[a] - x[b])
        d[a, a] = -d[a].sum()
    return d


def test_convection_is_a_divergence_of_polynomials():
    # collocation (I = identity), M = 1, D = exact differentiation on the nodes: for polynomial
    # fluxes the result is d/dx_fast P0 + d/dx_mid P1 + d/dx_slow P2 at the nodes, exactly.
    n = 6
    x = np.cos(np.pi * np.arange(n) / (n - 1))[::-1].copy()
    d = diff_matrix(x)
    eye = np.eye(n)
    zs, ys, xs = np.meshgrid(x, x, x, indexing="ij")      # axes [n(slow), m, l(fast)]
    p = np.zeros((3, 3, 1, n, n, n))
    want = np.zeros((3, 1, n, n, n))
    # component 0: P0 = xf^3 * ys, P1 = xf * ym^2, P2 = zs^4 + xf
    p[0, 0, 0] = xs ** 3 * ys
    p[0, 1, 0] = xs * ys ** 2
    p[0, 2, 0] = zs ** 4 + xs
    want[0, 0] = 3 * xs ** 2 * ys + 2 * xs * ys + 4 * zs ** 3
    # component 1: only the mid-axis term; component 2: only the slow-axis term
    p[1, 1, 0] = ys ** 5 * zs
    want[1, 0] = 5 * ys ** 4 * zs
    p[2, 2, 0] = xs * ys * zs ** 2
    want[2, 0] = 2 * xs * ys * zs
    got = oracle.convection_apply(p, np.ones((1, n, n, n)), d, eye)
    assert np.allclose(got, want, rtol=0, atol=1e-11)
    # the metric factor multiplies the flux before differentiation: M = xf  =>  d/dxf (xf * P0)
    p2 = np.zeros_like(p)
    p2[0, 0, 0] = xs ** 2
    got2 = oracle.convection_apply(p2, xs[None].copy(), d, eye)
    assert np.allclose(got2[0, 0], 3 * xs ** 2, rtol=0, atol=1e-11)


def test_convection_planted_mistakes():
    p, m, d, i = rand_case(3, 3, 2, 5)
    ref = kron_reference(p, m, d, i)
    err = lambda got: np.abs(got - ref).max() / np.abs(ref).max()
    assert err(oracle.convection_apply(p, m, d, i)) < 1e-13
    assert err(oracle.convection_apply(p, m, i, d)) > 1e-2                     # D and I swapped
    assert err(oracle.convection_apply(p, m, d.T.copy(), i.T.copy())) > 1e-2   # transposed matrices
    assert err(oracle.convection_apply(p[:, ::-1].copy(), m, d, i)) > 1e-2     # directions reversed
    assert err(oracle.convection_apply(p.transpose(1, 0, 2, 3, 4, 5).copy(), m, d, i)) > 1e-2
    assert err(oracle.convection_apply(p, np.ones_like(m), d, i)) > 1e-2       # dropped metric


def test_convection_linearity_and_shapes():
    p, m, d, i = rand_case(3, 4, 2, 9)
    q = np.random.default_rng(10).uniform(-1, 1, p.shape)
    a = oracle.convection_apply(p + 2 * q, m, d, i)
    b = oracle.convection_apply(p, m, d, i) + 2 * oracle.convection_apply(q, m, d, i)
    assert np.allclose(a, b, rtol=0, atol=1e-12 * np.abs(b).max())
    assert oracle.convection_apply(p[:, :, :0], m[:0], d, i).shape == (3, 0, 3, 3, 3)
    with pytest.raises(ValueError):
        oracle.convection_apply(p, m, d, i[:, :3])
    with pytest.raises(ValueError):
        oracle.convection_apply(p[:2], m, d, i)


def test_convection_golden_regression(repo_root):
    import os
    from paper_2604_19906_amd import workloads as wl
    path = os.path.join(repo_root, "tests", "golden", "convection_f64_nv3_nq4_E2.txt")
    want = np.array([float.fromhex(l) for l in open(path) if not l.startswith("#")])
    got = oracle.convection_apply(*wl.conv_inputs(wl.conv_custom(3, 2, "f64", key=78, nq=4)))
    assert np.array_equal(got.ravel(), want)

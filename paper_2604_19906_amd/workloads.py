"""Seeded synthetic inputs for the batched inverse-Helmholtz tensor-product operator.

This module only *draws inputs*: direction matrices, eigenvalue vectors, per-element shifts,
fields and the diagonal they define.  It holds none of the operator's arithmetic (no mode
product, no Kronecker product), so both the CPU oracle's tests and the GPU path's tests may
import it without sharing any part of the method.

The paper's own workload is a set of spectral elements taken from a Fortran DG-SEM code
(Sec. 6.1: 8192 elements per run); that data is not public, so the inputs here stand in for
it with the same structure: many independent elements, one small dense matrix per direction
shared by all elements, and one strictly positive diagonal cube per element.

Layout: every field is C-contiguous ``[E, n, n, n]`` (element-major, axis 2 fastest); every
direction matrix is row-major ``[n, n]``.  Axis 0 pairs with ``S_x``/``lam_x``, axis 1 with
``S_y``/``lam_y`` and axis 2 with ``S_z``/``lam_z``.

Fields are drawn in blocks of ``BLOCK`` elements, block ``b`` from its own seed, so that any
block of a multi-gigabyte field can be regenerated on its own.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Iterator, Tuple

import numpy as np

BASE_SEED = 19906
BLOCK = 4096

# stream ids below the (BASE_SEED, config) key
_STREAM_S, _STREAM_LAM, _STREAM_MU, _STREAM_U = 0, 1, 2, 3


@dataclass(frozen=True)
class Workload:
    """One synthetic configuration (shape, precision and value distributions)."""

    name: str
    index: int          # seed key; 0..4 are the five named configurations
    dtype: str          # "f64" or "f32"
    n: int              # points per direction (polynomial degree + 1)
    num_elems: int
    u_dist: str         # "uniform" -> U(-1,1), "normal" -> N(0,1)
    distinct_s: bool    # three different direction matrices (and eigenvalue vectors)

    @property
    def np_dtype(self):
        return np.float64 if self.dtype == "f64" else np.float32

    @property
    def word(self) -> int:
        return 8 if self.dtype == "f64" else 4

    @property
    def cube(self) -> int:
        return self.n ** 3

    @property
    def flop_per_elem(self) -> int:
        # six mode products of 2 n^4 flop each plus the n^3 diagonal multiplies
        return 12 * self.n ** 4 + self.n ** 3

    @property
    def bytes_per_elem(self) -> int:
        # read u_e, read D_e, write v_e
        return 3 * self.cube * self.word


CONFIGS = (
    Workload("cfg0_f64_n7_E1000", 0, "f64", 7, 1000, "uniform", False),
    Workload("cfg1_f64_n8_E131072", 1, "f64", 8, 131072, "uniform", False),
    Workload("cfg2_f64_n11_E262144", 2, "f64", 11, 262144, "normal", False),
    Workload("cfg3_f64_n16_E65536", 3, "f64", 16, 65536, "uniform", False),
    Workload("cfg4_f32_n13_E1048576", 4, "f32", 13, 1048576, "uniform", True),
)


def custom(n: int, num_elems: int, dtype: str = "f64", *, key: int = 100,
           u_dist: str = "uniform", distinct_s: bool = True) -> Workload:
    """A workload of arbitrary shape for edge-case tests (``key`` selects the seed)."""
    return Workload(f"custom_{dtype}_n{n}_E{num_elems}_k{key}", key, dtype, n, num_elems,
                    u_dist, distinct_s)


def _rng(*key: int) -> np.random.Generator:
    return np.random.default_rng(np.random.SeedSequence([BASE_SEED, *key]))


def orthogonal_matrix(n: int, rng: np.random.Generator) -> np.ndarray:
    """Haar-distributed ``n x n`` orthogonal matrix: Q of a Gaussian's QR with the signs of
    R's diagonal folded in.  Deterministic for a given generator state; not symmetric."""
    g = rng.standard_normal((n, n))
    q, r = np.linalg.qr(g)
    sgn = np.sign(np.diag(r))
    sgn[sgn == 0] = 1.0
    return np.ascontiguousarray(q * sgn[None, :])


def direction_matrices(w: Workload) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """``(S_x, S_y, S_z)`` in the workload's dtype.  When the workload shares one matrix the
    three returned arrays are the same object."""
    rng = _rng(w.index, _STREAM_S)
    if w.distinct_s:
        mats = [orthogonal_matrix(w.n, rng).astype(w.np_dtype) for _ in range(3)]
        return mats[0], mats[1], mats[2]
    s = orthogonal_matrix(w.n, rng).astype(w.np_dtype)
    return s, s, s


def eigenvalues(w: Workload) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """``(lam_x, lam_y, lam_z)``, each ``[n]`` fp64 drawn from U(0.1, 10); one vector per
    direction shared by all elements (the same vector three times if S is shared)."""
    rng = _rng(w.index, _STREAM_LAM)
    if w.distinct_s:
        lams = [rng.uniform(0.1, 10.0, w.n) for _ in range(3)]
        return lams[0], lams[1], lams[2]
    lam = rng.uniform(0.1, 10.0, w.n)
    return lam, lam, lam


def shifts(w: Workload, start: int = 0, stop: int | None = None) -> np.ndarray:
    """Per-element shift ``mu_e`` ~ U(0,1), fp64, for elements ``start..stop-1``."""
    stop = w.num_elems if stop is None else stop
    out = np.empty(stop - start, dtype=np.float64)
    for b, lo, hi in _blocks(start, stop):
        mu_b = _rng(w.index, _STREAM_MU, b).uniform(0.0, 1.0, BLOCK)
        out[lo - start:hi - start] = mu_b[lo - b * BLOCK:hi - b * BLOCK]
    return out


def _blocks(start: int, stop: int) -> Iterator[Tuple[int, int, int]]:
    """Yield ``(block id, lo, hi)`` for the parts of ``[start, stop)`` in each seed block."""
    b = start // BLOCK
    while b * BLOCK < stop:
        lo = max(start, b * BLOCK)
        hi = min(stop, (b + 1) * BLOCK)
        if hi > lo:
            yield b, lo, hi
        b += 1


def field_u(w: Workload, start: int = 0, stop: int | None = None) -> np.ndarray:
    """Input field ``u[start:stop]`` of shape ``[stop-start, n, n, n]`` in the workload's
    dtype.  Values are drawn in fp64 and rounded once."""
    stop = w.num_elems if stop is None else stop
    n = w.n
    out = np.empty((stop - start, n, n, n), dtype=w.np_dtype)
    for b, lo, hi in _blocks(start, stop):
        rng = _rng(w.index, _STREAM_U, b)
        # draw only as many elements of the block as are needed, always from its start
        cnt = hi - b * BLOCK
        if w.u_dist == "normal":
            blk = rng.standard_normal((cnt, n, n, n))
        else:
            blk = rng.uniform(-1.0, 1.0, (cnt, n, n, n))
        out[lo - start:hi - start] = blk[lo - b * BLOCK:]
    return out


def diagonal_d(w: Workload, start: int = 0, stop: int | None = None) -> np.ndarray:
    """Diagonal ``D[e,i,j,k] = 1 / (lam_x[i] + lam_y[j] + lam_z[k] + mu_e)`` for elements
    ``start..stop-1``, evaluated in fp64 and rounded once to the workload's dtype.  This is
    the input recipe of the workloads (an input, not a step of the operator)."""
    stop = w.num_elems if stop is None else stop
    lx, ly, lz = eigenvalues(w)
    mu = shifts(w, start, stop)
    lam3 = lx[:, None, None] + ly[None, :, None] + lz[None, None, :]
    out = np.empty((stop - start, w.n, w.n, w.n), dtype=w.np_dtype)
    step = 2048
    for lo in range(0, stop - start, step):
        hi = min(stop - start, lo + step)
        out[lo:hi] = 1.0 / (lam3[None] + mu[lo:hi, None, None, None])
    return out


def sep_inputs(w: Workload, start: int = 0, stop: int | None = None):
    """``(lam_x, lam_y, lam_z, mu)`` for elements ``start..stop-1`` in the workload's dtype:
    the numbers the separable-diagonal form takes instead of ``D`` (each rounded once from
    fp64; a shared eigenvalue vector is returned three times as the same array)."""
    lx, ly, lz = eigenvalues(w)
    mu = shifts(w, start, stop).astype(w.np_dtype)
    if lx is ly and ly is lz:
        lam = lx.astype(w.np_dtype)
        return lam, lam, lam, mu
    return lx.astype(w.np_dtype), ly.astype(w.np_dtype), lz.astype(w.np_dtype), mu


def make_inputs(w: Workload, start: int = 0, stop: int | None = None):
    """``(u, S_x, S_y, S_z, D)`` for elements ``start..stop-1`` as host arrays."""
    sx, sy, sz = direction_matrices(w)
    return field_u(w, start, stop), sx, sy, sz, diagonal_d(w, start, stop)


def to_device(w: Workload, threads: int = 12, chunk: int = 2 * BLOCK, with_d: bool = True):
    """Device tensors ``(u, S_x, S_y, S_z, D)`` of a whole workload on the current GPU
    (``(u, S_x, S_y, S_z)`` with ``with_d=False``, for the separable-diagonal form).
    Fields are generated block by block on the host (each block from its own seed, several
    blocks at a time) and copied into place, so host memory stays small even for fields of
    many gigabytes.  A shared matrix is uploaded once and returned three times."""
    from concurrent.futures import ThreadPoolExecutor

    import torch

    e, n = w.num_elems, w.n
    tdtype = torch.float64 if w.dtype == "f64" else torch.float32
    tu = torch.empty((e, n, n, n), dtype=tdtype, device="cuda")
    td = torch.empty((e, n, n, n), dtype=tdtype, device="cuda") if with_d else None
    spans = [(lo, min(e, lo + chunk)) for lo in range(0, e, chunk)]

    def gen(span):
        lo, hi = span
        return lo, hi, field_u(w, lo, hi), (diagonal_d(w, lo, hi) if with_d else None)

    with ThreadPoolExecutor(max_workers=threads) as ex:
        for lo, hi, hu, hd in ex.map(gen, spans):
            tu[lo:hi].copy_(torch.from_numpy(hu))
            if with_d:
                td[lo:hi].copy_(torch.from_numpy(hd))
    sx, sy, sz = direction_matrices(w)
    up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    if sx is sy and sy is sz:
        ts = up(sx)
        mats = (ts, ts, ts)
    else:
        mats = (up(sx), up(sy), up(sz))
    return (tu, *mats, td) if with_d else (tu, *mats)


# ------------------------------------------------------------------------------------------
# Inputs of the convection volume term (Eq. 1 of the paper).  The paper's own inputs come
# from a flow solver that is not available; these stand in for them: realistic one-dimensional
# operators, a positive metric factor, uniformly distributed fluxes.

@dataclass(frozen=True)
class ConvWorkload:
    """One synthetic configuration of the convection volume term: ``n`` nodes and ``q``
    quadrature points per direction (``nq = 0`` means as many as nodes)."""

    name: str
    index: int          # seed key, disjoint from the inverse-Helmholtz configurations
    dtype: str
    n: int
    num_elems: int
    nq: int = 0

    @property
    def q(self) -> int:
        return self.nq or self.n

    @property
    def np_dtype(self):
        return np.float64 if self.dtype == "f64" else np.float32

    @property
    def word(self) -> int:
        return 8 if self.dtype == "f64" else 4

    @property
    def bytes_per_elem(self) -> int:
        """Algorithmic traffic per element: nine flux cubes and the metric in, three cubes out."""
        return (10 * self.q ** 3 + 3 * self.n ** 3) * self.word

    @property
    def flop_per_elem(self) -> int:
        """Eight mode products per component (sum-factorised, terms merged) plus the metric
        scale and the two merges."""
        n, q = self.n, self.q
        return 3 * (6 * q ** 3 * n + 6 * q ** 2 * n ** 2 + 4 * q * n ** 3 + 3 * q ** 3 + 2 * n ** 3)


CONV_CONFIGS = (
    ConvWorkload("conv0_f64_n7_E512", 20, "f64", 7, 512),
    ConvWorkload("conv1_f64_n11_E32768", 21, "f64", 11, 32768),
    ConvWorkload("conv2_f32_n13_E65536", 22, "f32", 13, 65536),
    ConvWorkload("conv3_f64_n8_E65536", 23, "f64", 8, 65536),
    ConvWorkload("conv4_f64_n8_q12_E32768", 24, "f64", 8, 32768, 12),
)

CONV_BLOCK = 256
_STREAM_CM, _STREAM_CP = 5, 6


def conv_custom(n: int, num_elems: int, dtype: str = "f64", key: int = 120,
                nq: int = 0) -> ConvWorkload:
    return ConvWorkload(f"conv_custom_{dtype}_n{n}_q{nq or n}_E{num_elems}", key, dtype, n,
                        num_elems, nq)


def _lagrange_matrices(xq: np.ndarray, xv: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Values and first derivatives of the Lagrange basis on nodes ``xq`` at points ``xv``:
    ``I[v,q] = l_q(xv[v])``, ``D[v,q] = l_q'(xv[v])`` (product formulas, fp64)."""
    nq = len(xq)
    interp = np.empty((len(xv), nq))
    deriv = np.empty((len(xv), nq))
    for q in range(nq):
        others = [r for r in range(nq) if r != q]
        den = np.prod([xq[q] - xq[r] for r in others]) if others else 1.0
        for v, x in enumerate(xv):
            interp[v, q] = np.prod([x - xq[r] for r in others]) / den if others else 1.0
            total = 0.0
            for s in others:
                total += np.prod([x - xq[r] for r in others if r != s]) if len(others) > 1 else 1.0
            deriv[v, q] = total / den
    return interp, deriv


def conv_matrices(w: ConvWorkload) -> Tuple[np.ndarray, np.ndarray]:
    """``(D_vq, I_vq)``, each ``[n,q]``: differentiation and interpolation from the q
    Chebyshev-Gauss points (quadrature side) to the n Chebyshev-Lobatto points (node side)."""
    n, q = w.n, w.q
    xq = -np.cos(np.pi * (2 * np.arange(q) + 1) / (2 * q))
    xv = -np.cos(np.pi * np.arange(n) / (n - 1)) if n > 1 else np.zeros(1)
    interp, deriv = _lagrange_matrices(xq, xv)
    return deriv.astype(w.np_dtype), interp.astype(w.np_dtype)


def conv_metric(w: ConvWorkload, start: int = 0, stop: int | None = None) -> np.ndarray:
    """Metric factor ``M[start:stop]`` ~ U(0.5, 2), ``[stop-start, q, q, q]``."""
    stop = w.num_elems if stop is None else stop
    n = w.q
    out = np.empty((stop - start, n, n, n), dtype=w.np_dtype)
    b = start // CONV_BLOCK
    while b * CONV_BLOCK < stop:
        lo, hi = max(start, b * CONV_BLOCK), min(stop, (b + 1) * CONV_BLOCK)
        blk = _rng(w.index, _STREAM_CM, b).uniform(0.5, 2.0, (hi - b * CONV_BLOCK, n, n, n))
        out[lo - start:hi - start] = blk[lo - b * CONV_BLOCK:]
        b += 1
    return out


def conv_flux(w: ConvWorkload, start: int = 0, stop: int | None = None) -> np.ndarray:
    """Fluxes ``P[:, :, start:stop]`` ~ U(-1, 1), ``[3, 3, stop-start, q, q, q]``; every
    (component, direction, block of elements) has its own seed."""
    stop = w.num_elems if stop is None else stop
    n = w.q
    out = np.empty((3, 3, stop - start, n, n, n), dtype=w.np_dtype)
    b = start // CONV_BLOCK
    while b * CONV_BLOCK < stop:
        lo, hi = max(start, b * CONV_BLOCK), min(stop, (b + 1) * CONV_BLOCK)
        for c in range(3):
            for d in range(3):
                blk = _rng(w.index, _STREAM_CP, 3 * c + d, b).uniform(
                    -1.0, 1.0, (hi - b * CONV_BLOCK, n, n, n))
                out[c, d, lo - start:hi - start] = blk[lo - b * CONV_BLOCK:]
        b += 1
    return out


def conv_inputs(w: ConvWorkload, start: int = 0, stop: int | None = None):
    """``(P, M, D_vq, I_vq)`` for elements ``start..stop-1`` as host arrays."""
    d_vq, i_vq = conv_matrices(w)
    return conv_flux(w, start, stop), conv_metric(w, start, stop), d_vq, i_vq


def conv_to_device(w: ConvWorkload, threads: int = 12, chunk: int = 4 * CONV_BLOCK):
    """Device tensors ``(P, M, D_vq, I_vq)`` of a whole convection workload, generated block by
    block on the host and copied into place."""
    from concurrent.futures import ThreadPoolExecutor

    import torch

    e, n = w.num_elems, w.q
    tdtype = torch.float64 if w.dtype == "f64" else torch.float32
    tp = torch.empty((3, 3, e, n, n, n), dtype=tdtype, device="cuda")
    tm = torch.empty((e, n, n, n), dtype=tdtype, device="cuda")
    spans = [(lo, min(e, lo + chunk)) for lo in range(0, e, chunk)]

    def gen(span):
        lo, hi = span
        return lo, hi, conv_flux(w, lo, hi), conv_metric(w, lo, hi)

    with ThreadPoolExecutor(max_workers=threads) as ex:
        for lo, hi, hp, hm in ex.map(gen, spans):
            tp[:, :, lo:hi].copy_(torch.from_numpy(hp))
            tm[lo:hi].copy_(torch.from_numpy(hm))
    d_vq, i_vq = conv_matrices(w)
    up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    return tp, tm, up(d_vq), up(i_vq)


# ------------------------------------------------------------------------------------------
# Inputs of the operator on anisotropic elements: the recipe of the cubic workloads with one
# size per axis (an orthogonal matrix and an eigenvalue vector per direction, a shift per
# element, uniform u).  Shapes stand for extruded meshes (a different order along one axis).

@dataclass(frozen=True)
class AnisoWorkload:
    """One synthetic configuration of the operator with ``dims = (n_x, n_y, n_z)`` points."""

    name: str
    index: int          # seed key, disjoint from the other configurations
    dtype: str
    dims: Tuple[int, int, int]
    num_elems: int

    @property
    def np_dtype(self):
        return np.float64 if self.dtype == "f64" else np.float32

    @property
    def word(self) -> int:
        return 8 if self.dtype == "f64" else 4

    @property
    def points(self) -> int:
        return self.dims[0] * self.dims[1] * self.dims[2]

    @property
    def bytes_per_elem(self) -> int:
        """Algorithmic traffic per element: u_e and D_e in, v_e out."""
        return 3 * self.points * self.word

    @property
    def flop_per_elem(self) -> int:
        """Six mode products (2 n_axis flops per point each) and the scale."""
        return self.points * (4 * sum(self.dims) + 1)


ANISO_CONFIGS = (
    AnisoWorkload("aniso0_f64_5x6x7_E512", 30, "f64", (5, 6, 7), 512),
    AnisoWorkload("aniso1_f64_8x8x12_E131072", 31, "f64", (8, 8, 12), 131072),
    AnisoWorkload("aniso2_f64_11x11x14_E131072", 32, "f64", (11, 11, 14), 131072),
    AnisoWorkload("aniso3_f32_12x12x16_E262144", 33, "f32", (12, 12, 16), 262144),
)

_STREAM_AS, _STREAM_AL, _STREAM_AM, _STREAM_AU = 7, 8, 9, 10


def aniso_custom(dims, num_elems: int, dtype: str = "f64", key: int = 130) -> AnisoWorkload:
    dims = tuple(int(k) for k in dims)
    return AnisoWorkload(f"aniso_custom_{dtype}_{dims[0]}x{dims[1]}x{dims[2]}_E{num_elems}", key,
                         dtype, dims, num_elems)


def aniso_matrices(w: AnisoWorkload):
    """``(S_x, S_y, S_z)``: one orthogonal matrix per axis, ``[n_axis, n_axis]``."""
    rng = _rng(w.index, _STREAM_AS)
    return tuple(orthogonal_matrix(k, rng).astype(w.np_dtype) for k in w.dims)


def aniso_field_u(w: AnisoWorkload, start: int = 0, stop: int | None = None) -> np.ndarray:
    """``u[start:stop]`` of shape ``[stop-start, n_x, n_y, n_z]``, U(-1, 1), drawn in fp64 per
    seed block and rounded once."""
    stop = w.num_elems if stop is None else stop
    out = np.empty((stop - start, *w.dims), dtype=w.np_dtype)
    for b, lo, hi in _blocks(start, stop):
        cnt = hi - b * BLOCK
        blk = _rng(w.index, _STREAM_AU, b).uniform(-1.0, 1.0, (cnt, *w.dims))
        out[lo - start:hi - start] = blk[lo - b * BLOCK:]
    return out


def aniso_diagonal_d(w: AnisoWorkload, start: int = 0, stop: int | None = None) -> np.ndarray:
    """``D[e,i,j,k] = 1 / (lam_x[i] + lam_y[j] + lam_z[k] + mu_e)`` with ``lam`` ~ U(0.1, 10)
    per axis and ``mu_e`` ~ U(0, 1), evaluated in fp64 and rounded once (an input recipe)."""
    stop = w.num_elems if stop is None else stop
    rng = _rng(w.index, _STREAM_AL)
    lx, ly, lz = (rng.uniform(0.1, 10.0, k) for k in w.dims)
    lam3 = lx[:, None, None] + ly[None, :, None] + lz[None, None, :]
    out = np.empty((stop - start, *w.dims), dtype=w.np_dtype)
    for b, lo, hi in _blocks(start, stop):
        mu = _rng(w.index, _STREAM_AM, b).uniform(0.0, 1.0, BLOCK)[lo - b * BLOCK:hi - b * BLOCK]
        out[lo - start:hi - start] = 1.0 / (lam3[None] + mu[:, None, None, None])
    return out


def aniso_inputs(w: AnisoWorkload, start: int = 0, stop: int | None = None):
    """``(u, S_x, S_y, S_z, D)`` for elements ``start..stop-1`` as host arrays."""
    sx, sy, sz = aniso_matrices(w)
    return aniso_field_u(w, start, stop), sx, sy, sz, aniso_diagonal_d(w, start, stop)


def aniso_to_device(w: AnisoWorkload, threads: int = 12, chunk: int = 2 * BLOCK):
    """Device tensors ``(u, S_x, S_y, S_z, D)`` of a whole anisotropic workload, generated
    block by block on the host and copied into place."""
    from concurrent.futures import ThreadPoolExecutor

    import torch

    e = w.num_elems
    tdtype = torch.float64 if w.dtype == "f64" else torch.float32
    tu = torch.empty((e, *w.dims), dtype=tdtype, device="cuda")
    td = torch.empty((e, *w.dims), dtype=tdtype, device="cuda")
    spans = [(lo, min(e, lo + chunk)) for lo in range(0, e, chunk)]

    def gen(span):
        lo, hi = span
        return lo, hi, aniso_field_u(w, lo, hi), aniso_diagonal_d(w, lo, hi)

    with ThreadPoolExecutor(max_workers=threads) as ex:
        for lo, hi, hu, hd in ex.map(gen, spans):
            tu[lo:hi].copy_(torch.from_numpy(hu))
            td[lo:hi].copy_(torch.from_numpy(hd))
    mats = tuple(torch.from_numpy(np.ascontiguousarray(s)).cuda() for s in aniso_matrices(w))
    return (tu, *mats, td)

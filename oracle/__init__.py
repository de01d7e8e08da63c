"""CPU oracle for the batched inverse-Helmholtz tensor-product operator.

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, the smoke check and the benchmark's
CPU-baseline leg, never by the product package.  The arithmetic lives in ``tpo_oracle.c``
(plain C, fp64, left-to-right sums); this module compiles it with gcc and marshals NumPy
arrays into it.  Inputs of any float dtype are promoted to fp64 first, so an fp32 workload
is checked against the fp64 result on the same rounded inputs.

Operator and index conventions: see the header of ``tpo_oracle.c`` (Sec. 2.2 and the
reduction-lifting example of Sec. 5.2 of the paper).
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tpo_oracle.c")
_LIB = os.path.join(_HERE, "libtpo_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile ``tpo_oracle.c`` into ``libtpo_oracle.so`` next to it (gcc, -O2, no FMA
    contraction, OpenMP over elements only)."""
    if (not force and os.path.exists(_LIB)
            and os.path.getmtime(_LIB) >= os.path.getmtime(_SRC)):
        return _LIB
    tmp = _LIB + f".tmp{os.getpid()}"
    cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
           "-fPIC", "-shared", "-Wall", "-Wextra", "-o", tmp, _SRC]
    subprocess.run(cmd, check=True)
    os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        dp = ctypes.POINTER(ctypes.c_double)
        lib.tpo_oracle_ihelm_lifted.argtypes = [dp, dp, dp, dp, dp, dp, ctypes.c_int,
                                                ctypes.c_longlong, ctypes.c_int]
        lib.tpo_oracle_ihelm_lifted.restype = ctypes.c_int
        lib.tpo_oracle_ihelm_direct.argtypes = [dp, dp, dp, dp, dp, dp, ctypes.c_int,
                                                ctypes.c_longlong]
        lib.tpo_oracle_ihelm_direct.restype = ctypes.c_int
        lib.tpo_oracle_forward_lifted.argtypes = [dp, dp, dp, dp, dp, ctypes.c_int,
                                                  ctypes.c_longlong]
        lib.tpo_oracle_forward_lifted.restype = ctypes.c_int
        lib.tpo_oracle_ihelm_sep.argtypes = [dp] * 9 + [ctypes.c_int, ctypes.c_longlong,
                                                        ctypes.c_int]
        lib.tpo_oracle_ihelm_sep.restype = ctypes.c_int
        lib.tpo_oracle_backward_lifted.argtypes = [dp, dp, dp, dp, dp, ctypes.c_int,
                                                   ctypes.c_longlong]
        lib.tpo_oracle_backward_lifted.restype = ctypes.c_int
        lib.tpo_oracle_convection_direct.argtypes = [dp, dp, dp, dp, dp, ctypes.c_int, ctypes.c_int,
                                                     ctypes.c_longlong]
        lib.tpo_oracle_convection_direct.restype = ctypes.c_int
        lib.tpo_oracle_convection_lifted.argtypes = [dp, dp, dp, dp, dp, ctypes.c_int, ctypes.c_int,
                                                     ctypes.c_longlong, ctypes.c_int]
        lib.tpo_oracle_convection_lifted.restype = ctypes.c_int
        lib.tpo_oracle_ihelm_aniso.argtypes = [dp] * 6 + [ctypes.c_int] * 3 + [ctypes.c_longlong,
                                                                               ctypes.c_int]
        lib.tpo_oracle_ihelm_aniso.restype = ctypes.c_int
        lib.tpo_oracle_max_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a), dtype=np.float64)


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _check_shapes(u, sx, sy, sz, d):
    if u.ndim != 4 or not (u.shape[1] == u.shape[2] == u.shape[3]):
        raise ValueError(f"u must be [E,n,n,n], got {u.shape}")
    n = u.shape[1] if u.shape[0] else (sx.shape[0] if sx.ndim == 2 else 0)
    for name, s in (("S_x", sx), ("S_y", sy), ("S_z", sz)):
        if s.shape != (n, n):
            raise ValueError(f"{name} must be [{n},{n}], got {s.shape}")
    if d is not None and d.shape != u.shape:
        raise ValueError(f"D must have u's shape {u.shape}, got {d.shape}")
    return n


def max_threads() -> int:
    return int(_load().tpo_oracle_max_threads())


def ihelm_apply(u, s_x, s_y, s_z, d, nthreads: int = 0) -> np.ndarray:
    """``v = (S_x (x) S_y (x) S_z) diag(D) (S_x (x) S_y (x) S_z)^T u`` per element, by the
    lifted (sum-factorised) form.  Returns fp64 ``[E,n,n,n]``."""
    u, s_x, s_y, s_z, d = map(_f64, (u, s_x, s_y, s_z, d))
    n = _check_shapes(u, s_x, s_y, s_z, d)
    v = np.empty_like(u)
    rc = _load().tpo_oracle_ihelm_lifted(_ptr(u), _ptr(s_x), _ptr(s_y), _ptr(s_z), _ptr(d),
                                         _ptr(v), n, u.shape[0], nthreads)
    if rc != 0:
        raise RuntimeError(f"tpo_oracle_ihelm_lifted failed ({rc})")
    return v


def ihelm_apply_direct(u, s_x, s_y, s_z, d) -> np.ndarray:
    """Same operator by the unlifted six-deep sums (O(n^6) per element; small n only)."""
    u, s_x, s_y, s_z, d = map(_f64, (u, s_x, s_y, s_z, d))
    n = _check_shapes(u, s_x, s_y, s_z, d)
    v = np.empty_like(u)
    rc = _load().tpo_oracle_ihelm_direct(_ptr(u), _ptr(s_x), _ptr(s_y), _ptr(s_z), _ptr(d),
                                         _ptr(v), n, u.shape[0])
    if rc != 0:
        raise RuntimeError(f"tpo_oracle_ihelm_direct failed ({rc})")
    return v


def ihelm_apply_sep(u, s_x, s_y, s_z, lam_x, lam_y, lam_z, mu, nthreads: int = 0) -> np.ndarray:
    """The operator with the separable diagonal
    ``D[e,i,j,k] = 1 / (lam_x[i] + lam_y[j] + lam_z[k] + mu[e])`` (fp64, denominator summed left
    to right).  ``lam_*`` are ``[n]``, ``mu`` is ``[E]``.  Returns fp64 ``[E,n,n,n]``."""
    u, s_x, s_y, s_z, lam_x, lam_y, lam_z, mu = map(_f64, (u, s_x, s_y, s_z, lam_x, lam_y,
                                                            lam_z, mu))
    n = _check_shapes(u, s_x, s_y, s_z, None)
    for name, lam in (("lam_x", lam_x), ("lam_y", lam_y), ("lam_z", lam_z)):
        if lam.shape != (n,):
            raise ValueError(f"{name} must be [{n}], got {lam.shape}")
    if mu.shape != (u.shape[0],):
        raise ValueError(f"mu must be [{u.shape[0]}], got {mu.shape}")
    v = np.empty_like(u)
    rc = _load().tpo_oracle_ihelm_sep(_ptr(u), _ptr(s_x), _ptr(s_y), _ptr(s_z), _ptr(lam_x),
                                      _ptr(lam_y), _ptr(lam_z), _ptr(mu), _ptr(v), n,
                                      u.shape[0], nthreads)
    if rc != 0:
        raise RuntimeError(f"tpo_oracle_ihelm_sep failed ({rc})")
    return v


def forward(u, s_x, s_y, s_z) -> np.ndarray:
    """Forward half only: ``t = (S_x^T (x) S_y^T (x) S_z^T) u`` (the worked example of
    Sec. 5.2), lifted form."""
    u, s_x, s_y, s_z = map(_f64, (u, s_x, s_y, s_z))
    n = _check_shapes(u, s_x, s_y, s_z, None)
    t = np.empty_like(u)
    rc = _load().tpo_oracle_forward_lifted(_ptr(u), _ptr(s_x), _ptr(s_y), _ptr(s_z),
                                           _ptr(t), n, u.shape[0])
    if rc != 0:
        raise RuntimeError(f"tpo_oracle_forward_lifted failed ({rc})")
    return t


def backward(g, s_x, s_y, s_z) -> np.ndarray:
    """Backward half only: ``v = (S_x (x) S_y (x) S_z) g``, lifted form."""
    g, s_x, s_y, s_z = map(_f64, (g, s_x, s_y, s_z))
    n = _check_shapes(g, s_x, s_y, s_z, None)
    v = np.empty_like(g)
    rc = _load().tpo_oracle_backward_lifted(_ptr(g), _ptr(s_x), _ptr(s_y), _ptr(s_z),
                                            _ptr(v), n, g.shape[0])
    if rc != 0:
        raise RuntimeError(f"tpo_oracle_backward_lifted failed ({rc})")
    return v


def ihelm_apply_aniso(u, s_x, s_y, s_z, d, direct: bool = False) -> np.ndarray:
    """The operator on anisotropic elements: ``u``, ``D`` are ``[E,nx,ny,nz]``, ``S_x`` is
    ``[nx,nx]``, ``S_y`` ``[ny,ny]``, ``S_z`` ``[nz,nz]``.  ``direct=True``: the six-deep sums."""
    u, s_x, s_y, s_z, d = map(_f64, (u, s_x, s_y, s_z, d))
    if u.ndim != 4 or d.shape != u.shape:
        raise ValueError("u and D must both be [E,nx,ny,nz]")
    _, nx, ny, nz = u.shape
    for name, s, n in (("S_x", s_x, nx), ("S_y", s_y, ny), ("S_z", s_z, nz)):
        if s.shape != (n, n):
            raise ValueError(f"{name} must be [{n},{n}], got {s.shape}")
    v = np.empty_like(u)
    rc = _load().tpo_oracle_ihelm_aniso(_ptr(u), _ptr(s_x), _ptr(s_y), _ptr(s_z), _ptr(d),
                                        _ptr(v), nx, ny, nz, u.shape[0], int(direct))
    if rc != 0:
        raise RuntimeError(f"tpo_oracle_ihelm_aniso failed ({rc})")
    return v


def _check_convection(p, m, d_vq, i_vq):
    if d_vq.ndim != 2 or d_vq.shape != i_vq.shape:
        raise ValueError("D_vq and I_vq must both be [nv,nq]")
    nv, nq = d_vq.shape
    if m.ndim != 4 or m.shape[1:] != (nq, nq, nq):
        raise ValueError(f"M must be [E,{nq},{nq},{nq}], got {m.shape}")
    if p.shape != (3, 3) + m.shape:
        raise ValueError(f"P must be [3,3,E,{nq},{nq},{nq}], got {p.shape}")
    return nv, nq, m.shape[0]


def convection_apply(p, m, d_vq, i_vq, nthreads: int = 0, direct: bool = False) -> np.ndarray:
    """Volume integral of the convective flux (Eq. 1 of the paper):
    ``F[c,e,k,j,i] = sum_lmn (D[i,l] I[j,m] I[k,n] P[c,0] + I[i,l] D[j,m] I[k,n] P[c,1]
    + I[i,l] I[j,m] D[k,n] P[c,2]) * M[e,n,m,l]`` with ``P[c,d]`` read at ``[e,n,m,l]``.
    ``direct=True`` evaluates the six-deep sums as written (small sizes only).
    Returns fp64 ``[3,E,nv,nv,nv]``."""
    p, m, d_vq, i_vq = map(_f64, (p, m, d_vq, i_vq))
    nv, nq, e = _check_convection(p, m, d_vq, i_vq)
    f = np.empty((3, e, nv, nv, nv))
    if direct:
        rc = _load().tpo_oracle_convection_direct(_ptr(p), _ptr(m), _ptr(d_vq), _ptr(i_vq),
                                                  _ptr(f), nv, nq, e)
    else:
        rc = _load().tpo_oracle_convection_lifted(_ptr(p), _ptr(m), _ptr(d_vq), _ptr(i_vq),
                                                  _ptr(f), nv, nq, e, nthreads)
    if rc != 0:
        raise RuntimeError(f"tpo_oracle_convection failed ({rc})")
    return f


def max_rel_err_per_element(v_test, v_ref) -> float:
    """Worst over elements of ``max|v_test - v_ref| / max|v_ref|`` (max-norm relative error
    per element).  An all-zero reference element counts its absolute error."""
    a = np.asarray(v_test, dtype=np.float64)
    b = np.asarray(v_ref, dtype=np.float64)
    if a.shape != b.shape:
        raise ValueError("shape mismatch")
    if a.size == 0:
        return 0.0
    e = a.shape[0]
    num = np.abs(a - b).reshape(e, -1).max(axis=1)
    den = np.abs(b).reshape(e, -1).max(axis=1)
    den = np.where(den > 0, den, 1.0)
    return float((num / den).max())

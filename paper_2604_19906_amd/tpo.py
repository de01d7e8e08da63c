"""Thin ctypes binding over libtpo.so: same names as the C ABI in ``include/tpo.h``, argument
marshalling only.  Every step of the operator runs in the library's HIP kernels; there is no
fallback: if the library has not been built, loading raises.

Pointers are plain integers (``tensor.data_ptr()``), the stream is a ``hipStream_t`` as an
integer (``torch.cuda.current_stream().cuda_stream``).
"""
from __future__ import annotations

import ctypes
import os

TPO_F64, TPO_F32 = 0, 1
TPO_OK = 0
TPO_ERR_INVALID_ARG, TPO_ERR_UNSUPPORTED, TPO_ERR_NOT_INITIALIZED = -1, -2, -3
TPO_ERR_DEVICE, TPO_ERR_ALIAS = -4, -5
TPO_FORWARD, TPO_BACKWARD = 0, 1
TPO_VARIANT_AUTO, TPO_VARIANT_PENCIL, TPO_VARIANT_MFMA, TPO_VARIANT_PENCIL_MM = 0, 1, 2, 3
TPO_MAX_N = 16

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libtpo.so")
BENCH_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libtpo_bench.so")
_lib = None
_bench_lib = None


class TpoError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"{what}: {status_string(status)} ({status})")
        self.status = status


def lib():
    """Load libtpo.so (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2604_19906_amd.build`")
        l = ctypes.CDLL(LIB_PATH)
        vp, ci, cll = ctypes.c_void_p, ctypes.c_int, ctypes.c_longlong
        l.tpo_create.argtypes = []
        l.tpo_create.restype = ci
        l.tpo_destroy.argtypes = []
        l.tpo_destroy.restype = ci
        l.tpo_ihelm_apply.argtypes = [vp, vp, vp, vp, vp, vp, ci, cll, ci, vp]
        l.tpo_ihelm_apply.restype = ci
        l.tpo_ihelm_apply_variant.argtypes = [vp, vp, vp, vp, vp, vp, ci, cll, ci, vp, ci]
        l.tpo_ihelm_apply_variant.restype = ci
        l.tpo_ihelm_variant_for.argtypes = [ci, ci, ci]
        l.tpo_ihelm_variant_for.restype = ci
        l.tpo_ihelm_variant_for_batch.argtypes = [ci, ci, ci, cll]
        l.tpo_ihelm_variant_for_batch.restype = ci
        l.tpo_ihelm_has_variant.argtypes = [ci, ci, ci]
        l.tpo_ihelm_has_variant.restype = ci
        l.tpo_ihelm_apply_sep.argtypes = [vp] * 9 + [ci, cll, ci, vp]
        l.tpo_ihelm_apply_sep.restype = ci
        l.tpo_ihelm_apply_sep_variant.argtypes = [vp] * 9 + [ci, cll, ci, vp, ci]
        l.tpo_ihelm_apply_sep_variant.restype = ci
        l.tpo_ihelm_sep_variant_for.argtypes = [ci, ci]
        l.tpo_ihelm_sep_variant_for.restype = ci
        l.tpo_ihelm_sep_variant_for_batch.argtypes = [ci, ci, ci, cll]
        l.tpo_ihelm_sep_variant_for_batch.restype = ci
        l.tpo_ihelm_sep_has_variant.argtypes = [ci, ci, ci]
        l.tpo_ihelm_sep_has_variant.restype = ci
        l.tpo_ihelm_apply_aniso.argtypes = [vp, vp, vp, vp, vp, vp, ci, ci, ci, cll, ci, vp]
        l.tpo_ihelm_apply_aniso.restype = ci
        l.tpo_transform_apply.argtypes = [vp, vp, vp, vp, vp, ci, cll, ci, ci, vp]
        l.tpo_transform_apply.restype = ci
        l.tpo_convection_apply.argtypes = [vp, vp, vp, vp, vp, ci, ci, cll, ci, vp]
        l.tpo_convection_apply.restype = ci
        l.tpo_convection_has_shape.argtypes = [ci, ci, ci]
        l.tpo_convection_has_shape.restype = ci
        l.tpo_status_string.argtypes = [ci]
        l.tpo_status_string.restype = ctypes.c_char_p
        _lib = l
    return _lib


def status_string(status: int) -> str:
    return lib().tpo_status_string(int(status)).decode()


def tpo_create() -> int:
    return lib().tpo_create()


def tpo_destroy() -> int:
    return lib().tpo_destroy()


def tpo_ihelm_apply(u, S_x, S_y, S_z, D, v, n, num_elems, dtype, stream) -> int:
    """Raw call: integer device pointers in, status out."""
    return lib().tpo_ihelm_apply(u, S_x, S_y, S_z, D, v, int(n), int(num_elems), int(dtype),
                                 stream)


def tpo_ihelm_apply_variant(u, S_x, S_y, S_z, D, v, n, num_elems, dtype, stream,
                            variant) -> int:
    return lib().tpo_ihelm_apply_variant(u, S_x, S_y, S_z, D, v, int(n), int(num_elems),
                                         int(dtype), stream, int(variant))


def tpo_ihelm_variant_for(n: int, dtype: int, shared_s: bool = False) -> int:
    return lib().tpo_ihelm_variant_for(int(n), int(dtype), int(bool(shared_s)))


def tpo_ihelm_variant_for_batch(n: int, dtype: int, shared_s: bool, num_elems: int) -> int:
    return lib().tpo_ihelm_variant_for_batch(int(n), int(dtype), int(bool(shared_s)),
                                             int(num_elems))


def tpo_ihelm_has_variant(n: int, dtype: int, variant: int) -> bool:
    return bool(lib().tpo_ihelm_has_variant(int(n), int(dtype), int(variant)))


def tpo_ihelm_apply_sep(u, S_x, S_y, S_z, lam_x, lam_y, lam_z, mu, v, n, num_elems, dtype,
                        stream) -> int:
    """Raw call of the separable-diagonal form: integer device pointers in, status out."""
    return lib().tpo_ihelm_apply_sep(u, S_x, S_y, S_z, lam_x, lam_y, lam_z, mu, v, int(n),
                                     int(num_elems), int(dtype), stream)


def tpo_ihelm_apply_sep_variant(u, S_x, S_y, S_z, lam_x, lam_y, lam_z, mu, v, n, num_elems,
                                dtype, stream, variant) -> int:
    return lib().tpo_ihelm_apply_sep_variant(u, S_x, S_y, S_z, lam_x, lam_y, lam_z, mu, v,
                                             int(n), int(num_elems), int(dtype), stream,
                                             int(variant))


def tpo_ihelm_sep_variant_for(n: int, dtype: int) -> int:
    return lib().tpo_ihelm_sep_variant_for(int(n), int(dtype))


def tpo_ihelm_sep_variant_for_batch(n: int, dtype: int, shared_s: bool, num_elems: int) -> int:
    return lib().tpo_ihelm_sep_variant_for_batch(int(n), int(dtype), int(bool(shared_s)),
                                                 int(num_elems))


def tpo_ihelm_sep_has_variant(n: int, dtype: int, variant: int) -> bool:
    return bool(lib().tpo_ihelm_sep_has_variant(int(n), int(dtype), int(variant)))


def tpo_ihelm_apply_aniso(u, S_x, S_y, S_z, D, v, n_x, n_y, n_z, num_elems, dtype, stream) -> int:
    """Raw call of the operator on anisotropic elements: integer device pointers in, status out."""
    return lib().tpo_ihelm_apply_aniso(u, S_x, S_y, S_z, D, v, int(n_x), int(n_y), int(n_z),
                                       int(num_elems), int(dtype), stream)


def tpo_transform_apply(u, S_x, S_y, S_z, t, n, num_elems, dtype, direction, stream) -> int:
    """Raw call of one half of the operator: integer device pointers in, status out."""
    return lib().tpo_transform_apply(u, S_x, S_y, S_z, t, int(n), int(num_elems), int(dtype),
                                     int(direction), stream)


def tpo_convection_apply(P, M, D_vq, I_vq, F, n_v, n_q, num_elems, dtype, stream) -> int:
    """Raw call of the convection volume term: integer device pointers in, status out."""
    return lib().tpo_convection_apply(P, M, D_vq, I_vq, F, int(n_v), int(n_q), int(num_elems),
                                      int(dtype), stream)


def tpo_convection_has_shape(n_v: int, n_q: int, dtype: int) -> bool:
    return bool(lib().tpo_convection_has_shape(int(n_v), int(n_q), int(dtype)))


def bench_lib():
    """Load libtpo_bench.so, the benchmark's measurement aid (once).  Raises if it is missing."""
    global _bench_lib
    if _bench_lib is None:
        if not os.path.exists(BENCH_LIB_PATH):
            raise RuntimeError(
                f"{BENCH_LIB_PATH} is missing: build it with `python -m paper_2604_19906_amd.build`")
        l = ctypes.CDLL(BENCH_LIB_PATH)
        vp, ci, cll = ctypes.c_void_p, ctypes.c_int, ctypes.c_longlong
        l.tpo_stream_scale.argtypes = [vp, vp, vp, cll, ci, vp]
        l.tpo_stream_scale.restype = ci
        _bench_lib = l
    return _bench_lib


def tpo_stream_scale(u, D, v, count, dtype, stream) -> int:
    """Measurement aid (libtpo_bench.so): v[i] = u[i] * D[i] over flat device arrays."""
    return bench_lib().tpo_stream_scale(u, D, v, int(count), int(dtype), stream)


def check(status: int, what: str = "tpo call") -> None:
    if status != TPO_OK:
        raise TpoError(status, what)


def apply_tensors(u, S_x, S_y, S_z, D, v=None, variant: int = TPO_VARIANT_AUTO):
    """Convenience over torch device tensors: marshals pointers, shape and the current
    stream; raises TpoError on a non-zero status.  Returns ``v`` (allocated if None)."""
    import torch

    if u.dim() != 4 or not u.is_cuda:
        raise ValueError("u must be a device tensor of shape [E,n,n,n]")
    for t in (u, S_x, S_y, S_z, D):
        if not t.is_contiguous() or t.dtype != u.dtype or not t.is_cuda:
            raise ValueError("all tensors must be contiguous device tensors of one dtype")
    e, n = u.shape[0], u.shape[1]
    if tuple(u.shape[1:]) != (n, n, n) or tuple(D.shape) != tuple(u.shape):
        raise ValueError("u and D must both be [E,n,n,n]")
    for s in (S_x, S_y, S_z):
        if tuple(s.shape) != (n, n):
            raise ValueError("S matrices must be [n,n]")
    if v is None:
        v = torch.empty_like(u)
    elif (tuple(v.shape) != tuple(u.shape) or v.dtype != u.dtype or not v.is_contiguous()
          or not v.is_cuda):
        raise ValueError("v must match u")
    dtype = {torch.float64: TPO_F64, torch.float32: TPO_F32}[u.dtype]
    stream = torch.cuda.current_stream().cuda_stream
    check(tpo_ihelm_apply_variant(u.data_ptr(), S_x.data_ptr(), S_y.data_ptr(),
                                  S_z.data_ptr(), D.data_ptr(), v.data_ptr(), n, e, dtype,
                                  stream, variant), "tpo_ihelm_apply")
    return v


def apply_sep_tensors(u, S_x, S_y, S_z, lam_x, lam_y, lam_z, mu, v=None,
                      variant: int = TPO_VARIANT_AUTO):
    """Separable-diagonal form over torch device tensors (``lam_*`` are ``[n]``, ``mu`` is
    ``[E]``); marshalling only, like :func:`apply_tensors`."""
    import torch

    if u.dim() != 4 or not u.is_cuda:
        raise ValueError("u must be a device tensor of shape [E,n,n,n]")
    for t in (u, S_x, S_y, S_z, lam_x, lam_y, lam_z, mu):
        if not t.is_contiguous() or t.dtype != u.dtype or not t.is_cuda:
            raise ValueError("all tensors must be contiguous device tensors of one dtype")
    e, n = u.shape[0], u.shape[1]
    if tuple(u.shape[1:]) != (n, n, n):
        raise ValueError("u must be [E,n,n,n]")
    for s in (S_x, S_y, S_z):
        if tuple(s.shape) != (n, n):
            raise ValueError("S matrices must be [n,n]")
    for lam in (lam_x, lam_y, lam_z):
        if tuple(lam.shape) != (n,):
            raise ValueError("lam vectors must be [n]")
    if tuple(mu.shape) != (e,):
        raise ValueError("mu must be [E]")
    if v is None:
        v = torch.empty_like(u)
    elif (tuple(v.shape) != tuple(u.shape) or v.dtype != u.dtype or not v.is_contiguous()
          or not v.is_cuda):
        raise ValueError("v must match u")
    dtype = {torch.float64: TPO_F64, torch.float32: TPO_F32}[u.dtype]
    stream = torch.cuda.current_stream().cuda_stream
    check(tpo_ihelm_apply_sep_variant(u.data_ptr(), S_x.data_ptr(), S_y.data_ptr(),
                                      S_z.data_ptr(), lam_x.data_ptr(), lam_y.data_ptr(),
                                      lam_z.data_ptr(), mu.data_ptr(), v.data_ptr(), n, e,
                                      dtype, stream, variant), "tpo_ihelm_apply_sep")
    return v


def transform_tensors(u, S_x, S_y, S_z, direction: int, t=None):
    """One half of the operator over torch device tensors; marshalling only."""
    import torch

    if u.dim() != 4 or not u.is_cuda:
        raise ValueError("u must be a device tensor of shape [E,n,n,n]")
    for x in (u, S_x, S_y, S_z):
        if not x.is_contiguous() or x.dtype != u.dtype or not x.is_cuda:
            raise ValueError("all tensors must be contiguous device tensors of one dtype")
    e, n = u.shape[0], u.shape[1]
    if tuple(u.shape[1:]) != (n, n, n):
        raise ValueError("u must be [E,n,n,n]")
    for s in (S_x, S_y, S_z):
        if tuple(s.shape) != (n, n):
            raise ValueError("S matrices must be [n,n]")
    if t is None:
        t = torch.empty_like(u)
    elif (tuple(t.shape) != tuple(u.shape) or t.dtype != u.dtype or not t.is_contiguous()
          or not t.is_cuda):
        raise ValueError("t must match u")
    dtype = {torch.float64: TPO_F64, torch.float32: TPO_F32}[u.dtype]
    check(tpo_transform_apply(u.data_ptr(), S_x.data_ptr(), S_y.data_ptr(), S_z.data_ptr(),
                              t.data_ptr(), n, e, dtype, direction,
                              torch.cuda.current_stream().cuda_stream), "tpo_transform_apply")
    return t


def convection_tensors(P, M, D_vq, I_vq, F=None):
    """Convection volume term over torch device tensors (``P`` ``[3,3,E,nq,nq,nq]``, ``M``
    ``[E,nq,nq,nq]``, ``D_vq``/``I_vq`` ``[nv,nq]``); marshalling only.  Returns ``F``
    ``[3,E,nv,nv,nv]``."""
    import torch

    for x in (P, M, D_vq, I_vq):
        if not x.is_contiguous() or x.dtype != P.dtype or not x.is_cuda:
            raise ValueError("all tensors must be contiguous device tensors of one dtype")
    if D_vq.dim() != 2 or tuple(I_vq.shape) != tuple(D_vq.shape):
        raise ValueError("D_vq and I_vq must both be [nv,nq]")
    nv, nq = D_vq.shape
    if M.dim() != 4 or tuple(M.shape[1:]) != (nq, nq, nq):
        raise ValueError("M must be [E,nq,nq,nq]")
    e = M.shape[0]
    if tuple(P.shape) != (3, 3, e, nq, nq, nq):
        raise ValueError("P must be [3,3,E,nq,nq,nq]")
    if F is None:
        F = torch.empty((3, e, nv, nv, nv), dtype=P.dtype, device=P.device)
    elif (tuple(F.shape) != (3, e, nv, nv, nv) or F.dtype != P.dtype or not F.is_contiguous()
          or not F.is_cuda):
        raise ValueError("F must be [3,E,nv,nv,nv]")
    dtype = {torch.float64: TPO_F64, torch.float32: TPO_F32}[P.dtype]
    check(tpo_convection_apply(P.data_ptr(), M.data_ptr(), D_vq.data_ptr(), I_vq.data_ptr(),
                               F.data_ptr(), nv, nq, e, dtype,
                               torch.cuda.current_stream().cuda_stream), "tpo_convection_apply")
    return F


def apply_aniso_tensors(u, S_x, S_y, S_z, D, v=None):
    """The operator on anisotropic elements over torch device tensors (``u``, ``D``
    ``[E,nx,ny,nz]``; ``S_x`` ``[nx,nx]``, ``S_y`` ``[ny,ny]``, ``S_z`` ``[nz,nz]``);
    marshalling only."""
    import torch

    if u.dim() != 4 or not u.is_cuda or tuple(D.shape) != tuple(u.shape):
        raise ValueError("u and D must be device tensors of shape [E,nx,ny,nz]")
    for x in (u, S_x, S_y, S_z, D):
        if not x.is_contiguous() or x.dtype != u.dtype or not x.is_cuda:
            raise ValueError("all tensors must be contiguous device tensors of one dtype")
    e, nx, ny, nz = u.shape
    for s, n in ((S_x, nx), (S_y, ny), (S_z, nz)):
        if tuple(s.shape) != (n, n):
            raise ValueError("S matrices must be [nx,nx], [ny,ny], [nz,nz]")
    if v is None:
        v = torch.empty_like(u)
    elif (tuple(v.shape) != tuple(u.shape) or v.dtype != u.dtype or not v.is_contiguous()
          or not v.is_cuda):
        raise ValueError("v must match u")
    dtype = {torch.float64: TPO_F64, torch.float32: TPO_F32}[u.dtype]
    check(tpo_ihelm_apply_aniso(u.data_ptr(), S_x.data_ptr(), S_y.data_ptr(), S_z.data_ptr(),
                                D.data_ptr(), v.data_ptr(), nx, ny, nz, e, dtype,
                                torch.cuda.current_stream().cuda_stream), "tpo_ihelm_apply_aniso")
    return v

"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol
the header declares, and validates arguments before touching the device."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2604_19906_amd import tpo


def declared_functions(repo_root, header="tpo.h"):
    text = open(os.path.join(repo_root, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tpo_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(repo_root):
    names = declared_functions(repo_root)
    assert {"tpo_create", "tpo_destroy", "tpo_ihelm_apply", "tpo_status_string"} <= set(names)
    l = tpo.lib()
    for name in names:
        assert hasattr(l, name), f"{name} declared in tpo.h but not exported"
    # every header under include/ has its library: the measurement aid lives in its own
    assert sorted(os.listdir(os.path.join(repo_root, "include"))) == ["tpo.h", "tpo_bench.h"]
    aid = declared_functions(repo_root, "tpo_bench.h")
    assert aid == ["tpo_stream_scale"]
    for name in aid:
        assert hasattr(tpo.bench_lib(), name), f"{name} declared in tpo_bench.h but not exported"
        assert not hasattr(l, name), f"{name} belongs to libtpo_bench.so, not to the operator library"


def test_status_strings():
    for s in (0, -1, -2, -3, -4, -5):
        assert len(tpo.status_string(s)) > 1
    assert tpo.status_string(0) == "ok"
    assert "unknown" in tpo.status_string(-99)


def _buf(nbytes):
    a = np.zeros(nbytes // 8 + 2, dtype=np.float64)
    return a, a.ctypes.data


def test_argument_validation_precedes_any_device_use():
    # Host addresses stand in for device pointers: validation only looks at their values.
    n, e = 4, 10
    keep, p = [], []
    for _ in range(6):
        a, addr = _buf(e * n ** 3 * 8)
        keep.append(a)
        p.append(addr)
    u, sx, sy, sz, d, v = p
    ap = tpo.tpo_ihelm_apply
    assert ap(u, sx, sy, sz, d, v, 0, e, tpo.TPO_F64, None) == tpo.TPO_ERR_INVALID_ARG
    assert ap(u, sx, sy, sz, d, v, -3, e, tpo.TPO_F64, None) == tpo.TPO_ERR_INVALID_ARG
    assert ap(u, sx, sy, sz, d, v, n, -1, tpo.TPO_F64, None) == tpo.TPO_ERR_INVALID_ARG
    assert ap(u, sx, sy, sz, d, v, n, e, 7, None) == tpo.TPO_ERR_INVALID_ARG
    assert ap(u, sx, sy, sz, d, v, 17, e, tpo.TPO_F64, None) == tpo.TPO_ERR_UNSUPPORTED
    assert ap(u, sx, sy, sz, d, v, 1000, e, tpo.TPO_F32, None) == tpo.TPO_ERR_UNSUPPORTED
    for k in range(6):
        q = list(p)
        q[k] = None
        assert ap(*q, n, e, tpo.TPO_F64, None) == tpo.TPO_ERR_INVALID_ARG
    # misaligned pointer
    assert ap(u + 4, sx, sy, sz, d, v, n, e, tpo.TPO_F64, None) == tpo.TPO_ERR_INVALID_ARG
    assert ap(u + 2, sx, sy, sz, d, v, n, e, tpo.TPO_F32, None) == tpo.TPO_ERR_INVALID_ARG
    # aliasing: partial overlap with u, any overlap with D or S
    assert ap(u, sx, sy, sz, d, u + 8, n, e, tpo.TPO_F64, None) == tpo.TPO_ERR_ALIAS
    assert ap(u, sx, sy, sz, d, d, n, e, tpo.TPO_F64, None) == tpo.TPO_ERR_ALIAS
    assert ap(u, sx, sy, sz, d, d + 64, n, e, tpo.TPO_F64, None) == tpo.TPO_ERR_ALIAS
    assert ap(u, v + 16, sy, sz, d, v, n, e, tpo.TPO_F64, None) == tpo.TPO_ERR_ALIAS
    assert ap(u, sx, sy, v, d, v, n, e, tpo.TPO_F64, None) == tpo.TPO_ERR_ALIAS
    # unknown variant
    assert tpo.tpo_ihelm_apply_variant(u, sx, sy, sz, d, v, n, e, tpo.TPO_F64, None, 9) \
        == tpo.TPO_ERR_INVALID_ARG
    # empty batch is a no-op, even with NULL data pointers
    assert ap(None, None, None, None, None, None, n, 0, tpo.TPO_F64, None) == tpo.TPO_OK


def test_valid_call_without_create_reports_not_initialized():
    import torch
    if torch.cuda.is_available():
        pytest.skip("covered by the GPU tests")
    n, e = 3, 2
    keep, p = [], []
    for _ in range(6):
        a, addr = _buf(e * n ** 3 * 8)
        keep.append(a)
        p.append(addr)
    # in-place (v == u) passes the alias check; without a device nothing is launched
    rc = tpo.tpo_ihelm_apply(p[0], p[1], p[2], p[3], p[4], p[0], n, e, tpo.TPO_F64, None)
    assert rc == tpo.TPO_ERR_NOT_INITIALIZED
    assert tpo.tpo_destroy() == tpo.TPO_ERR_NOT_INITIALIZED
    assert tpo.tpo_create() == tpo.TPO_ERR_DEVICE


def test_sep_argument_validation():
    n, e = 4, 10
    keep, p = [], []
    for _ in range(9):
        a, addr = _buf(e * n ** 3 * 8)
        keep.append(a)
        p.append(addr)
    u, sx, sy, sz, lx, ly, lz, mu, v = p
    ap = tpo.tpo_ihelm_apply_sep
    assert ap(u, sx, sy, sz, lx, ly, lz, mu, v, 0, e, tpo.TPO_F64, None) == tpo.TPO_ERR_INVALID_ARG
    assert ap(u, sx, sy, sz, lx, ly, lz, mu, v, n, -1, tpo.TPO_F64, None) == tpo.TPO_ERR_INVALID_ARG
    assert ap(u, sx, sy, sz, lx, ly, lz, mu, v, n, e, 3, None) == tpo.TPO_ERR_INVALID_ARG
    assert ap(u, sx, sy, sz, lx, ly, lz, mu, v, 17, e, tpo.TPO_F64, None) == tpo.TPO_ERR_UNSUPPORTED
    for k in range(9):
        q = list(p)
        q[k] = None
        assert ap(*q, n, e, tpo.TPO_F64, None) == tpo.TPO_ERR_INVALID_ARG
    assert ap(u, sx, sy, sz, lx + 4, ly, lz, mu, v, n, e, tpo.TPO_F64, None) == tpo.TPO_ERR_INVALID_ARG
    # aliasing: v may be u exactly, nothing else
    assert ap(u, sx, sy, sz, lx, ly, lz, mu, u + 8, n, e, tpo.TPO_F64, None) == tpo.TPO_ERR_ALIAS
    assert ap(u, sx, sy, sz, lx, ly, lz, v + 8, v, n, e, tpo.TPO_F64, None) == tpo.TPO_ERR_ALIAS
    assert ap(u, sx, sy, sz, v, ly, lz, mu, v, n, e, tpo.TPO_F64, None) == tpo.TPO_ERR_ALIAS
    assert ap(u, sx, v + 16, sz, lx, ly, lz, mu, v, n, e, tpo.TPO_F64, None) == tpo.TPO_ERR_ALIAS
    # valid arguments, E = 0: no-op; E > 0 without a device: not initialised
    assert ap(u, sx, sy, sz, lx, ly, lz, mu, v, n, 0, tpo.TPO_F64, None) == tpo.TPO_OK
    assert ap(u, sx, sy, sz, lx, ly, lz, mu, u, n, e, tpo.TPO_F64, None) == tpo.TPO_ERR_NOT_INITIALIZED
    assert tpo.tpo_ihelm_apply_sep_variant(u, sx, sy, sz, lx, ly, lz, mu, v, n, e, tpo.TPO_F64,
                                           None, 9) == tpo.TPO_ERR_INVALID_ARG
    assert tpo.tpo_ihelm_apply_sep_variant(u, sx, sy, sz, lx, ly, lz, mu, v, n, e, tpo.TPO_F64,
                                           None, tpo.TPO_VARIANT_PENCIL_MM) == tpo.TPO_ERR_UNSUPPORTED


def test_transform_argument_validation():
    n, e = 4, 10
    keep, p = [], []
    for _ in range(5):
        a, addr = _buf(e * n ** 3 * 8)
        keep.append(a)
        p.append(addr)
    u, sx, sy, sz, t = p
    ap = tpo.tpo_transform_apply
    F = tpo.TPO_FORWARD
    assert ap(u, sx, sy, sz, t, 0, e, tpo.TPO_F64, F, None) == tpo.TPO_ERR_INVALID_ARG
    assert ap(u, sx, sy, sz, t, n, -2, tpo.TPO_F64, F, None) == tpo.TPO_ERR_INVALID_ARG
    assert ap(u, sx, sy, sz, t, n, e, 9, F, None) == tpo.TPO_ERR_INVALID_ARG
    assert ap(u, sx, sy, sz, t, n, e, tpo.TPO_F64, 5, None) == tpo.TPO_ERR_INVALID_ARG
    assert ap(u, sx, sy, sz, t, 17, e, tpo.TPO_F32, F, None) == tpo.TPO_ERR_UNSUPPORTED
    for k in range(5):
        q = list(p)
        q[k] = None
        assert ap(*q, n, e, tpo.TPO_F64, F, None) == tpo.TPO_ERR_INVALID_ARG
    assert ap(u + 4, sx, sy, sz, t, n, e, tpo.TPO_F64, F, None) == tpo.TPO_ERR_INVALID_ARG
    assert ap(u, sx, sy, sz, u + 8, n, e, tpo.TPO_F64, F, None) == tpo.TPO_ERR_ALIAS
    assert ap(u, sx, t + 8, sz, t, n, e, tpo.TPO_F64, tpo.TPO_BACKWARD, None) == tpo.TPO_ERR_ALIAS
    assert ap(u, sx, sy, sz, t, n, 0, tpo.TPO_F64, F, None) == tpo.TPO_OK
    assert ap(u, sx, sy, sz, u, n, e, tpo.TPO_F64, F, None) == tpo.TPO_ERR_NOT_INITIALIZED


def test_convection_argument_validation():
    n, e = 3, 4
    keep, p = [], []
    for size in (9 * e * n ** 3 * 8, e * n ** 3 * 8, n * n * 8, n * n * 8, 3 * e * n ** 3 * 8):
        a, addr = _buf(size)
        keep.append(a)
        p.append(addr)
    pp, m, d, i, f = p
    ap = tpo.tpo_convection_apply
    assert ap(pp, m, d, i, f, 0, n, e, tpo.TPO_F64, None) == tpo.TPO_ERR_INVALID_ARG
    assert ap(pp, m, d, i, f, n, n, -1, tpo.TPO_F64, None) == tpo.TPO_ERR_INVALID_ARG
    assert ap(pp, m, d, i, f, n, n, e, 2, None) == tpo.TPO_ERR_INVALID_ARG
    assert ap(pp, m, d, i, f, 17, 17, e, tpo.TPO_F64, None) == tpo.TPO_ERR_UNSUPPORTED
    assert ap(pp, m, d, i, f, n, 16, e, tpo.TPO_F64, None) == tpo.TPO_ERR_UNSUPPORTED   # no such shape
    assert tpo.tpo_convection_has_shape(3, 3, tpo.TPO_F64) and tpo.tpo_convection_has_shape(3, 4, tpo.TPO_F32)
    assert tpo.tpo_convection_has_shape(8, 12, tpo.TPO_F64)
    assert not tpo.tpo_convection_has_shape(3, 16, tpo.TPO_F64)
    assert not tpo.tpo_convection_has_shape(4, 3, tpo.TPO_F64)
    assert not tpo.tpo_convection_has_shape(17, 17, tpo.TPO_F64)
    for k in range(5):
        q = list(p)
        q[k] = None
        assert ap(*q, n, n, e, tpo.TPO_F64, None) == tpo.TPO_ERR_INVALID_ARG
    assert ap(pp + 4, m, d, i, f, n, n, e, tpo.TPO_F64, None) == tpo.TPO_ERR_INVALID_ARG
    assert ap(pp, m, d, i, pp + 64, n, n, e, tpo.TPO_F64, None) == tpo.TPO_ERR_ALIAS
    assert ap(pp, m, d, i, m, n, n, e, tpo.TPO_F64, None) == tpo.TPO_ERR_ALIAS
    assert ap(pp, m, f + 8, i, f, n, n, e, tpo.TPO_F64, None) == tpo.TPO_ERR_ALIAS
    assert ap(pp, m, d, i, f, n, n, 0, tpo.TPO_F64, None) == tpo.TPO_OK
    assert ap(pp, m, d, i, f, n, n, e, tpo.TPO_F64, None) == tpo.TPO_ERR_NOT_INITIALIZED


def test_aniso_argument_validation():
    keep, p = [], []
    for _ in range(6):
        a, addr = _buf(10 * 4 * 5 * 6 * 8)
        keep.append(a)
        p.append(addr)
    u, sx, sy, sz, d, v = p
    ap = tpo.tpo_ihelm_apply_aniso
    assert ap(u, sx, sy, sz, d, v, 4, 0, 6, 10, tpo.TPO_F64, None) == tpo.TPO_ERR_INVALID_ARG
    assert ap(u, sx, sy, sz, d, v, 4, 5, 17, 10, tpo.TPO_F64, None) == tpo.TPO_ERR_UNSUPPORTED
    assert ap(u, sx, sy, sz, d, v, 4, 5, 6, -1, tpo.TPO_F64, None) == tpo.TPO_ERR_INVALID_ARG
    assert ap(u, sx, sy, sz, d, v, 4, 5, 6, 10, 4, None) == tpo.TPO_ERR_INVALID_ARG
    assert ap(None, sx, sy, sz, d, v, 4, 5, 6, 10, tpo.TPO_F64, None) == tpo.TPO_ERR_INVALID_ARG
    assert ap(u, sx, sy, sz, d, d, 4, 5, 6, 10, tpo.TPO_F64, None) == tpo.TPO_ERR_ALIAS
    assert ap(u, sx, sy, sz, d, v, 4, 5, 6, 0, tpo.TPO_F64, None) == tpo.TPO_OK
    assert ap(u, sx, sy, sz, d, u, 4, 5, 6, 10, tpo.TPO_F64, None) == tpo.TPO_ERR_NOT_INITIALIZED
    # cubic shapes are tpo_ihelm_apply
    assert ap(u, sx, sy, sz, d, v, 17, 17, 17, 10, tpo.TPO_F64, None) == tpo.TPO_ERR_UNSUPPORTED


def test_sep_variant_queries():
    for dt in (tpo.TPO_F64, tpo.TPO_F32):
        for n in range(1, tpo.TPO_MAX_N + 1):
            var = tpo.tpo_ihelm_sep_variant_for(n, dt)
            assert var in (tpo.TPO_VARIANT_PENCIL, tpo.TPO_VARIANT_PENCIL_MM, tpo.TPO_VARIANT_MFMA)
            assert tpo.tpo_ihelm_sep_has_variant(n, dt, var)
            assert tpo.tpo_ihelm_sep_has_variant(n, dt, tpo.TPO_VARIANT_AUTO)
            assert tpo.tpo_ihelm_sep_has_variant(n, dt, tpo.TPO_VARIANT_PENCIL)
            assert tpo.tpo_ihelm_sep_has_variant(n, dt, tpo.TPO_VARIANT_MFMA)
            assert tpo.tpo_ihelm_sep_has_variant(n, dt, tpo.TPO_VARIANT_PENCIL_MM) == (dt == tpo.TPO_F32)
    # the separable form follows the D form's choice of family, batch-aware query included
    assert tpo.tpo_ihelm_sep_variant_for_batch(16, tpo.TPO_F64, True, 65536) == tpo.TPO_VARIANT_MFMA
    assert tpo.tpo_ihelm_sep_variant_for_batch(16, tpo.TPO_F64, False, 65536) == tpo.TPO_VARIANT_PENCIL
    assert tpo.tpo_ihelm_sep_variant_for_batch(15, tpo.TPO_F32, False, 65536) == tpo.TPO_VARIANT_MFMA
    assert tpo.tpo_ihelm_sep_variant_for_batch(13, tpo.TPO_F32, False, 65536) == tpo.TPO_VARIANT_PENCIL_MM
    assert tpo.tpo_ihelm_sep_variant_for_batch(13, tpo.TPO_F32, False, -2) == tpo.TPO_ERR_INVALID_ARG
    for n in range(1, 17):
        for dt in (tpo.TPO_F64, tpo.TPO_F32):
            assert tpo.tpo_ihelm_sep_variant_for_batch(n, dt, False, 1 << 22) \
                == tpo.tpo_ihelm_sep_variant_for(n, dt)
    assert tpo.tpo_ihelm_sep_variant_for(17, tpo.TPO_F64) == tpo.TPO_ERR_UNSUPPORTED
    assert tpo.tpo_ihelm_sep_variant_for(0, tpo.TPO_F32) == tpo.TPO_ERR_INVALID_ARG


def test_variant_queries():
    for dt in (tpo.TPO_F64, tpo.TPO_F32):
        for n in range(1, tpo.TPO_MAX_N + 1):
            for shared in (False, True):
                var = tpo.tpo_ihelm_variant_for(n, dt, shared)
                assert var in (tpo.TPO_VARIANT_PENCIL, tpo.TPO_VARIANT_MFMA,
                               tpo.TPO_VARIANT_PENCIL_MM)
                assert tpo.tpo_ihelm_has_variant(n, dt, var)
            assert tpo.tpo_ihelm_has_variant(n, dt, tpo.TPO_VARIANT_PENCIL)
            assert tpo.tpo_ihelm_has_variant(n, dt, tpo.TPO_VARIANT_AUTO)
            # the 4x4x1 matrix-core pencil kernels exist for fp32 only
            assert tpo.tpo_ihelm_has_variant(n, dt, tpo.TPO_VARIANT_PENCIL_MM) == (dt == tpo.TPO_F32)
    assert tpo.tpo_ihelm_variant_for(17, tpo.TPO_F64) == tpo.TPO_ERR_UNSUPPORTED
    assert tpo.tpo_ihelm_variant_for(0, tpo.TPO_F64) == tpo.TPO_ERR_INVALID_ARG
    assert tpo.tpo_ihelm_variant_for(4, 5) == tpo.TPO_ERR_INVALID_ARG
    # the batch-aware query: equal to the plain one for large batches; fp64 n=16 with a shared
    # matrix takes the pencil kernels around the paper's batch of 8192 elements
    for dt in (tpo.TPO_F64, tpo.TPO_F32):
        for n in range(1, 17):
            for shared in (False, True):
                assert tpo.tpo_ihelm_variant_for_batch(n, dt, shared, 1 << 22) \
                    == tpo.tpo_ihelm_variant_for(n, dt, shared)
    assert tpo.tpo_ihelm_variant_for_batch(16, tpo.TPO_F64, True, 8192) == tpo.TPO_VARIANT_MFMA
    assert tpo.tpo_ihelm_variant_for_batch(16, tpo.TPO_F64, True, 65536) == tpo.TPO_VARIANT_MFMA
    assert tpo.tpo_ihelm_variant_for_batch(16, tpo.TPO_F64, False, 8192) == tpo.TPO_VARIANT_PENCIL
    assert tpo.tpo_ihelm_variant_for_batch(4, tpo.TPO_F64, True, -1) == tpo.TPO_ERR_INVALID_ARG
    assert not tpo.tpo_ihelm_has_variant(17, tpo.TPO_F64, tpo.TPO_VARIANT_PENCIL)

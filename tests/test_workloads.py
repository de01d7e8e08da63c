"""Seeded input generators: determinism, block regeneration, shapes and distributions."""
import numpy as np
import pytest

from paper_2604_19906_amd import workloads as wl


def test_named_configs():
    c = wl.CONFIGS
    assert [(w.dtype, w.n, w.num_elems) for w in c] == [
        ("f64", 7, 1000), ("f64", 8, 131072), ("f64", 11, 262144),
        ("f64", 16, 65536), ("f32", 13, 1048576)]
    assert c[2].u_dist == "normal" and c[4].distinct_s and not c[0].distinct_s
    assert c[2].flop_per_elem == 12 * 11 ** 4 + 11 ** 3
    assert c[2].bytes_per_elem == 3 * 1331 * 8


def test_deterministic_and_block_regenerable():
    w = wl.custom(5, 3 * wl.BLOCK + 17, "f64", key=11)
    a = wl.field_u(w, 4000, 4200)
    b = wl.field_u(w)[4000:4200]
    assert np.array_equal(a, b)
    d1 = wl.diagonal_d(w, wl.BLOCK - 3, wl.BLOCK + 5)
    d2 = wl.diagonal_d(w)[wl.BLOCK - 3:wl.BLOCK + 5]
    assert np.array_equal(d1, d2)
    assert np.array_equal(wl.shifts(w, 10, 20), wl.shifts(w)[10:20])
    assert wl.field_u(w, 7, 7).shape == (0, 5, 5, 5)


def test_direction_matrices_orthogonal_nonsymmetric():
    for w in (wl.CONFIGS[0], wl.CONFIGS[2], wl.CONFIGS[3]):
        sx, sy, sz = wl.direction_matrices(w)
        assert sx is sy and sy is sz
        assert np.allclose(sx.T @ sx, np.eye(w.n), atol=1e-13)
        assert not np.allclose(sx, sx.T)
    w = wl.CONFIGS[4]
    sx, sy, sz = wl.direction_matrices(w)
    assert sx.dtype == np.float32 and not np.array_equal(sx, sy) and not np.array_equal(sy, sz)
    assert np.allclose(sx.astype(np.float64).T @ sx.astype(np.float64), np.eye(13), atol=1e-6)


def test_value_ranges():
    w = wl.CONFIGS[0]
    u, sx, sy, sz, d = wl.make_inputs(w)
    assert u.shape == (1000, 7, 7, 7) and u.flags.c_contiguous and d.flags.c_contiguous
    assert -1 <= u.min() < -0.99 and 0.99 < u.max() <= 1
    assert d.min() > 1 / 31.0 and d.max() < 1 / 0.3
    w2 = wl.custom(11, 64, "f64", key=2, u_dist="normal")
    un = wl.field_u(w2)
    assert abs(un.mean()) < 0.02 and abs(un.std() - 1) < 0.02
    w4 = wl.custom(13, 8, "f32", key=4)
    u4, *_rest, d4 = wl.make_inputs(w4)
    assert u4.dtype == np.float32 and d4.dtype == np.float32


def test_sep_inputs_match_the_diagonal():
    # the separable-diagonal inputs are the numbers the D recipe is built from
    w = wl.custom(5, 9, "f64", key=11, distinct_s=True)
    lx, ly, lz, mu = wl.sep_inputs(w)
    d = wl.diagonal_d(w)
    want = 1.0 / (lx[None, :, None, None] + ly[None, None, :, None] + lz[None, None, None, :]
                  + mu[:, None, None, None])
    assert np.array_equal(d, want)
    lx2, _, _, mu2 = wl.sep_inputs(w, 3, 7)
    assert np.array_equal(mu2, mu[3:7]) and np.array_equal(lx2, lx)
    w32 = wl.custom(4, 3, "f32", key=12, distinct_s=False)
    l32 = wl.sep_inputs(w32)
    assert all(a.dtype == np.float32 for a in l32) and l32[0] is l32[1]


def test_convection_inputs():
    w = wl.conv_custom(6, 600, "f64", key=31)
    d, i = wl.conv_matrices(w)
    # interpolation reproduces constants, differentiation annihilates them and is exact on x
    assert np.allclose(i.sum(axis=1), 1.0) and np.allclose(d.sum(axis=1), 0.0, atol=1e-12)
    xq = -np.cos(np.pi * (2 * np.arange(6) + 1) / 12)
    xv = -np.cos(np.pi * np.arange(6) / 5)
    assert np.allclose(i @ xq ** 3, xv ** 3) and np.allclose(d @ xq ** 3, 3 * xv ** 2)
    p, m, _, _ = wl.conv_inputs(w, 250, 270)            # crosses a seed block
    assert p.shape == (3, 3, 20, 6, 6, 6) and m.shape == (20, 6, 6, 6)
    assert np.array_equal(p, wl.conv_flux(w)[:, :, 250:270])
    assert np.array_equal(m, wl.conv_metric(w)[250:270])
    assert m.min() >= 0.5 and m.max() <= 2.0 and np.abs(p).max() <= 1.0
    assert not np.array_equal(p[0, 0], p[0, 1]) and not np.array_equal(p[0, 0], p[1, 0])
    assert wl.conv_inputs(wl.conv_custom(4, 3, "f32"))[0].dtype == np.float32


def test_anisotropic_inputs():
    w = wl.ANISO_CONFIGS[0]
    u, sx, sy, sz, d = wl.aniso_inputs(w)
    assert u.shape == d.shape == (w.num_elems, *w.dims)
    for s, k in zip((sx, sy, sz), w.dims):
        assert s.shape == (k, k)
        assert np.allclose(s.T @ s, np.eye(k), atol=1e-13)
        assert not np.allclose(s, s.T)
    assert d.min() > 1 / 31.0 - 1e-12 and d.max() < 1 / 0.3
    assert np.abs(u).max() <= 1.0
    # any range of elements can be regenerated on its own, across seed blocks
    big = wl.aniso_custom((3, 4, 5), 9000, "f32", key=131)
    assert np.array_equal(wl.aniso_field_u(big, 4000, 4200), wl.aniso_field_u(big)[4000:4200])
    assert np.array_equal(wl.aniso_diagonal_d(big, 4000, 4200), wl.aniso_diagonal_d(big)[4000:4200])
    assert wl.aniso_field_u(big).dtype == np.float32
    assert w.bytes_per_elem == 3 * 5 * 6 * 7 * 8 and w.flop_per_elem == 210 * (4 * 18 + 1)

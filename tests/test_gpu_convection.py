"""GPU parity of the convection volume term (tpo_convection_apply, Eq. 1 of the paper) against
the CPU oracle on the same seeded inputs.  Error measure: per (component, element) cube,
max|F - F_ref| / max|F_ref|; bar 1e-12 (fp64) / 2e-5 (fp32)."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import TOL, dev
from paper_2604_19906_amd import tpo
from paper_2604_19906_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def library():
    assert torch.cuda.is_available(), "GPU tests need a device"
    tpo.check(tpo.tpo_create(), "tpo_create")
    yield
    tpo.check(tpo.tpo_destroy(), "tpo_destroy")


def cube_err(got, ref):
    """Worst over (c, e) of the max-norm relative error of one output cube."""
    g = np.asarray(got, dtype=np.float64).reshape(-1, *got.shape[2:])
    r = np.asarray(ref, dtype=np.float64).reshape(-1, *ref.shape[2:])
    return oracle.max_rel_err_per_element(g, r)


def run_convection(p, m, d, i):
    tf = tpo.convection_tensors(dev(p), dev(m), dev(d), dev(i))
    torch.cuda.synchronize()
    return tf.cpu().numpy()


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("n", list(range(1, 17)))
def test_convection_all_n_small_batches(n, dtype):
    for e in (1, 23, 70):
        w = wl.conv_custom(n, e, dtype, key=800 + n)
        p, m, d, i = wl.conv_inputs(w)
        print(f"case convection n={n} {dtype} E={e}", flush=True)
        got = run_convection(p, m, d, i)
        assert got.dtype == p.dtype and got.shape == (3, e, n, n, n)
        err = cube_err(got, oracle.convection_apply(p, m, d, i))
        assert err <= TOL[dtype], f"convection n={n} {dtype} E={e}: err {err:.3e}"


RECT_SHAPES = [(nv, nq) for nv in range(2, 13) for nq in sorted({nv + 1, nv + 2, (3 * nv + 1) // 2})
               if nq <= 16]


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("nv,nq", RECT_SHAPES)
def test_convection_rectangular_shapes(nv, nq, dtype):
    dt = tpo.TPO_F64 if dtype == "f64" else tpo.TPO_F32
    assert tpo.tpo_convection_has_shape(nv, nq, dt)
    for e in (1, 29):
        w = wl.conv_custom(nv, e, dtype, key=1000 + 20 * nv + nq, nq=nq)
        p, m, d, i = wl.conv_inputs(w)
        assert d.shape == (nv, nq) and m.shape == (e, nq, nq, nq)
        print(f"case convection nv={nv} nq={nq} {dtype} E={e}", flush=True)
        got = run_convection(p, m, d, i)
        assert got.shape == (3, e, nv, nv, nv)
        err = cube_err(got, oracle.convection_apply(p, m, d, i))
        assert err <= TOL[dtype], f"convection nv={nv} nq={nq} {dtype} E={e}: err {err:.3e}"


def test_convection_general_matrices_and_direct_form():
    # nothing in the kernel relies on D and I being a differentiation / interpolation pair
    rng = np.random.default_rng(99)
    n, e = 5, 9
    p = rng.uniform(-1, 1, (3, 3, e, n, n, n))
    m = rng.uniform(0.5, 2, (e, n, n, n))
    d, i = rng.standard_normal((n, n)), rng.standard_normal((n, n))
    got = run_convection(p, m, d, i)
    assert cube_err(got, oracle.convection_apply(p, m, d, i, direct=True)) <= 1e-12


def sample_spans(e):
    rng = np.random.default_rng(4242 + e)
    spans = [(0, min(128, e)), (max(0, e - 128), e)]
    for s in rng.integers(0, max(1, e - 64), 6):
        spans.append((int(s), int(min(e, s + 64))))
    return spans


@pytest.mark.parametrize("idx", [0, 1, 2, 3, 4])
def test_convection_full_size_configs(idx):
    w = wl.CONV_CONFIGS[idx]
    print(f"case convection {w.name}: generating", flush=True)
    tp, tm, td, ti = wl.conv_to_device(w)
    assert tpo.tpo_convection_has_shape(w.n, w.q, tpo.TPO_F64 if w.dtype == "f64" else tpo.TPO_F32)
    tf = torch.full((3, w.num_elems, w.n, w.n, w.n), float("nan"), dtype=tp.dtype, device="cuda")
    tpo.convection_tensors(tp, tm, td, ti, tf)
    torch.cuda.synchronize()
    d, i = wl.conv_matrices(w)
    worst = 0.0
    for lo, hi in sample_spans(w.num_elems):
        p, m = wl.conv_flux(w, lo, hi), wl.conv_metric(w, lo, hi)
        assert np.array_equal(p, tp[:, :, lo:hi].cpu().numpy())       # same inputs on both sides
        ref = oracle.convection_apply(p, m, d, i)
        worst = max(worst, cube_err(tf[:, lo:hi].cpu().numpy(), ref))
    assert worst <= TOL[w.dtype], f"{w.name}: sampled err {worst:.3e}"
    # every cube: nothing left unwritten, and agreement with a device einsum in fp64
    assert not torch.isnan(tf).any()
    d64, i64 = td.double(), ti.double()
    worst_all = 0.0
    step = 2048
    for lo in range(0, w.num_elems, step):
        hi = min(w.num_elems, lo + step)
        mp = tm[lo:hi].double()[None, None] * tp[:, :, lo:hi].double()
        ref = (torch.einsum("il,jm,kn,cenml->cekji", d64, i64, i64, mp[:, 0])
               + torch.einsum("il,jm,kn,cenml->cekji", i64, d64, i64, mp[:, 1])
               + torch.einsum("il,jm,kn,cenml->cekji", i64, i64, d64, mp[:, 2]))
        num = (tf[:, lo:hi].double() - ref).abs().flatten(2).max(dim=2).values
        den = ref.abs().flatten(2).max(dim=2).values
        worst_all = max(worst_all, float((num / den).max()))
    assert worst_all <= TOL[w.dtype], f"{w.name}: full err {worst_all:.3e}"
    print(f"  {w.name}: sampled {worst:.2e}, all cubes {worst_all:.2e}", flush=True)


def test_convection_golden_file(repo_root):
    import os
    path = os.path.join(repo_root, "tests", "golden", "convection_f64_nv3_nq4_E2.txt")
    want = np.array([float.fromhex(l) for l in open(path) if not l.startswith("#")])
    got = run_convection(*wl.conv_inputs(wl.conv_custom(3, 2, "f64", key=78, nq=4)))
    assert cube_err(got, want.reshape(got.shape)) <= 1e-12


def test_convection_status_codes_and_determinism():
    w = wl.conv_custom(6, 11, "f64", key=900)
    t = [dev(a) for a in wl.conv_inputs(w)]
    a = tpo.convection_tensors(*t)
    b = tpo.convection_tensors(*t)
    torch.cuda.synchronize()
    assert torch.equal(a, b)
    ptrs = [x.data_ptr() for x in t]
    out = torch.empty_like(a)
    ap = tpo.tpo_convection_apply
    assert ap(*ptrs, out.data_ptr(), 6, 6, 0, tpo.TPO_F64, None) == tpo.TPO_OK
    assert ap(*ptrs, out.data_ptr(), 6, 5, 11, tpo.TPO_F64, None) == tpo.TPO_ERR_UNSUPPORTED
    assert not tpo.tpo_convection_has_shape(6, 5, tpo.TPO_F64)
    assert ap(*ptrs, t[0].data_ptr(), 6, 6, 11, tpo.TPO_F64, None) == tpo.TPO_ERR_ALIAS

"""GPU parity of the operator on anisotropic elements (tpo_ihelm_apply_aniso, the kernel with
runtime sizes) against the CPU oracle.  Bar as for the cubic operator.  The batch sizes leave a
ragged last workgroup for every number of elements per workgroup."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import TOL, dev, oracle_every_element
from paper_2604_19906_amd import tpo
from paper_2604_19906_amd import workloads as wl

pytestmark = pytest.mark.gpu

SHAPES = [(1, 1, 2), (2, 1, 1), (2, 3, 4), (4, 3, 2), (5, 5, 7), (7, 5, 5), (3, 16, 2), (16, 1, 16),
          (8, 12, 10), (11, 13, 9), (16, 16, 15), (15, 16, 16), (16, 15, 16), (6, 6, 16),
          (4, 4, 5), (9, 8, 8), (12, 12, 13), (13, 12, 12), (1, 16, 16), (16, 16, 1), (11, 11, 12)]


@pytest.fixture(scope="module", autouse=True)
def library():
    assert torch.cuda.is_available(), "GPU tests need a device"
    tpo.check(tpo.tpo_create(), "tpo_create")
    yield
    tpo.check(tpo.tpo_destroy(), "tpo_destroy")


def aniso_inputs(dims, e, dtype, seed):
    """Seeded inputs: orthogonal S per axis (sizes differ), positive D, uniform u."""
    rng = np.random.default_rng([19906, 77, seed])
    npdt = np.float64 if dtype == "f64" else np.float32
    mats = [wl.orthogonal_matrix(n, rng).astype(npdt) for n in dims]
    u = rng.uniform(-1, 1, (e, *dims)).astype(npdt)
    d = rng.uniform(0.03, 3.3, (e, *dims)).astype(npdt)
    return u, mats[0], mats[1], mats[2], d


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("dims", SHAPES)
def test_aniso_shapes(dims, dtype):
    for e in (1, 37, 203):
        u, sx, sy, sz, d = aniso_inputs(dims, e, dtype, 100 * dims[0] + 10 * dims[1] + dims[2])
        print(f"case aniso dims={dims} {dtype} E={e}", flush=True)
        got = tpo.apply_aniso_tensors(*map(dev, (u, sx, sy, sz, d)))
        torch.cuda.synchronize()
        got = got.cpu().numpy()
        assert got.dtype == u.dtype and got.shape == u.shape
        err = oracle.max_rel_err_per_element(got, oracle.ihelm_apply_aniso(u, sx, sy, sz, d))
        assert err <= TOL[dtype], f"aniso {dims} {dtype} E={e}: err {err:.3e}"


def test_aniso_cubic_shapes_take_the_tuned_kernels():
    w = wl.custom(9, 50, "f64", key=1400, distinct_s=True)
    u, sx, sy, sz, d = wl.make_inputs(w)
    t = list(map(dev, (u, sx, sy, sz, d)))
    a = tpo.apply_aniso_tensors(*t)
    b = tpo.apply_tensors(*t)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


def test_aniso_large_batch_in_place_and_status_codes():
    dims, e = (10, 12, 14), 20000
    u, sx, sy, sz, d = aniso_inputs(dims, e, "f64", 5)
    t = list(map(dev, (u, sx, sy, sz, d)))
    tpo.apply_aniso_tensors(*t, v=t[0])                     # v == u
    torch.cuda.synchronize()
    got = t[0].cpu().numpy()
    idx = np.r_[0:64, e - 64:e, np.random.default_rng(3).integers(0, e, 128)]
    ref = oracle.ihelm_apply_aniso(u[idx], sx, sy, sz, d[idx])
    assert oracle.max_rel_err_per_element(got[idx], ref) <= 1e-12
    # every element against a device einsum
    t64 = [dev(a) for a in (u, sx, sy, sz, d)]
    fw = torch.einsum("li,mj,qk,elmq->eijk", t64[1], t64[2], t64[3], t64[0])
    full = torch.einsum("il,jm,kq,elmq->eijk", t64[1], t64[2], t64[3], t64[4] * fw)
    num = (t[0] - full).abs().flatten(1).max(dim=1).values
    den = full.abs().flatten(1).max(dim=1).values
    assert float((num / den).max()) <= 1e-12
    ptrs = [x.data_ptr() for x in t64]
    out = torch.empty_like(t64[0])
    ap = tpo.tpo_ihelm_apply_aniso
    assert ap(*ptrs, out.data_ptr(), 10, 12, 17, e, tpo.TPO_F64, None) == tpo.TPO_ERR_UNSUPPORTED
    assert ap(*ptrs, out.data_ptr(), 10, 0, 14, e, tpo.TPO_F64, None) == tpo.TPO_ERR_INVALID_ARG
    assert ap(*ptrs, out.data_ptr(), 10, 12, 14, 0, tpo.TPO_F64, None) == tpo.TPO_OK
    assert ap(*ptrs[:4], ptrs[4], ptrs[4], 10, 12, 14, e, tpo.TPO_F64, None) == tpo.TPO_ERR_ALIAS


# the named anisotropic workloads at full size, as the benchmark launches them: every element
# against the oracle (its anisotropic function is single-threaded, so blocks run in a pool)
@pytest.mark.parametrize("idx", [0, 1, 2, 3])
def test_aniso_named_workloads(idx):
    w = wl.ANISO_CONFIGS[idx]
    print(f"case {w.name}: generating", flush=True)
    tu, tsx, tsy, tsz, td = wl.aniso_to_device(w)
    tv = torch.full_like(tu, float("nan"))
    tpo.apply_aniso_tensors(tu, tsx, tsy, tsz, td, v=tv)
    torch.cuda.synchronize()
    assert not torch.isnan(tv).any()
    print(f"case {w.name}: oracle over all {w.num_elems} elements", flush=True)
    worst = oracle_every_element(
        w.num_elems,
        lambda lo, hi: wl.aniso_inputs(w, lo, hi),
        lambda lo, hi: (tu[lo:hi], None, None, None, td[lo:hi]),
        oracle.ihelm_apply_aniso, {"aniso": tv}, TOL[w.dtype], w.name,
        block=4096, workers=14, oracle_in_pool=True)
    print(f"  {w.name}: all elements {worst['aniso']:.2e}", flush=True)

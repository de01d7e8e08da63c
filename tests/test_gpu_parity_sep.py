"""GPU parity of the separable-diagonal form (tpo_ihelm_apply_sep), called through the C ABI,
against the CPU oracle on the same seeded inputs.  Same bar as the D form: max-norm relative
error per element <= 1e-12 (fp64) / 2e-5 (fp32).  In fp32 both sides start from the same
fp32-rounded lam and mu; the kernel then sums and divides in fp32, the oracle in fp64."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import TOL, VARIANTS, dev, oracle_every_element
from paper_2604_19906_amd import tpo
from paper_2604_19906_amd import workloads as wl

pytestmark = pytest.mark.gpu

DT = {"f64": tpo.TPO_F64, "f32": tpo.TPO_F32}


@pytest.fixture(scope="module", autouse=True)
def library():
    assert torch.cuda.is_available(), "GPU tests need a device"
    tpo.check(tpo.tpo_create(), "tpo_create")
    yield
    tpo.check(tpo.tpo_destroy(), "tpo_destroy")


def sep_variants_for(n, dtype):
    return [name for name, var in VARIANTS.items()
            if tpo.tpo_ihelm_sep_has_variant(n, DT[dtype], var)]


def run_sep(u, sx, sy, sz, lx, ly, lz, mu, variant=tpo.TPO_VARIANT_AUTO):
    t = [dev(a) for a in (u, sx, sy, sz, lx, ly, lz, mu)]
    tv = tpo.apply_sep_tensors(*t, variant=variant)
    torch.cuda.synchronize()
    return tv.cpu().numpy()


def check_sep(w, variant_name, lo=0, hi=None):
    u, sx, sy, sz, _ = wl.make_inputs(w, lo, hi)
    lx, ly, lz, mu = wl.sep_inputs(w, lo, hi)
    got = run_sep(u, sx, sy, sz, lx, ly, lz, mu, VARIANTS[variant_name])
    ref = oracle.ihelm_apply_sep(u, sx, sy, sz, lx, ly, lz, mu)
    assert got.dtype == u.dtype and got.shape == u.shape
    err = oracle.max_rel_err_per_element(got, ref)
    assert err <= TOL[w.dtype], f"{w.name} sep {variant_name}: err {err:.3e}"
    return err


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("n", list(range(1, 17)))
def test_sep_all_n_small_batches(n, dtype):
    names = sep_variants_for(n, dtype)
    assert "pencil" in names
    for name in names:
        for e in (1, 67, 203):
            w = wl.custom(n, e, dtype, key=300 + n, distinct_s=True)
            print(f"case sep n={n} {dtype} E={e} variant={name}", flush=True)
            check_sep(w, name)
        w = wl.custom(n, 131, dtype, key=350 + n, distinct_s=False)
        print(f"case sep n={n} {dtype} E=131 shared S variant={name}", flush=True)
        check_sep(w, name)


def test_sep_config0_all_elements_and_default_entry_point():
    w = wl.CONFIGS[0]
    for name in sep_variants_for(w.n, w.dtype):
        check_sep(w, name)
    u, sx, _, _, _ = wl.make_inputs(w)
    lx, _, _, mu = wl.sep_inputs(w)
    tu, ts, tl, tm = dev(u), dev(sx), dev(lx), dev(mu)
    tv = torch.empty_like(tu)
    rc = tpo.tpo_ihelm_apply_sep(tu.data_ptr(), ts.data_ptr(), ts.data_ptr(), ts.data_ptr(),
                                 tl.data_ptr(), tl.data_ptr(), tl.data_ptr(), tm.data_ptr(),
                                 tv.data_ptr(), w.n, w.num_elems, tpo.TPO_F64,
                                 torch.cuda.current_stream().cuda_stream)
    assert rc == tpo.TPO_OK
    torch.cuda.synchronize()
    ref = oracle.ihelm_apply_sep(u, sx, sx, sx, lx, lx, lx, mu)
    assert oracle.max_rel_err_per_element(tv.cpu().numpy(), ref) <= 1e-12


def test_sep_fp64_agrees_with_the_d_form_to_a_few_ulp():
    # same family, D built by the same expression with IEEE division: the kernel's reciprocal
    # is within 2 ulp of it, which six orthogonal mode products cannot amplify
    for n in (5, 8, 11, 16):
        w = wl.custom(n, 97, "f64", key=400 + n, distinct_s=True)
        u, sx, sy, sz, d = wl.make_inputs(w)
        lx, ly, lz, mu = wl.sep_inputs(w)
        t = [dev(a) for a in (u, sx, sy, sz)]
        a = tpo.apply_tensors(*t, dev(d), variant=tpo.TPO_VARIANT_PENCIL)
        b = tpo.apply_sep_tensors(*t, dev(lx), dev(ly), dev(lz), dev(mu),
                                  variant=tpo.TPO_VARIANT_PENCIL)
        torch.cuda.synchronize()
        err = oracle.max_rel_err_per_element(b.cpu().numpy(), a.cpu().numpy())
        assert err <= 4 * np.finfo(np.float64).eps, f"n={n}: {err:.3e}"


# the four large configurations at full size, in the launch configuration the benchmark uses;
# the oracle checks every element of every family's result
@pytest.mark.parametrize("idx", [1, 2, 3, 4])
def test_sep_full_size_configs(idx):
    w = wl.CONFIGS[idx]
    print(f"case sep {w.name}: generating", flush=True)
    tu, tsx, tsy, tsz = wl.to_device(w, with_d=False)
    lx, ly, lz, mu = wl.sep_inputs(w)
    tlx, tly, tlz, tmu = dev(lx), dev(ly), dev(lz), dev(mu)
    sx, sy, sz = wl.direction_matrices(w)
    outs = {}
    for name in sep_variants_for(w.n, w.dtype) + ["auto"]:
        print(f"case sep {w.name} variant={name}", flush=True)
        tv = torch.full_like(tu, float("nan"))
        tpo.apply_sep_tensors(tu, tsx, tsy, tsz, tlx, tly, tlz, tmu, tv,
                              variant=tpo.TPO_VARIANT_AUTO if name == "auto" else VARIANTS[name])
        torch.cuda.synchronize()
        assert not torch.isnan(tv).any()
        outs[name] = tv
    print(f"case sep {w.name}: oracle over all {w.num_elems} elements", flush=True)
    worst = oracle_every_element(
        w.num_elems,
        lambda lo, hi: (wl.field_u(w, lo, hi), sx, sy, sz, lx, ly, lz, mu[lo:hi]),
        lambda lo, hi: (tu[lo:hi], None, None, None, None, None, None, tmu[lo:hi]),
        oracle.ihelm_apply_sep, outs, TOL[w.dtype], "sep " + w.name)
    print(f"  {w.name} sep: " + ", ".join(f"{k} {v:.2e}" for k, v in worst.items()), flush=True)


def test_sep_in_place_ragged_and_status_codes():
    w = wl.custom(7, 45, "f64", key=500, distinct_s=True)
    u, sx, sy, sz, _ = wl.make_inputs(w)
    lx, ly, lz, mu = wl.sep_inputs(w)
    ref = oracle.ihelm_apply_sep(u, sx, sy, sz, lx, ly, lz, mu)
    t = [dev(a) for a in (u, sx, sy, sz, lx, ly, lz, mu)]
    tpo.apply_sep_tensors(*t, v=t[0])                     # v == u
    torch.cuda.synchronize()
    assert oracle.max_rel_err_per_element(t[0].cpu().numpy(), ref) <= 1e-12
    # a family without a kernel for the type (the 4x4x1 kernels are fp32 only)
    ptrs = [x.data_ptr() for x in t]
    tv = torch.empty_like(t[0])
    rc = tpo.tpo_ihelm_apply_sep_variant(*ptrs, tv.data_ptr(), 7, 45, tpo.TPO_F64, None,
                                         tpo.TPO_VARIANT_PENCIL_MM)
    assert rc == tpo.TPO_ERR_UNSUPPORTED
    # every family that has a D form has the separable form too
    for var in (tpo.TPO_VARIANT_PENCIL, tpo.TPO_VARIANT_MFMA):
        assert tpo.tpo_ihelm_sep_has_variant(7, tpo.TPO_F64, var) == 1
    # E = 0 is a no-op
    assert tpo.tpo_ihelm_apply_sep(*ptrs, tv.data_ptr(), 7, 0, tpo.TPO_F64, None) == tpo.TPO_OK

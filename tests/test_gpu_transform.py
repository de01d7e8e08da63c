"""GPU parity of the transform halves on their own (tpo_transform_apply) against the CPU oracle.
Bar: max-norm relative error per element <= 1e-12 (fp64) / 2e-5 (fp32)."""
import numpy as np
import pytest
import torch

import oracle
from gpu_util import TOL, dev
from paper_2604_19906_amd import tpo
from paper_2604_19906_amd import workloads as wl

pytestmark = pytest.mark.gpu

DIRS = {"forward": (tpo.TPO_FORWARD, oracle.forward), "backward": (tpo.TPO_BACKWARD, oracle.backward)}


@pytest.fixture(scope="module", autouse=True)
def library():
    assert torch.cuda.is_available(), "GPU tests need a device"
    tpo.check(tpo.tpo_create(), "tpo_create")
    yield
    tpo.check(tpo.tpo_destroy(), "tpo_destroy")


def run_transform(u, sx, sy, sz, direction):
    tu = dev(u)
    if sx is sy and sy is sz:
        ts = dev(sx)
        mats = (ts, ts, ts)
    else:
        mats = (dev(sx), dev(sy), dev(sz))
    tt = tpo.transform_tensors(tu, *mats, direction)
    torch.cuda.synchronize()
    return tt.cpu().numpy()


@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("n", list(range(1, 17)))
def test_transform_all_n_small_batches(n, dtype):
    for name, (direction, ref_fn) in DIRS.items():
        for e, distinct in ((1, True), (67, True), (203, True), (131, False)):
            w = wl.custom(n, e, dtype, key=600 + n, distinct_s=distinct)
            u, sx, sy, sz, _ = wl.make_inputs(w)
            print(f"case transform {name} n={n} {dtype} E={e} distinct={distinct}", flush=True)
            got = run_transform(u, sx, sy, sz, direction)
            assert got.dtype == u.dtype and got.shape == u.shape
            err = oracle.max_rel_err_per_element(got, ref_fn(u, sx, sy, sz))
            assert err <= TOL[dtype], f"{name} n={n} {dtype} E={e}: err {err:.3e}"


def sample_spans(e):
    rng = np.random.default_rng(777 + e)
    spans = [(0, min(512, e)), (max(0, e - 512), e)]
    for s in rng.integers(0, max(1, e - 256), 6):
        spans.append((int(s), int(min(e, s + 256))))
    return spans


@pytest.mark.parametrize("idx", [1, 2, 3, 4])
def test_transform_full_size_configs(idx):
    w = wl.CONFIGS[idx]
    print(f"case transform {w.name}: generating", flush=True)
    tu, tsx, tsy, tsz = wl.to_device(w, with_d=False)
    tt = torch.empty_like(tu)
    sx, sy, sz = wl.direction_matrices(w)
    s64 = [s.double() for s in (tsx, tsy, tsz)]
    for name, (direction, ref_fn) in DIRS.items():
        print(f"case transform {w.name} {name}", flush=True)
        tt.fill_(float("nan"))
        tpo.transform_tensors(tu, tsx, tsy, tsz, direction, tt)
        torch.cuda.synchronize()
        worst = 0.0
        for lo, hi in sample_spans(w.num_elems):
            ref = ref_fn(wl.field_u(w, lo, hi), sx, sy, sz)
            worst = max(worst, oracle.max_rel_err_per_element(tt[lo:hi].cpu().numpy(), ref))
        assert worst <= TOL[w.dtype], f"{w.name} {name}: sampled err {worst:.3e}"
        assert not torch.isnan(tt).any()
        spec = "li,mj,qk,elmq->eijk" if direction == tpo.TPO_FORWARD else "il,jm,kq,elmq->eijk"
        worst_all = 0.0
        step = 8192
        for lo in range(0, w.num_elems, step):
            hi = min(w.num_elems, lo + step)
            ref = torch.einsum(spec, *s64, tu[lo:hi].double())
            num = (tt[lo:hi].double() - ref).abs().flatten(1).max(dim=1).values
            den = ref.abs().flatten(1).max(dim=1).values
            worst_all = max(worst_all, float((num / den).max()))
        assert worst_all <= TOL[w.dtype], f"{w.name} {name}: full err {worst_all:.3e}"
        print(f"  {w.name} {name}: sampled {worst:.2e}, all elements {worst_all:.2e}", flush=True)


def test_transform_in_place_composition_and_status_codes():
    w = wl.custom(6, 75, "f64", key=700, distinct_s=True)
    u, sx, sy, sz, d = wl.make_inputs(w)
    t = [dev(a) for a in (u, sx, sy, sz)]
    # forward in place, scale, backward in place == the whole operator
    work = t[0].clone()
    tpo.transform_tensors(work, t[1], t[2], t[3], tpo.TPO_FORWARD, work)
    work *= dev(d)
    tpo.transform_tensors(work, t[1], t[2], t[3], tpo.TPO_BACKWARD, work)
    torch.cuda.synchronize()
    ref = oracle.ihelm_apply(u, sx, sy, sz, d)
    assert oracle.max_rel_err_per_element(work.cpu().numpy(), ref) <= 1e-12
    ptrs = [x.data_ptr() for x in t]
    out = torch.empty_like(t[0])
    assert tpo.tpo_transform_apply(*ptrs, out.data_ptr(), 6, 75, tpo.TPO_F64, 2, None) \
        == tpo.TPO_ERR_INVALID_ARG
    assert tpo.tpo_transform_apply(*ptrs, out.data_ptr(), 6, 0, tpo.TPO_F64, tpo.TPO_FORWARD, None) \
        == tpo.TPO_OK

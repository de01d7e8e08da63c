"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same
seeded inputs.  Bar: max-norm relative error per element <= 1e-12 (fp64) / 2e-5 (fp32)."""
import os

import numpy as np
import pytest
import torch

import oracle
from gpu_util import TOL, VARIANTS, dev, oracle_every_element, run, upload_full
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


def variants_for(n, dtype):
    return [name for name, var in VARIANTS.items() if tpo.tpo_ihelm_has_variant(n, DT[dtype], var)]


def check_against_oracle(w, variant_name, lo=0, hi=None):
    u, sx, sy, sz, d = wl.make_inputs(w, lo, hi)
    got = run(u, sx, sy, sz, d, VARIANTS[variant_name])
    ref = oracle.ihelm_apply(u, sx, sy, sz, d)
    assert got.dtype == u.dtype and got.shape == u.shape
    err = oracle.max_rel_err_per_element(got, ref)
    assert err <= TOL[w.dtype], f"{w.name} {variant_name}: err {err:.3e}"
    return err


# every supported n, both precisions, every kernel family; E spans several workgroups and
# leaves a ragged tail for every group size
@pytest.mark.parametrize("dtype", ["f64", "f32"])
@pytest.mark.parametrize("n", list(range(1, 17)))
def test_all_n_small_batches(n, dtype):
    for name in variants_for(n, dtype):
        for e in (1, 67, 203):
            w = wl.custom(n, e, dtype, key=200 + n, distinct_s=True)
            print(f"case n={n} {dtype} E={e} variant={name}", flush=True)
            check_against_oracle(w, name)
        # one matrix shared by the three directions (same pointer): its own kernel instantiation
        w = wl.custom(n, 131, dtype, key=250 + n, distinct_s=False)
        print(f"case n={n} {dtype} E=131 shared S variant={name}", flush=True)
        check_against_oracle(w, name)


def test_config0_all_elements():
    w = wl.CONFIGS[0]
    for name in variants_for(w.n, w.dtype):
        check_against_oracle(w, name)
    # the default entry point (10 arguments) picks its own family
    u, sx, sy, sz, d = wl.make_inputs(w)
    tu, ts, td = dev(u), dev(sx), dev(d)
    tv = torch.empty_like(tu)
    rc = tpo.tpo_ihelm_apply(tu.data_ptr(), ts.data_ptr(), ts.data_ptr(), ts.data_ptr(),
                             td.data_ptr(), tv.data_ptr(), w.n, w.num_elems, tpo.TPO_F64,
                             torch.cuda.current_stream().cuda_stream)
    assert rc == tpo.TPO_OK
    torch.cuda.synchronize()
    ref = oracle.ihelm_apply(u, sx, sy, sz, d)
    assert oracle.max_rel_err_per_element(tv.cpu().numpy(), ref) <= 1e-12


def test_golden_file(repo_root):
    path = os.path.join(repo_root, "tests", "golden", "ihelm_f64_n3_E2.txt")
    want = np.array([float.fromhex(l) for l in open(path) if not l.startswith("#")])
    w = wl.custom(3, 2, "f64", key=77)
    for name in variants_for(3, "f64"):
        got = run(*wl.make_inputs(w), VARIANTS[name])
        assert oracle.max_rel_err_per_element(got, want.reshape(got.shape)) <= 1e-12


def oracle_over_all_elements(w, tu, td, outs):
    """Every element of workload ``w`` against the oracle (see gpu_util.oracle_every_element)."""
    sx, sy, sz = wl.direction_matrices(w)
    return oracle_every_element(
        w.num_elems,
        lambda lo, hi: (wl.field_u(w, lo, hi), sx, sy, sz, wl.diagonal_d(w, lo, hi)),
        lambda lo, hi: (tu[lo:hi], None, None, None, td[lo:hi]),
        oracle.ihelm_apply, outs, TOL[w.dtype], w.name)


# the four large configurations at full size, in the launch configuration the benchmark uses;
# the oracle checks every element of every family's result
@pytest.mark.parametrize("idx", [1, 2, 3, 4])
def test_full_size_configs(idx):
    w = wl.CONFIGS[idx]
    print(f"case {w.name}: generating", flush=True)
    tu, tsx, tsy, tsz, td = upload_full(w)
    outs = {}
    for name in variants_for(w.n, w.dtype) + ["auto"]:
        print(f"case {w.name} variant={name}", flush=True)
        tv = torch.full_like(tu, float("nan"))
        if name == "auto":          # the 10-argument entry point, the call the benchmark times
            rc = tpo.tpo_ihelm_apply(tu.data_ptr(), tsx.data_ptr(), tsy.data_ptr(), tsz.data_ptr(),
                                     td.data_ptr(), tv.data_ptr(), w.n, w.num_elems, DT[w.dtype],
                                     torch.cuda.current_stream().cuda_stream)
            assert rc == tpo.TPO_OK
        else:
            tpo.apply_tensors(tu, tsx, tsy, tsz, td, tv, variant=VARIANTS[name])
        torch.cuda.synchronize()
        assert not torch.isnan(tv).any()
        outs[name] = tv
    print(f"case {w.name}: oracle over all {w.num_elems} elements", flush=True)
    worst = oracle_over_all_elements(w, tu, td, outs)
    print(f"  {w.name}: " + ", ".join(f"{k} {v:.2e}" for k, v in worst.items()), flush=True)


# the paper's batch (Sec. 6.1: 8192 elements per call) with the shapes of the four large
# configurations: the 10-argument entry point and the separable form, every element against the
# oracle
@pytest.mark.parametrize("idx", [1, 2, 3, 4])
def test_paper_batch_8192(idx):
    c = wl.CONFIGS[idx]
    w = wl.Workload(c.name + "_E8192", c.index, c.dtype, c.n, 8192, c.u_dist, c.distinct_s)
    u, sx, sy, sz, d = wl.make_inputs(w)
    ref = oracle.ihelm_apply(u, sx, sy, sz, d)
    tu, td = dev(u), dev(d)
    if sx is sy and sy is sz:
        tsx = tsy = tsz = dev(sx)
    else:
        tsx, tsy, tsz = dev(sx), dev(sy), dev(sz)
    tv = torch.full_like(tu, float("nan"))
    rc = tpo.tpo_ihelm_apply(tu.data_ptr(), tsx.data_ptr(), tsy.data_ptr(), tsz.data_ptr(),
                             td.data_ptr(), tv.data_ptr(), w.n, w.num_elems, DT[w.dtype],
                             torch.cuda.current_stream().cuda_stream)
    assert rc == tpo.TPO_OK
    torch.cuda.synchronize()
    err = oracle.max_rel_err_per_element(tv.cpu().numpy(), ref)
    assert err <= TOL[w.dtype], f"{w.name}: err {err:.3e}"
    lam = wl.sep_inputs(w)
    ref_sep = oracle.ihelm_apply_sep(u, sx, sy, sz, *lam)
    tv.fill_(float("nan"))
    tpo.apply_sep_tensors(tu, tsx, tsy, tsz, *map(dev, lam), v=tv)
    torch.cuda.synchronize()
    err_sep = oracle.max_rel_err_per_element(tv.cpu().numpy(), ref_sep)
    assert err_sep <= TOL[w.dtype], f"{w.name} sep: err {err_sep:.3e}"
    print(f"  {w.name}: {err:.2e}, separable {err_sep:.2e}", flush=True)


# fp32 n = 14, 15, 16: the family the 10-argument entry point takes there (matrix-core tiles)
# at the batch size of the large workloads, every element against the oracle
@pytest.mark.parametrize("n", [14, 15, 16])
def test_f32_large_n_at_scale(n):
    w = wl.custom(n, 262144 + 37, "f32", key=900 + n, distinct_s=True)
    assert tpo.tpo_ihelm_variant_for(n, tpo.TPO_F32, 0) == tpo.TPO_VARIANT_MFMA
    print(f"case f32 n={n} E={w.num_elems}: generating", flush=True)
    tu, tsx, tsy, tsz, td = upload_full(w)
    tv = torch.full_like(tu, float("nan"))
    rc = tpo.tpo_ihelm_apply(tu.data_ptr(), tsx.data_ptr(), tsy.data_ptr(), tsz.data_ptr(),
                             td.data_ptr(), tv.data_ptr(), n, w.num_elems, tpo.TPO_F32,
                             torch.cuda.current_stream().cuda_stream)
    assert rc == tpo.TPO_OK
    torch.cuda.synchronize()
    assert not torch.isnan(tv).any()
    worst = oracle_over_all_elements(w, tu, td, {"auto": tv})
    print(f"  f32 n={n}: {worst['auto']:.2e}", flush=True)


# the persistent matrix-core kernel (fp64 n = 11: a fixed grid of workgroups walks over the
# elements): batches larger than the resident grid so that every workgroup iterates, with a
# ragged tail, out of place and in place
@pytest.mark.parametrize("e", [4099, 20011])
def test_persistent_mfma_loop_iterates(e):
    w = wl.custom(11, e, "f64", key=1400 + e % 7, distinct_s=True)
    u, sx, sy, sz, d = wl.make_inputs(w)
    ref = oracle.ihelm_apply(u, sx, sy, sz, d)
    tu, tsx, tsy, tsz, td = map(dev, (u, sx, sy, sz, d))
    var = tpo.TPO_VARIANT_MFMA
    v1 = tpo.apply_tensors(tu, tsx, tsy, tsz, td, variant=var)
    torch.cuda.synchronize()
    assert oracle.max_rel_err_per_element(v1.cpu().numpy(), ref) <= TOL["f64"]
    v2 = tpo.apply_tensors(tu, tsx, tsy, tsz, td, variant=var)
    assert torch.equal(v1, v2)
    tpo.apply_tensors(tu, tsx, tsy, tsz, td, tu, variant=var)        # v == u
    torch.cuda.synchronize()
    assert torch.equal(tu, v1)
    # one matrix shared by the three directions: the other instantiation of the same loop
    w2 = wl.custom(11, e, "f64", key=1410 + e % 7, distinct_s=False)
    u, sx, sy, sz, d = wl.make_inputs(w2)
    got = run(u, sx, sy, sz, d, var)
    assert oracle.max_rel_err_per_element(got, oracle.ihelm_apply(u, sx, sy, sz, d)) <= TOL["f64"]


# The launchers switch settings (elements per workgroup, hints, die renumbering) with the batch
# size: both sides of every switch point, with odd batch sizes so that the last workgroup of the
# several-elements-per-workgroup settings is ragged; out of place, then in place.
@pytest.mark.parametrize("n,dtype,name,sizes", [
    (11, "f64", "pencil", (6144, 6145, 8193, 20011)),
    (8, "f64", "pencil", (4096, 4097, 24575, 24577)),
    (9, "f64", "pencil", (16384, 16385)),
    (13, "f32", "pencil_mm", (262144, 262147)),
])
def test_batch_size_dependent_settings(n, dtype, name, sizes):
    for e in sizes:
        w = wl.custom(n, e, dtype, key=1500 + n, distinct_s=(dtype == "f32"))
        print(f"case n={n} {dtype} E={e} variant={name}", flush=True)
        u, sx, sy, sz, d = wl.make_inputs(w)
        ref = oracle.ihelm_apply(u, sx, sy, sz, d)
        tu, td = dev(u), dev(d)
        if sx is sy and sy is sz:
            tsx = dev(sx)
            mats = (tsx, tsx, tsx)
        else:
            mats = (dev(sx), dev(sy), dev(sz))
        v1 = tpo.apply_tensors(tu, *mats, td, variant=VARIANTS[name])
        torch.cuda.synchronize()
        err = oracle.max_rel_err_per_element(v1.cpu().numpy(), ref)
        assert err <= TOL[dtype], f"{w.name} {name}: err {err:.3e}"
        tpo.apply_tensors(tu, *mats, td, tu, variant=VARIANTS[name])      # v == u
        torch.cuda.synchronize()
        assert torch.equal(tu, v1)


# small n with millions of elements: many workgroups per launch, several elements per
# workgroup, a ragged last group; every element checked against the oracle
@pytest.mark.parametrize("n,dtype,e", [(1, "f64", (1 << 22) + 3), (2, "f32", (1 << 22) + 5),
                                       (3, "f64", (1 << 21) + 7), (4, "f32", (1 << 20) + 9)])
def test_many_small_elements(n, dtype, e):
    w = wl.custom(n, e, dtype, key=700 + n, distinct_s=True)
    for name in variants_for(n, dtype):
        print(f"case n={n} {dtype} E={e} variant={name}", flush=True)
        check_against_oracle(w, name)


def test_in_place_and_determinism():
    for dtype, n, e in (("f64", 11, 301), ("f32", 13, 150), ("f64", 16, 40), ("f64", 8, 77)):
        w = wl.custom(n, e, dtype, key=300 + n)
        u, sx, sy, sz, d = wl.make_inputs(w)
        for name in variants_for(n, dtype):
            var = VARIANTS[name]
            tu, tsx, tsy, tsz, td = map(dev, (u, sx, sy, sz, d))
            v1 = tpo.apply_tensors(tu, tsx, tsy, tsz, td, variant=var)
            v2 = tpo.apply_tensors(tu, tsx, tsy, tsz, td, variant=var)
            assert torch.equal(v1, v2)                       # bitwise repeatable
            tpo.apply_tensors(tu, tsx, tsy, tsz, td, tu, variant=var)   # v == u
            assert torch.equal(tu, v1)


def test_equal_valued_matrices_in_distinct_buffers():
    w = wl.custom(7, 90, "f64", key=41, distinct_s=False)
    u, sx, sy, sz, d = wl.make_inputs(w)
    for name in variants_for(7, "f64"):
        a = run(u, sx, sy, sz, d, VARIANTS[name], same_s_pointer=True)
        b = run(u, sx, sy.copy(), sz.copy(), d, VARIANTS[name], same_s_pointer=False)
        assert np.array_equal(a, b)


def test_word_aligned_base_pointers():
    # fields that start one word into an allocation: only 8-byte (4-byte) aligned
    for dtype, n, e in (("f64", 11, 64), ("f32", 13, 64), ("f32", 5, 33)):
        w = wl.custom(n, e, dtype, key=500 + n)
        u, sx, sy, sz, d = wl.make_inputs(w)
        ref = oracle.ihelm_apply(u, sx, sy, sz, d)
        for name in variants_for(n, dtype):
            def shifted(a):
                flat = torch.empty(a.size + 1, dtype=dev(a).dtype, device="cuda")
                view = flat[1:].view(a.shape)
                view.copy_(torch.from_numpy(a))
                return view
            tu, td = shifted(u), shifted(d)
            tsx, tsy, tsz = shifted(sx), shifted(sy), shifted(sz)
            tv = shifted(np.zeros_like(u))
            tpo.apply_tensors(tu, tsx, tsy, tsz, td, tv, variant=VARIANTS[name])
            torch.cuda.synchronize()
            assert oracle.max_rel_err_per_element(tv.cpu().numpy(), ref) <= TOL[dtype]


def test_side_stream_ordering():
    w = wl.custom(9, 500, "f64", key=61)
    u, sx, sy, sz, d = wl.make_inputs(w)
    ref = oracle.ihelm_apply(u, sx, sy, sz, d)
    s = torch.cuda.Stream()
    tsx, tsy, tsz, td = map(dev, (sx, sy, sz, d))
    torch.cuda.synchronize()
    with torch.cuda.stream(s):
        tu = torch.from_numpy(u).cuda()          # upload, apply and scale on the same stream
        tv = tpo.apply_tensors(tu, tsx, tsy, tsz, td)
        tv2 = tv * 2.0
    s.synchronize()
    assert oracle.max_rel_err_per_element(tv2.cpu().numpy(), 2.0 * ref) <= 1e-12


def test_status_codes_on_device():
    w = wl.custom(4, 8, "f64", key=71)
    u, sx, sy, sz, d = wl.make_inputs(w)
    tu, tsx, tsy, tsz, td = map(dev, (u, sx, sy, sz, d))
    tv = torch.empty_like(tu)
    st = torch.cuda.current_stream().cuda_stream
    args = (tu.data_ptr(), tsx.data_ptr(), tsy.data_ptr(), tsz.data_ptr(), td.data_ptr(),
            tv.data_ptr())
    assert tpo.tpo_ihelm_apply(*args, 4, 0, tpo.TPO_F64, st) == tpo.TPO_OK       # empty batch
    assert tpo.tpo_ihelm_apply(*args, 17, 8, tpo.TPO_F64, st) == tpo.TPO_ERR_UNSUPPORTED
    assert tpo.tpo_ihelm_apply(*args[:5], td.data_ptr(), 4, 8, tpo.TPO_F64, st) \
        == tpo.TPO_ERR_ALIAS
    # reference counting: a second create/destroy pair leaves the library usable
    assert tpo.tpo_create() == tpo.TPO_OK
    assert tpo.tpo_destroy() == tpo.TPO_OK
    assert tpo.tpo_ihelm_apply(*args, 4, 8, tpo.TPO_F64, st) == tpo.TPO_OK
    # dropping the last reference makes apply refuse; creating again restores it
    assert tpo.tpo_destroy() == tpo.TPO_OK
    assert tpo.tpo_ihelm_apply(*args, 4, 8, tpo.TPO_F64, st) == tpo.TPO_ERR_NOT_INITIALIZED
    assert tpo.tpo_destroy() == tpo.TPO_ERR_NOT_INITIALIZED
    assert tpo.tpo_create() == tpo.TPO_OK
    assert tpo.tpo_ihelm_apply(*args, 4, 8, tpo.TPO_F64, st) == tpo.TPO_OK
    torch.cuda.synchronize()
    ref = oracle.ihelm_apply(u, sx, sy, sz, d)
    assert oracle.max_rel_err_per_element(tv.cpu().numpy(), ref) <= 1e-12


def test_degenerate_inputs():
    # identity matrices and unit diagonal: every product multiplies by 1 or adds 0, v == u bit for
    # bit; zero field in, zero field out; a NaN stays inside its own element
    for dtype, n in (("f64", 11), ("f32", 13), ("f64", 16), ("f32", 16), ("f64", 1)):
        w = wl.custom(n, 53, dtype, key=1200 + n)
        u = wl.field_u(w)
        eye = np.eye(n, dtype=u.dtype)
        ones = np.ones_like(u)
        for name in variants_for(n, dtype):
            assert np.array_equal(run(u, eye, eye, eye, ones, VARIANTS[name]), u), (dtype, n, name)
            u2, sx, sy, sz, d = wl.make_inputs(w)
            assert not run(np.zeros_like(u2), sx, sy, sz, d, VARIANTS[name]).any()
            u3 = u2.copy()
            u3[17, 0, 0, 0] = np.nan
            got = run(u3, sx, sy, sz, d, VARIANTS[name])
            bad = np.isnan(got).reshape(53, -1).any(axis=1)
            assert bad[17] and bad.sum() == 1, (dtype, n, name)
            clean = run(u2, sx, sy, sz, d, VARIANTS[name])
            assert np.array_equal(np.delete(got, 17, axis=0), np.delete(clean, 17, axis=0))


def test_graph_capture_and_replay():
    # the call only enqueues a kernel on the caller's stream (no allocation, no synchronisation),
    # so it can be captured into a HIP graph; every replay must equal the eager result on the
    # inputs present at replay time
    w = wl.custom(11, 300, "f64", key=1300, distinct_s=True)
    u, sx, sy, sz, d = wl.make_inputs(w)
    tu, tsx, tsy, tsz, td = map(dev, (u, sx, sy, sz, d))
    tv = torch.empty_like(tu)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        tpo.apply_tensors(tu, tsx, tsy, tsz, td, tv)          # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        tpo.apply_tensors(tu, tsx, tsy, tsz, td, tv)
    rng = np.random.default_rng(5)
    for rep in range(3):
        new_u = rng.uniform(-1, 1, u.shape)
        tu.copy_(torch.from_numpy(new_u))
        tv.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        eager = tpo.apply_tensors(tu, tsx, tsy, tsz, td)
        torch.cuda.synchronize()
        assert torch.equal(tv, eager), f"replay {rep}"
        ref = oracle.ihelm_apply(new_u, sx, sy, sz, d)
        assert oracle.max_rel_err_per_element(tv.cpu().numpy(), ref) <= 1e-12


def test_graph_with_every_entry_point():
    # the other entry points enqueue one kernel each in the same way: one graph holding the
    # separable form, a forward transform, the convection term and an anisotropic call, replayed
    # on changed inputs, each replay equal to the eager results
    w = wl.custom(9, 150, "f64", key=1310, distinct_s=True)
    u, sx, sy, sz, d = wl.make_inputs(w)
    lam = wl.sep_inputs(w, 0, w.num_elems)
    cw = wl.conv_custom(9, 60, "f64", key=1311)
    cp, cm, cd, ci = wl.conv_inputs(cw)
    rng = np.random.default_rng(6)
    dims = (9, 7, 10)
    mats = [wl.orthogonal_matrix(k, rng) for k in dims]
    ua = rng.uniform(-1, 1, (90, *dims))
    da = rng.uniform(0.03, 3.3, (90, *dims))
    tu, tsx, tsy, tsz = map(dev, (u, sx, sy, sz))
    tl = list(map(dev, lam))
    tc = list(map(dev, (cp, cm, cd, ci)))
    ta = [dev(ua)] + list(map(dev, mats)) + [dev(da)]
    out_sep, out_fwd, out_an = torch.empty_like(tu), torch.empty_like(tu), torch.empty_like(ta[0])
    out_conv = torch.empty_like(tc[0][0])

    def enqueue(o_sep, o_fwd, o_conv, o_an):
        tpo.apply_sep_tensors(tu, tsx, tsy, tsz, *tl, v=o_sep)
        tpo.transform_tensors(tu, tsx, tsy, tsz, tpo.TPO_FORWARD, t=o_fwd)
        tpo.convection_tensors(*tc, F=o_conv)
        tpo.apply_aniso_tensors(*ta, v=o_an)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        enqueue(out_sep, out_fwd, out_conv, out_an)             # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        enqueue(out_sep, out_fwd, out_conv, out_an)
    for rep in range(3):
        tu.copy_(torch.from_numpy(rng.uniform(-1, 1, u.shape)))
        tc[0].copy_(torch.from_numpy(rng.uniform(-1, 1, cp.shape)))
        ta[0].copy_(torch.from_numpy(rng.uniform(-1, 1, ua.shape)))
        for o in (out_sep, out_fwd, out_conv, out_an):
            o.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        eager = [torch.empty_like(o) for o in (out_sep, out_fwd, out_conv, out_an)]
        enqueue(*eager)
        torch.cuda.synchronize()
        for name, got, want in zip(("sep", "forward", "convection", "aniso"),
                                   (out_sep, out_fwd, out_conv, out_an), eager):
            assert torch.equal(got, want), f"replay {rep}: {name}"
    ref = oracle.ihelm_apply_aniso(ta[0].cpu().numpy(), *mats, da)
    assert oracle.max_rel_err_per_element(out_an.cpu().numpy(), ref) <= 1e-12

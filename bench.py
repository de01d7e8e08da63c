#!/usr/bin/env python3
"""Benchmark of the batched inverse-Helmholtz tensor-product operator on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload IDX] [--variant NAME]

A step is one pass of the whole hot path (six mode products plus the diagonal scale, one
library call) over every element of the workload, with u, D, S and v resident in HBM.  The
default workload is the fp64 n=11 configuration the headline metric is quoted on.  Prints ONE
JSON line on stdout; progress goes to stderr.

Beside the whole-job throughput the line carries
  "roofline":     algorithmic HBM bytes per launch / average kernel time (HIP events on the
                  launch stream) against the 8 TB/s HBM peak, and the measured HBM traffic per
                  launch from profiles/traffic.json when it was taken for the current kernel
                  sources (else null);
  "cpu_baseline": the CPU oracle, as it stands, timed on this machine's host cores on a
                  bounded sample of the same workload.  A reported baseline, not a target.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E, published
FP_PEAK_TFLOPS = {"f64": 78.6, "f32": 157.3}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def timed_passes(run, ns, cores, cpu_seconds=16.0, max_passes=64):
    """Whole passes of the oracle over a sample of ns elements until about cpu_seconds of CPU
    work (wall time x threads) are done; returns (elements/s, passes, wall seconds)."""
    passes, wall = 0, 0.0
    t1 = time.perf_counter()
    while wall * cores < cpu_seconds and passes < max_passes:
        run()
        passes += 1
        wall = time.perf_counter() - t1
    return passes * ns / wall, passes, wall


def loaded_state(torch, launch, seconds=0.3, batch=20):
    """Keeps the GPU busy with `launch` for about `seconds` before anything is timed: after idling
    (input generation on the host takes seconds) the clocks need some hundred milliseconds of
    load to settle, and kernels of a few hundred microseconds measured inside that ramp come out
    up to 15 % slower than in steady state, whatever the number of warm-up steps."""
    t0 = time.perf_counter()
    done = 0
    while time.perf_counter() - t0 < seconds and done < 20000:
        for _ in range(batch):
            launch()
        done += batch
        torch.cuda.synchronize()


# Sources that make up the kernels of each operation (headers they include, their instantiation
# files); everything an operation's kernels are compiled from.
_COMMON = ["tpo_internal.h", "tpo_pencil.hpp", "tpo_pencil_mm.hpp"]
KERNEL_SOURCES = {
    "ihelm": _COMMON + ["tpo_mfma.hpp", "tpo_mfma_f64.hip", "tpo_mfma_f32.hip", "tpo_pencil_f64.hip",
                        "tpo_pencil_f32.hip", "tpo_pencil_mm_f32.hip"],
    "transform": _COMMON + ["tpo_transform.hpp", "tpo_transform_f64.hip", "tpo_transform_f32.hip"],
    "convection": _COMMON + ["tpo_convection.hpp", "tpo_convection_f64.hip", "tpo_convection_f32.hip"],
    "aniso": ["tpo_internal.h", "tpo_pencil.hpp", "tpo_generic.hip"],
}


def kernel_source_hash(op: str = "ihelm") -> str:
    """Hash of the code an operation's kernels are built from (comments and layout left out: they
    do not change the kernel); ties stored HBM-traffic counters to the code they measured."""
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2604_19906_amd", "csrc")
    for name in sorted(KERNEL_SOURCES[op]):
        text = open(os.path.join(csrc, name), encoding="utf-8").read()
        text = re.sub(r"/\*.*?\*/", " ", text, flags=re.S)
        text = re.sub(r"//[^\n]*", " ", text)
        h.update(name.encode())
        h.update(" ".join(text.split()).encode())
    return h.hexdigest()[:16]


def stored_traffic(workload: str, variant: str, op: str = "ihelm"):
    """HBM bytes per launch from the rocprofv3 --pmc summaries, or None when there is no
    entry for this workload/variant or the kernel sources changed since it was taken."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        table = json.load(open(path))
    except (OSError, ValueError):
        return None
    ent = table.get(f"{workload}:{variant}")
    if not ent or ent.get("source_hash") != kernel_source_hash(op):
        return None
    return ent.get("hbm_bytes_per_launch")


def bench_convection(args, torch, tpo, wl) -> int:
    """The convection volume term (Eq. 1 of the paper) on one of its synthetic configurations:
    same timing scheme, its own algorithmic traffic (13 cubes per element)."""
    import numpy as np
    import oracle

    if args.variant != "auto":
        log("bench.py: the convection term has one kernel family; --variant does not apply")
        return 2
    w = wl.CONV_CONFIGS[args.workload if args.workload < len(wl.CONV_CONFIGS) else 1]
    if args.elems:
        w = wl.ConvWorkload(w.name + f"_E{args.elems}", w.index, w.dtype, w.n, args.elems, w.nq)
    dt = tpo.TPO_F64 if w.dtype == "f64" else tpo.TPO_F32
    t0 = time.time()
    tp, tm, td, ti = wl.conv_to_device(w)
    tf = torch.empty((3, w.num_elems, w.n, w.n, w.n), dtype=tp.dtype, device="cuda")
    torch.cuda.synchronize()
    alg_bytes = w.bytes_per_elem * w.num_elems
    alg_flop = w.flop_per_elem * w.num_elems
    log(f"[bench] {w.name} (convection): inputs resident after {time.time() - t0:.1f}s "
        f"({alg_bytes / 1e9:.2f} GB for P, M, F)")
    stream = torch.cuda.current_stream()
    ptrs = (tp.data_ptr(), tm.data_ptr(), td.data_ptr(), ti.data_ptr(), tf.data_ptr())

    def step():
        rc = tpo.tpo_convection_apply(*ptrs, w.n, w.q, w.num_elems, dt, stream.cuda_stream)
        if rc != tpo.TPO_OK:
            raise tpo.TpoError(rc, "tpo_convection_apply")

    # plain streaming kernel over three cubes of this workload (F is overwritten again below):
    # the streaming ceiling, and the calibration of the HBM counters in profiler runs
    cube_words = min(tm.numel(), tf[0].numel())     # F cubes are smaller when n_v < n_q
    for _ in range(3):
        rc = tpo.tpo_stream_scale(tp[0, 0].data_ptr(), tp[0, 1].data_ptr(), tf[0].data_ptr(),
                                  cube_words, dt, stream.cuda_stream)
        if rc != tpo.TPO_OK:            # cubes that do not start on 16-byte boundaries
            log("[bench] streaming calibration skipped: " + tpo.status_string(rc))
            break
    loaded_state(torch, step)
    for _ in range(args.warmup):
        step()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in range(args.steps)]
    torch.cuda.synchronize()
    t_begin = time.perf_counter()
    for a, b in evs:
        a.record(stream)
        step()
        b.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_begin
    kernel_ms = [a.elapsed_time(b) for a, b in evs]
    avg_kernel_ms = sum(kernel_ms) / len(kernel_ms)
    ms_per_step = wall * 1e3 / args.steps
    achieved_gbs = alg_bytes / (avg_kernel_ms * 1e-3) / 1e9
    achieved_tflops = alg_flop / (avg_kernel_ms * 1e-3) / 1e12
    log(f"[bench] kernel avg {avg_kernel_ms:.4f} ms (min {min(kernel_ms):.4f}, max "
        f"{max(kernel_ms):.4f}); wall/step {ms_per_step:.4f} ms; {achieved_gbs:.0f} GB/s; "
        f"{achieved_tflops:.2f} TFLOP/s")

    d, i = wl.conv_matrices(w)
    hi = min(16, w.num_elems)
    ref = oracle.convection_apply(wl.conv_flux(w, 0, hi), wl.conv_metric(w, 0, hi), d, i)
    got = tf[:, :hi].cpu().numpy()
    err = oracle.max_rel_err_per_element(got.reshape(-1, *got.shape[2:]),
                                         ref.reshape(-1, *ref.shape[2:]))
    tol = 1e-12 if w.dtype == "f64" else 2e-5
    if not err <= tol:
        log(f"[bench] PARITY FAILURE on the timed output: {err:.3e} > {tol}")
        return 1

    cpu = None
    if not args.no_cpu_baseline:
        ns = min(4096, w.num_elems)
        hp, hm = wl.conv_flux(w, 0, ns), wl.conv_metric(w, 0, ns)
        cores = oracle.max_threads()
        oracle.convection_apply(hp[:, :, :16], hm[:16], d, i)
        rate, passes, cpu_s = timed_passes(lambda: oracle.convection_apply(hp, hm, d, i), ns, cores)
        cpu = {"value": rate, "unit": "elements/s", "cores": cores, "kind": "oracle",
               "sample": f"first {ns} elements of {w.name}, {passes} pass(es), {cores} host "
                         f"thread(s) ({cpu_s:.2f} s wall)"}
        log(f"[bench] CPU oracle baseline: {rate:.0f} elements/s on {cores} threads")

    out = {
        "metric": "elements/s + GFLOP/s and % of binding roofline, convection volume term",
        "value": w.num_elems / (ms_per_step * 1e-3), "unit": "elements/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": w.name, "op": "convection", "n": w.n, "n_q": w.q,
                   "num_elems": w.num_elems,
                   "layout": "P [3,3,E,n,n,n], M [E,n,n,n], F [3,E,n,n,n]", "parallelism": "1 GPU"},
        "gflops": alg_flop / (ms_per_step * 1e-3) / 1e9,
        "kernel_ms_avg": avg_kernel_ms, "kernel_ms_min": min(kernel_ms),
        "fp_frac_of_peak": achieved_tflops / FP_PEAK_TFLOPS[w.dtype],
        "parity_max_rel_err_sample": err,
        "roofline": {"bound": "hbm", "achieved": achieved_gbs, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved_gbs / HBM_PEAK_GBS,
                     "traffic": stored_traffic(w.name + ":convection", "pencil", "convection")},
        "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)
    tpo.tpo_destroy()
    return 0


def bench_aniso(args, torch, tpo, wl) -> int:
    """The operator on anisotropic elements (n_x, n_y, n_z points along the three axes) on one of
    its synthetic configurations: same timing scheme, 3 * n_x * n_y * n_z words per element."""
    import oracle

    if args.variant != "auto":
        log("bench.py: anisotropic elements have one kernel family; --variant does not apply")
        return 2
    w = wl.ANISO_CONFIGS[args.workload if args.workload < len(wl.ANISO_CONFIGS) else 2]
    if args.elems:
        w = wl.AnisoWorkload(w.name + f"_E{args.elems}", w.index, w.dtype, w.dims, args.elems)
    dt = tpo.TPO_F64 if w.dtype == "f64" else tpo.TPO_F32
    t0 = time.time()
    tu, tsx, tsy, tsz, td = wl.aniso_to_device(w)
    tv = torch.empty_like(tu)
    torch.cuda.synchronize()
    alg_bytes = w.bytes_per_elem * w.num_elems
    alg_flop = w.flop_per_elem * w.num_elems
    log(f"[bench] {w.name} (aniso): inputs resident after {time.time() - t0:.1f}s "
        f"({alg_bytes / 1e9:.2f} GB for u, D, v)")
    stream = torch.cuda.current_stream()
    ptrs = (tu.data_ptr(), tsx.data_ptr(), tsy.data_ptr(), tsz.data_ptr(), td.data_ptr(),
            tv.data_ptr())

    def step():
        rc = tpo.tpo_ihelm_apply_aniso(*ptrs, *w.dims, w.num_elems, dt, stream.cuda_stream)
        if rc != tpo.TPO_OK:
            raise tpo.TpoError(rc, "tpo_ihelm_apply_aniso")

    # streaming ceiling and counter calibration first: v = u .* D over the same three fields,
    # after 0.3 s of it to bring the clocks to their loaded state
    def stream_step():
        rc = tpo.tpo_stream_scale(ptrs[0], ptrs[4], ptrs[5], tu.numel(), dt, stream.cuda_stream)
        if rc != tpo.TPO_OK:
            raise tpo.TpoError(rc, "tpo_stream_scale")

    loaded_state(torch, stream_step)
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record(stream)
    for _ in range(10):
        stream_step()
    b.record(stream)
    torch.cuda.synchronize()
    stream_gbs = alg_bytes / (a.elapsed_time(b) / 10 * 1e-3) / 1e9
    log(f"[bench] streaming ceiling v=u.*D: {stream_gbs:.0f} GB/s")

    for _ in range(args.warmup):
        step()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in range(args.steps)]
    torch.cuda.synchronize()
    t_begin = time.perf_counter()
    for a, b in evs:
        a.record(stream)
        step()
        b.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_begin
    kernel_ms = [a.elapsed_time(b) for a, b in evs]
    avg_kernel_ms = sum(kernel_ms) / len(kernel_ms)
    ms_per_step = wall * 1e3 / args.steps
    achieved_gbs = alg_bytes / (avg_kernel_ms * 1e-3) / 1e9
    achieved_tflops = alg_flop / (avg_kernel_ms * 1e-3) / 1e12
    log(f"[bench] kernel avg {avg_kernel_ms:.4f} ms (min {min(kernel_ms):.4f}, max "
        f"{max(kernel_ms):.4f}); wall/step {ms_per_step:.4f} ms; {achieved_gbs:.0f} GB/s; "
        f"{achieved_tflops:.2f} TFLOP/s")

    step()
    torch.cuda.synchronize()
    hi = min(64, w.num_elems)
    ref = oracle.ihelm_apply_aniso(*wl.aniso_inputs(w, 0, hi))
    err = oracle.max_rel_err_per_element(tv[:hi].cpu().numpy(), ref)
    tol = 1e-12 if w.dtype == "f64" else 2e-5
    if not err <= tol:
        log(f"[bench] PARITY FAILURE on the timed output: {err:.3e} > {tol}")
        return 1

    cpu = None
    if not args.no_cpu_baseline:
        ns = min(16384, w.num_elems)
        hin = wl.aniso_inputs(w, 0, ns)
        oracle.ihelm_apply_aniso(hin[0][:64], *hin[1:4], hin[4][:64])        # load + warm
        rate, passes, cpu_s = timed_passes(lambda: oracle.ihelm_apply_aniso(*hin), ns, 1)
        cpu = {"value": rate, "unit": "elements/s", "cores": 1, "kind": "oracle",
               "sample": f"first {ns} elements of {w.name}, {passes} pass(es), 1 host thread "
                         f"({cpu_s:.2f} s wall)"}
        log(f"[bench] CPU oracle baseline: {rate:.0f} elements/s on 1 thread")

    out = {
        "metric": "elements/s + GFLOP/s and % of binding roofline, anisotropic TPO apply",
        "value": w.num_elems / (ms_per_step * 1e-3), "unit": "elements/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": w.name, "op": "aniso", "dims": list(w.dims),
                   "num_elems": w.num_elems, "layout": "[E,n_x,n_y,n_z] element-contiguous",
                   "parallelism": "1 GPU"},
        "gflops": alg_flop / (ms_per_step * 1e-3) / 1e9,
        "kernel_ms_avg": avg_kernel_ms, "kernel_ms_min": min(kernel_ms),
        "fp_frac_of_peak": achieved_tflops / FP_PEAK_TFLOPS[w.dtype],
        "stream_ceiling_gbs": stream_gbs,
        "parity_max_rel_err_sample": err,
        "roofline": {"bound": "hbm", "achieved": achieved_gbs, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved_gbs / HBM_PEAK_GBS,
                     "traffic": stored_traffic(w.name + ":aniso", "aniso", "aniso")},
        "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)
    tpo.tpo_destroy()
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", type=int, default=2, help="index into the named configurations")
    ap.add_argument("--variant", default="auto", choices=["auto", "pencil", "mfma", "pencil_mm"])
    ap.add_argument("--op", default="ihelm", choices=["ihelm", "ihelm_sep", "forward", "backward", "convection", "aniso"],
                    help="ihelm: D read from HBM (the headline); ihelm_sep: D evaluated in the "
                         "kernel from lam_x, lam_y, lam_z, mu (two HBM streams instead of three); "
                         "forward / backward: one half of the operator on its own; convection: the "
                         "convection volume term; aniso: the operator on anisotropic elements "
                         "(--workload indexes the configurations of these two on their own)")
    ap.add_argument("--elems", type=int, default=0, help="override the element count (experiments)")
    ap.add_argument("--n", type=int, default=0, help="override the points per direction (experiments)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample", type=int, default=262144,
                    help="elements the CPU oracle is timed on (all host threads)")
    args = ap.parse_args()

    if args.gpus != 1:
        log("bench.py: the library runs on ONE GPU; elements are independent, so a multi-GPU "
            "run would be a contiguous split of the element range with no exchange. "
            "Run with --gpus 1.")
        return 2

    import numpy as np
    import torch

    from paper_2604_19906_amd import tpo
    from paper_2604_19906_amd import workloads as wl

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible")
        return 1
    torch.cuda.set_device(0)
    tpo.check(tpo.tpo_create(), "tpo_create")      # raises if libtpo.so is missing

    if args.op == "convection":
        return bench_convection(args, torch, tpo, wl)
    if args.op == "aniso":
        return bench_aniso(args, torch, tpo, wl)

    w = wl.CONFIGS[args.workload]
    if args.elems:
        w = wl.Workload(w.name + f"_E{args.elems}", w.index, w.dtype, w.n, args.elems,
                        w.u_dist, w.distinct_s)
    if args.n:
        w = wl.Workload(w.name + f"_n{args.n}", w.index, w.dtype, args.n, w.num_elems,
                        w.u_dist, w.distinct_s)
    variant = {"auto": tpo.TPO_VARIANT_AUTO, "pencil": tpo.TPO_VARIANT_PENCIL,
               "mfma": tpo.TPO_VARIANT_MFMA,
               "pencil_mm": tpo.TPO_VARIANT_PENCIL_MM}[args.variant]
    dt = tpo.TPO_F64 if w.dtype == "f64" else tpo.TPO_F32
    sep = args.op == "ihelm_sep"
    half = args.op in ("forward", "backward")
    if half:
        if args.variant != "auto":
            log("bench.py: the transform halves have one kernel family; --variant does not apply")
            return 2
        chosen = tpo.TPO_VARIANT_PENCIL
    elif sep:
        chosen = variant or tpo.tpo_ihelm_sep_variant_for_batch(w.n, dt, not w.distinct_s, w.num_elems)
    else:
        chosen = variant or tpo.tpo_ihelm_variant_for_batch(w.n, dt, not w.distinct_s, w.num_elems)
    chosen_name = {tpo.TPO_VARIANT_PENCIL: "pencil", tpo.TPO_VARIANT_MFMA: "mfma",
                   tpo.TPO_VARIANT_PENCIL_MM: "pencil_mm"}[chosen]

    # ---- inputs: seeded, generated block by block on the host, resident in HBM -------------
    t0 = time.time()
    tu, tsx, tsy, tsz, td = wl.to_device(w)
    tv = torch.empty_like(tu)
    tlam = [torch.from_numpy(np.ascontiguousarray(a)).cuda() for a in wl.sep_inputs(w)]
    torch.cuda.synchronize()
    nfields = 2 if (sep or half) else 3
    log(f"[bench] {w.name} ({args.op}): inputs resident after {time.time() - t0:.1f}s "
        f"({3 * tu.numel() * tu.element_size() / 1e9:.2f} GB for u, D, v); variant {chosen_name}")

    stream = torch.cuda.current_stream()
    ptrs = (tu.data_ptr(), tsx.data_ptr(), tsy.data_ptr(), tsz.data_ptr(), td.data_ptr(),
            tv.data_ptr())
    sep_ptrs = ptrs[:4] + tuple(t.data_ptr() for t in tlam) + (tv.data_ptr(),)

    direction = tpo.TPO_FORWARD if args.op == "forward" else tpo.TPO_BACKWARD

    def step():
        if half:
            rc = tpo.tpo_transform_apply(*ptrs[:4], ptrs[5], w.n, w.num_elems, dt, direction,
                                         stream.cuda_stream)
        elif sep:
            rc = tpo.tpo_ihelm_apply_sep_variant(*sep_ptrs, w.n, w.num_elems, dt,
                                                 stream.cuda_stream, variant)
        else:
            rc = tpo.tpo_ihelm_apply_variant(*ptrs, w.n, w.num_elems, dt, stream.cuda_stream,
                                             variant)
        if rc != tpo.TPO_OK:
            raise tpo.TpoError(rc, "tpo_" + args.op + "_apply")

    # ---- streaming ceiling first: the plain v = u .* D kernel over the same three fields, same
    # traffic, no other work; run for 0.3 s before it is timed, which also brings the clocks to
    # their loaded state before the warm-up steps
    def stream_step():
        rc = tpo.tpo_stream_scale(ptrs[0], ptrs[4], ptrs[5], tu.numel(), dt, stream.cuda_stream)
        if rc != tpo.TPO_OK:
            raise tpo.TpoError(rc, "tpo_stream_scale")

    loaded_state(torch, stream_step)
    sev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in range(10)]
    for a, b in sev:
        a.record(stream)
        stream_step()
        b.record(stream)
    torch.cuda.synchronize()
    stream_ms = sum(a.elapsed_time(b) for a, b in sev) / len(sev)
    stream_gbs = w.bytes_per_elem * w.num_elems / (stream_ms * 1e-3) / 1e9
    log(f"[bench] streaming ceiling v=u.*D: {stream_ms:.4f} ms = {stream_gbs:.0f} GB/s")

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()

    # ---- timed region: exactly K steps, device-synchronised on both sides -------------------
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in range(args.steps)]
    torch.cuda.synchronize()
    t_begin = time.perf_counter()
    for a, b in evs:
        a.record(stream)
        step()
        b.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_begin
    kernel_ms = [a.elapsed_time(b) for a, b in evs]
    avg_kernel_ms = sum(kernel_ms) / len(kernel_ms)
    ms_per_step = wall * 1e3 / args.steps

    elems_per_s = w.num_elems / (ms_per_step * 1e-3)
    # algorithmic traffic: u and v, plus D when it is an input; the separable form adds
    # 3 adds and a division per point to the flop count
    alg_bytes = w.bytes_per_elem * w.num_elems * nfields // 3
    if half:
        alg_flop = 6 * w.n ** 4 * w.num_elems
    else:
        alg_flop = (w.flop_per_elem + (4 * w.n ** 3 if sep else 0)) * w.num_elems
    achieved_gbs = alg_bytes / (avg_kernel_ms * 1e-3) / 1e9
    achieved_tflops = alg_flop / (avg_kernel_ms * 1e-3) / 1e12
    log(f"[bench] kernel avg {avg_kernel_ms:.4f} ms (min {min(kernel_ms):.4f}, max "
        f"{max(kernel_ms):.4f}); wall/step {ms_per_step:.4f} ms; {achieved_gbs:.0f} GB/s; "
        f"{achieved_tflops:.2f} TFLOP/s")

    # ---- sanity: the timed output is the operator's (oracle on a few elements) --------------
    import oracle
    step()
    torch.cuda.synchronize()
    sx, sy, sz = wl.direction_matrices(w)
    lo, hi = 0, min(64, w.num_elems)
    if half:
        ref = (oracle.forward if args.op == "forward" else oracle.backward)(
            wl.field_u(w, lo, hi), sx, sy, sz)
    elif sep:
        ref = oracle.ihelm_apply_sep(wl.field_u(w, lo, hi), sx, sy, sz, *wl.sep_inputs(w, lo, hi))
    else:
        ref = oracle.ihelm_apply(wl.field_u(w, lo, hi), sx, sy, sz, wl.diagonal_d(w, lo, hi))
    got = tv[lo:hi].cpu().numpy()
    err = oracle.max_rel_err_per_element(got, ref)
    err_global = float(np.abs(got.astype(np.float64) - ref).max() / np.abs(ref).max())
    tol = 1e-12 if w.dtype == "f64" else 2e-5
    if not err <= tol:
        log(f"[bench] PARITY FAILURE on the timed output: {err:.3e} > {tol}")
        return 1

    # ---- CPU baseline: the oracle on this machine's host cores, bounded sample ---------------
    cpu = None
    if not args.no_cpu_baseline:
        ns = min(args.cpu_sample, w.num_elems)
        hu = wl.field_u(w, 0, ns)
        cores = oracle.max_threads()
        if half:
            fn = oracle.forward if args.op == "forward" else oracle.backward
            cores = 1                        # the oracle's transform halves are single-threaded
            ns = min(ns, 16384)
            hu = hu[:ns]
            fn(hu[:256], sx, sy, sz)                                        # load + warm
            run = lambda: fn(hu, sx, sy, sz)
        elif sep:
            hl = wl.sep_inputs(w, 0, ns)
            oracle.ihelm_apply_sep(hu[:256], sx, sy, sz, *hl[:3], hl[3][:256])   # load + warm
            run = lambda: oracle.ihelm_apply_sep(hu, sx, sy, sz, *hl)
        else:
            hd = wl.diagonal_d(w, 0, ns)
            oracle.ihelm_apply(hu[:256], sx, sy, sz, hd[:256])          # load + warm
            run = lambda: oracle.ihelm_apply(hu, sx, sy, sz, hd)
        rate, passes, cpu_s = timed_passes(run, ns, cores)
        cpu = {"value": rate, "unit": "elements/s", "cores": cores, "kind": "oracle",
               "sample": f"first {ns} elements of {w.name}, {passes} pass(es), {cores} host "
                         f"thread(s) ({cpu_s:.2f} s wall)",
               "gflops": rate * w.flop_per_elem / 1e9}
        log(f"[bench] CPU oracle baseline: {rate:.0f} elements/s on {cores} threads")
        if not half and not sep:
            # the same oracle on one thread, on the paper's batch of 8192 elements (Sec. 6.1)
            n1 = min(8192, w.num_elems)
            t1 = time.perf_counter()
            oracle.ihelm_apply(hu[:n1], sx, sy, sz, hd[:n1], nthreads=1)
            one_s = time.perf_counter() - t1
            cpu["one_thread"] = {"value": n1 / one_s, "unit": "elements/s", "cores": 1,
                                 "sample": f"first {n1} elements, one pass ({one_s:.2f} s wall)"}
            log(f"[bench] CPU oracle baseline: {n1 / one_s:.0f} elements/s on 1 thread")

    srt = sorted(kernel_ms)
    median_ms = 0.5 * (srt[(len(srt) - 1) // 2] + srt[len(srt) // 2])
    fp_frac = achieved_tflops / FP_PEAK_TFLOPS[w.dtype]
    out = {
        "metric": "elements/s + GFLOP/s and % of binding roofline, fp64 n=11 TPO apply",
        "value": elems_per_s,
        "unit": "elements/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": w.name, "op": args.op, "n": w.n, "num_elems": w.num_elems,
                   "variant": chosen_name, "layout": "[E,n,n,n] element-contiguous",
                   "parallelism": "1 GPU"},
        "gflops": alg_flop / (ms_per_step * 1e-3) / 1e9,
        "kernel_ms_avg": avg_kernel_ms,
        "kernel_ms_median": median_ms,
        "kernel_ms_min": min(kernel_ms),
        "fp_frac_of_peak": fp_frac,
        "stream_ceiling_gbs": stream_gbs,
        # fraction of what the plain streaming kernel reaches on the same arrays (three fields)
        "frac_of_stream_ceiling": (w.bytes_per_elem * w.num_elems / (avg_kernel_ms * 1e-3) / 1e9)
                                  / stream_gbs if not (sep or half) else None,
        # both fractions of their roofs; the operator sits left of the ridge, so HBM binds
        "binding_roofline": "hbm", "hbm_frac": achieved_gbs / HBM_PEAK_GBS, "fp_frac": fp_frac,
        "parity_max_rel_err_sample": err,
        "parity_global_rel_err_sample": err_global,
        # achieved / frac: from the AVERAGE kernel time of the K timed launches; the *_median
        # pair from their median (a few slow launches at the start move the average only)
        "roofline": {"bound": "hbm", "achieved": achieved_gbs, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved_gbs / HBM_PEAK_GBS,
                     "achieved_median": alg_bytes / (median_ms * 1e-3) / 1e9,
                     "frac_median": alg_bytes / (median_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                     "traffic": stored_traffic(w.name + (":sep" if sep else ":" + args.op if half else ""),
                                               chosen_name, "transform" if half else "ihelm")},
        "cpu_baseline": cpu,
    }
    print(json.dumps(out), flush=True)
    tpo.tpo_destroy()
    return 0


if __name__ == "__main__":
    sys.exit(main())

"""Helpers for the GPU tests: upload seeded host inputs, call the C-ABI library through the
binding, download the result.  Nothing here computes the operator."""
import numpy as np
import torch

from paper_2604_19906_amd import tpo
from paper_2604_19906_amd import workloads as wl

TOL = {"f64": 1e-12, "f32": 2e-5}      # max-norm relative error per element
VARIANTS = {"pencil": tpo.TPO_VARIANT_PENCIL, "mfma": tpo.TPO_VARIANT_MFMA,
            "pencil_mm": tpo.TPO_VARIANT_PENCIL_MM}


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def run(u, sx, sy, sz, d, variant=tpo.TPO_VARIANT_AUTO, same_s_pointer=None):
    """Host arrays in, host array out; all work in between is one library call."""
    tu, td = dev(u), dev(d)
    if same_s_pointer is None:
        same_s_pointer = sx is sy and sy is sz
    if same_s_pointer:
        ts = dev(sx)
        tsx = tsy = tsz = ts
    else:
        tsx, tsy, tsz = dev(sx), dev(sy), dev(sz)
    tv = tpo.apply_tensors(tu, tsx, tsy, tsz, td, variant=variant)
    torch.cuda.synchronize()
    return tv.cpu().numpy()


def upload_full(w):
    return wl.to_device(w)


def oracle_every_element(num_elems, host_block, device_inputs, oracle_fn, outs, tol, label,
                         block=16384, workers=6, oracle_in_pool=False):
    """The oracle on EVERY element of a full-size workload, block by block.

    ``host_block(lo, hi)`` draws the block's host inputs again from the seeds (oracle inputs are
    never read back from the device); ``device_inputs(lo, hi)`` returns the device copies of the
    per-element arrays among them, in the same order, and is only compared with them;
    ``oracle_fn(*host inputs)`` is the CPU oracle; ``outs`` maps a name to a device result.
    Blocks are drawn by a thread pool; the oracle runs in the calling thread (it has its own
    OpenMP threads) unless ``oracle_in_pool`` (for its single-threaded functions).
    Returns name -> worst max-norm relative error per element."""
    from concurrent.futures import ThreadPoolExecutor

    import oracle

    spans = [(lo, min(num_elems, lo + block)) for lo in range(0, num_elems, block)]
    worst = {name: 0.0 for name in outs}

    def work(span):
        lo, hi = span
        host = host_block(lo, hi)
        return lo, hi, host, (oracle_fn(*host) if oracle_in_pool else None)

    with ThreadPoolExecutor(max_workers=workers) as ex:
        for lo, hi, host, ref in ex.map(work, spans):
            for h, t in zip(host, device_inputs(lo, hi)):
                if t is not None:
                    assert np.array_equal(h, t.cpu().numpy()), f"{label}: inputs differ at {lo}"
            if ref is None:
                ref = oracle_fn(*host)
            for name, tv in outs.items():
                err = oracle.max_rel_err_per_element(tv[lo:hi].cpu().numpy(), ref)
                assert err <= tol, f"{label} {name}: elements {lo}..{hi}: err {err:.3e}"
                worst[name] = max(worst[name], err)
    return worst

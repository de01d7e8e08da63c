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

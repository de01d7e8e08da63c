// Internal interfaces of libtpo (not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>

#include "tpo.h"

namespace tpo {

struct ApplyArgs {
    const void *u, *sx, *sy, *sz, *d;
    void *v;
    long long num_elems;
    hipStream_t stream;
};

// One kernel instantiation for a fixed (n, dtype): how to launch it and how to prepare it
// once per device (e.g. raise its dynamic-LDS limit).
struct KernelEntry {
    hipError_t (*launch)(const ApplyArgs &);
    hipError_t (*prepare)();
};

// dtype index: 0 = f64, 1 = f32.  n in 1..TPO_MAX_N.  Returns nullptr when the family has
// no kernel for that shape.
const KernelEntry *pencil_entry(int n, int dtype);
const KernelEntry *mfma_entry(int n, int dtype);
const KernelEntry *pencil_mm_entry(int n, int dtype);   // fp32 only

// Pure host validation shared by the entry points; touches no HIP state.
int validate_apply(const void *u, const void *sx, const void *sy, const void *sz,
                   const void *d, const void *v, int n, long long num_elems, int dtype,
                   int variant);

}  // namespace tpo

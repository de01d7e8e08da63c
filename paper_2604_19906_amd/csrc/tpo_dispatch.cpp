// Kernel-family lookup: maps (n, dtype) to the instantiation tables of each family.
#include "tpo_internal.h"

namespace tpo {

const KernelEntry *pencil_entry_f64(int n);
const KernelEntry *pencil_entry_f32(int n);
const KernelEntry *mfma_entry_f64(int n);
const KernelEntry *mfma_entry_f32(int n);
const KernelEntry *pencil_mm_entry_f32(int n);
const ConvectionEntry *convection_entry_f64(int n);
const ConvectionEntry *convection_entry_f32(int n);
const TransformEntry *transform_entry_f64(int n);
const TransformEntry *transform_entry_f32(int n);

const KernelEntry *pencil_entry(int n, int dtype)
{
    return dtype == TPO_F64 ? pencil_entry_f64(n) : pencil_entry_f32(n);
}

const KernelEntry *mfma_entry(int n, int dtype)
{
    return dtype == TPO_F64 ? mfma_entry_f64(n) : mfma_entry_f32(n);
}

const KernelEntry *pencil_mm_entry(int n, int dtype)
{
    return dtype == TPO_F32 ? pencil_mm_entry_f32(n) : nullptr;
}

const ConvectionEntry *convection_entry(int n, int dtype)
{
    return dtype == TPO_F64 ? convection_entry_f64(n) : convection_entry_f32(n);
}

const TransformEntry *transform_entry(int n, int dtype)
{
    return dtype == TPO_F64 ? transform_entry_f64(n) : transform_entry_f32(n);
}

}  // namespace tpo

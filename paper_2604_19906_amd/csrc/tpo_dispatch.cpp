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

const ConvectionEntry *convection_rect_entry_f64(int n_v, int n_q);
const ConvectionEntry *convection_rect_entry_f32(int n_v, int n_q);
int convection_rect_count_f64();
int convection_rect_count_f32();
const ConvectionEntry *convection_rect_at_f64(int k);
const ConvectionEntry *convection_rect_at_f32(int k);

const ConvectionEntry *convection_entry(int n_v, int n_q, int dtype)
{
    if (n_v == n_q) return dtype == TPO_F64 ? convection_entry_f64(n_v) : convection_entry_f32(n_v);
    return dtype == TPO_F64 ? convection_rect_entry_f64(n_v, n_q)
                            : convection_rect_entry_f32(n_v, n_q);
}

int convection_rect_count(int dtype)
{
    return dtype == TPO_F64 ? convection_rect_count_f64() : convection_rect_count_f32();
}

const ConvectionEntry *convection_rect_at(int k, int dtype)
{
    return dtype == TPO_F64 ? convection_rect_at_f64(k) : convection_rect_at_f32(k);
}

const TransformEntry *transform_entry(int n, int dtype)
{
    return dtype == TPO_F64 ? transform_entry_f64(n) : transform_entry_f32(n);
}

}  // namespace tpo

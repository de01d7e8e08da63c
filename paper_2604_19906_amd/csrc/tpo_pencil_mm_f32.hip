// Instantiations of the fp32 pencil kernels with 4x4x1 matrix-core products, n = 1 .. 16.
#include "tpo_pencil_mm.hpp"

namespace tpo {

const KernelEntry *pencil_mm_entry_f32(int n)
{
    static const KernelEntry table[TPO_MAX_N] = {
        TPO_PENCIL_MM_ENTRY(1),  TPO_PENCIL_MM_ENTRY(2),  TPO_PENCIL_MM_ENTRY(3),
        TPO_PENCIL_MM_ENTRY(4),  TPO_PENCIL_MM_ENTRY(5),  TPO_PENCIL_MM_ENTRY(6),
        TPO_PENCIL_MM_ENTRY(7),  TPO_PENCIL_MM_ENTRY(8),  TPO_PENCIL_MM_ENTRY(9),
        TPO_PENCIL_MM_ENTRY(10), TPO_PENCIL_MM_ENTRY(11), TPO_PENCIL_MM_ENTRY(12),
        TPO_PENCIL_MM_ENTRY(13), TPO_PENCIL_MM_ENTRY(14), TPO_PENCIL_MM_ENTRY(15),
        TPO_PENCIL_MM_ENTRY(16),
    };
    return (n >= 1 && n <= TPO_MAX_N) ? &table[n - 1] : nullptr;
}

}  // namespace tpo

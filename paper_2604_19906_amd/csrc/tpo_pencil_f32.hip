// Instantiations of the pencil kernel family for float, n = 1 .. 16.
#include "tpo_pencil.hpp"

namespace tpo {

const KernelEntry *pencil_entry_f32(int n)
{
    static const KernelEntry table[TPO_MAX_N] = {
        TPO_PENCIL_ENTRY(float, 1),  TPO_PENCIL_ENTRY(float, 2),  TPO_PENCIL_ENTRY(float, 3),
        TPO_PENCIL_ENTRY(float, 4),  TPO_PENCIL_ENTRY(float, 5),  TPO_PENCIL_ENTRY(float, 6),
        TPO_PENCIL_ENTRY(float, 7),  TPO_PENCIL_ENTRY(float, 8),  TPO_PENCIL_ENTRY(float, 9),
        TPO_PENCIL_ENTRY(float, 10), TPO_PENCIL_ENTRY(float, 11), TPO_PENCIL_ENTRY(float, 12),
        TPO_PENCIL_ENTRY(float, 13), TPO_PENCIL_ENTRY(float, 14), TPO_PENCIL_ENTRY(float, 15),
        TPO_PENCIL_ENTRY(float, 16),
    };
    return (n >= 1 && n <= TPO_MAX_N) ? &table[n - 1] : nullptr;
}

}  // namespace tpo

// Instantiations of the convection volume-term kernels for float, n = 1 .. 16.
#include "tpo_convection.hpp"

namespace tpo {

const ConvectionEntry *convection_entry_f32(int n)
{
    static const ConvectionEntry table[TPO_MAX_N] = {
        TPO_CONVECTION_ENTRY(float, 1), TPO_CONVECTION_ENTRY(float, 2),
        TPO_CONVECTION_ENTRY(float, 3), TPO_CONVECTION_ENTRY(float, 4),
        TPO_CONVECTION_ENTRY(float, 5), TPO_CONVECTION_ENTRY(float, 6),
        TPO_CONVECTION_ENTRY(float, 7), TPO_CONVECTION_ENTRY(float, 8),
        TPO_CONVECTION_ENTRY(float, 9), TPO_CONVECTION_ENTRY(float, 10),
        TPO_CONVECTION_ENTRY(float, 11), TPO_CONVECTION_ENTRY(float, 12),
        TPO_CONVECTION_ENTRY(float, 13), TPO_CONVECTION_ENTRY(float, 14),
        TPO_CONVECTION_ENTRY(float, 15), TPO_CONVECTION_ENTRY(float, 16),
    };
    return (n >= 1 && n <= TPO_MAX_N) ? &table[n - 1] : nullptr;
}

}  // namespace tpo

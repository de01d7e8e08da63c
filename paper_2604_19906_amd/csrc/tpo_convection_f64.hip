// Instantiations of the convection volume-term kernels for double, n = 1 .. 16.
#include "tpo_convection.hpp"

namespace tpo {

const ConvectionEntry *convection_entry_f64(int n)
{
    static const ConvectionEntry table[TPO_MAX_N] = {
        TPO_CONVECTION_ENTRY(double, 1), TPO_CONVECTION_ENTRY(double, 2),
        TPO_CONVECTION_ENTRY(double, 3), TPO_CONVECTION_ENTRY(double, 4),
        TPO_CONVECTION_ENTRY(double, 5), TPO_CONVECTION_ENTRY(double, 6),
        TPO_CONVECTION_ENTRY(double, 7), TPO_CONVECTION_ENTRY(double, 8),
        TPO_CONVECTION_ENTRY(double, 9), TPO_CONVECTION_ENTRY(double, 10),
        TPO_CONVECTION_ENTRY(double, 11), TPO_CONVECTION_ENTRY(double, 12),
        TPO_CONVECTION_ENTRY(double, 13), TPO_CONVECTION_ENTRY(double, 14),
        TPO_CONVECTION_ENTRY(double, 15), TPO_CONVECTION_ENTRY(double, 16),
    };
    return (n >= 1 && n <= TPO_MAX_N) ? &table[n - 1] : nullptr;
}

}  // namespace tpo

// Instantiations of the transform kernels (forward and backward half on their own) for double,
// n = 1 .. 16.
#include "tpo_transform.hpp"

namespace tpo {

const TransformEntry *transform_entry_f64(int n)
{
    static const TransformEntry table[TPO_MAX_N] = {
        TPO_TRANSFORM_ENTRY(double, 1), TPO_TRANSFORM_ENTRY(double, 2),
        TPO_TRANSFORM_ENTRY(double, 3), TPO_TRANSFORM_ENTRY(double, 4),
        TPO_TRANSFORM_ENTRY(double, 5), TPO_TRANSFORM_ENTRY(double, 6),
        TPO_TRANSFORM_ENTRY(double, 7), TPO_TRANSFORM_ENTRY(double, 8),
        TPO_TRANSFORM_ENTRY(double, 9), TPO_TRANSFORM_ENTRY(double, 10),
        TPO_TRANSFORM_ENTRY(double, 11), TPO_TRANSFORM_ENTRY(double, 12),
        TPO_TRANSFORM_ENTRY(double, 13), TPO_TRANSFORM_ENTRY(double, 14),
        TPO_TRANSFORM_ENTRY(double, 15), TPO_TRANSFORM_ENTRY(double, 16),
    };
    return (n >= 1 && n <= TPO_MAX_N) ? &table[n - 1] : nullptr;
}

}  // namespace tpo

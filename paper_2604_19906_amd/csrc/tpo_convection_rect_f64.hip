// Instantiations of the rectangular convection kernels for double: n_v nodes, n_q > n_v quadrature
// points per direction, n_q in {n_v + 1, n_v + 2, ceil(3 n_v / 2)} (over-integration), n_q <= 16.
#include "tpo_convection.hpp"

namespace tpo {

const ConvectionEntry *convection_rect_entry_f64(int n_v, int n_q)
{
    static const ConvectionRectEntry table[] = {
        TPO_CONVECTION_RECT_ENTRY(double, 2, 3),
        TPO_CONVECTION_RECT_ENTRY(double, 2, 4),
        TPO_CONVECTION_RECT_ENTRY(double, 3, 4),
        TPO_CONVECTION_RECT_ENTRY(double, 3, 5),
        TPO_CONVECTION_RECT_ENTRY(double, 4, 5),
        TPO_CONVECTION_RECT_ENTRY(double, 4, 6),
        TPO_CONVECTION_RECT_ENTRY(double, 5, 6),
        TPO_CONVECTION_RECT_ENTRY(double, 5, 7),
        TPO_CONVECTION_RECT_ENTRY(double, 5, 8),
        TPO_CONVECTION_RECT_ENTRY(double, 6, 7),
        TPO_CONVECTION_RECT_ENTRY(double, 6, 8),
        TPO_CONVECTION_RECT_ENTRY(double, 6, 9),
        TPO_CONVECTION_RECT_ENTRY(double, 7, 8),
        TPO_CONVECTION_RECT_ENTRY(double, 7, 9),
        TPO_CONVECTION_RECT_ENTRY(double, 7, 11),
        TPO_CONVECTION_RECT_ENTRY(double, 8, 9),
        TPO_CONVECTION_RECT_ENTRY(double, 8, 10),
        TPO_CONVECTION_RECT_ENTRY(double, 8, 12),
        TPO_CONVECTION_RECT_ENTRY(double, 9, 10),
        TPO_CONVECTION_RECT_ENTRY(double, 9, 11),
        TPO_CONVECTION_RECT_ENTRY(double, 9, 14),
        TPO_CONVECTION_RECT_ENTRY(double, 10, 11),
        TPO_CONVECTION_RECT_ENTRY(double, 10, 12),
        TPO_CONVECTION_RECT_ENTRY(double, 10, 15),
        TPO_CONVECTION_RECT_ENTRY(double, 11, 12),
        TPO_CONVECTION_RECT_ENTRY(double, 11, 13),
        TPO_CONVECTION_RECT_ENTRY(double, 12, 13),
        TPO_CONVECTION_RECT_ENTRY(double, 12, 14),
    };
    for (const ConvectionRectEntry &r : table)
        if (r.n_v == n_v && r.n_q == n_q) return &r.entry;
    return nullptr;
}

int convection_rect_count_f64() { return 28; }
const ConvectionEntry *convection_rect_at_f64(int k)
{
    // prepare() walks every instantiation through this accessor
    static const int shapes[][2] = {{2, 3}, {2, 4}, {3, 4}, {3, 5}, {4, 5}, {4, 6}, {5, 6}, {5, 7}, {5, 8}, {6, 7}, {6, 8}, {6, 9}, {7, 8}, {7, 9}, {7, 11}, {8, 9}, {8, 10}, {8, 12}, {9, 10}, {9, 11}, {9, 14}, {10, 11}, {10, 12}, {10, 15}, {11, 12}, {11, 13}, {12, 13}, {12, 14}};
    return (k >= 0 && k < 28) ? convection_rect_entry_f64(shapes[k][0], shapes[k][1]) : nullptr;
}

}  // namespace tpo

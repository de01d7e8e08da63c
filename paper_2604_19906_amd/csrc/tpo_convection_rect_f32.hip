// Instantiations of the rectangular convection kernels for float: n_v nodes, n_q > n_v quadrature
// points per direction, n_q in {n_v + 1, n_v + 2, ceil(3 n_v / 2)} (over-integration), n_q <= 16.
#include "tpo_convection.hpp"

namespace tpo {

const ConvectionEntry *convection_rect_entry_f32(int n_v, int n_q)
{
    static const ConvectionRectEntry table[] = {
        TPO_CONVECTION_RECT_ENTRY(float, 2, 3),
        TPO_CONVECTION_RECT_ENTRY(float, 2, 4),
        TPO_CONVECTION_RECT_ENTRY(float, 3, 4),
        TPO_CONVECTION_RECT_ENTRY(float, 3, 5),
        TPO_CONVECTION_RECT_ENTRY(float, 4, 5),
        TPO_CONVECTION_RECT_ENTRY(float, 4, 6),
        TPO_CONVECTION_RECT_ENTRY(float, 5, 6),
        TPO_CONVECTION_RECT_ENTRY(float, 5, 7),
        TPO_CONVECTION_RECT_ENTRY(float, 5, 8),
        TPO_CONVECTION_RECT_ENTRY(float, 6, 7),
        TPO_CONVECTION_RECT_ENTRY(float, 6, 8),
        TPO_CONVECTION_RECT_ENTRY(float, 6, 9),
        TPO_CONVECTION_RECT_ENTRY(float, 7, 8),
        TPO_CONVECTION_RECT_ENTRY(float, 7, 9),
        TPO_CONVECTION_RECT_ENTRY(float, 7, 11),
        TPO_CONVECTION_RECT_ENTRY(float, 8, 9),
        TPO_CONVECTION_RECT_ENTRY(float, 8, 10),
        TPO_CONVECTION_RECT_ENTRY(float, 8, 12),
        TPO_CONVECTION_RECT_ENTRY(float, 9, 10),
        TPO_CONVECTION_RECT_ENTRY(float, 9, 11),
        TPO_CONVECTION_RECT_ENTRY(float, 9, 14),
        TPO_CONVECTION_RECT_ENTRY(float, 10, 11),
        TPO_CONVECTION_RECT_ENTRY(float, 10, 12),
        TPO_CONVECTION_RECT_ENTRY(float, 10, 15),
        TPO_CONVECTION_RECT_ENTRY(float, 11, 12),
        TPO_CONVECTION_RECT_ENTRY(float, 11, 13),
        TPO_CONVECTION_RECT_ENTRY(float, 12, 13),
        TPO_CONVECTION_RECT_ENTRY(float, 12, 14),
    };
    for (const ConvectionRectEntry &r : table)
        if (r.n_v == n_v && r.n_q == n_q) return &r.entry;
    return nullptr;
}

int convection_rect_count_f32() { return 28; }
const ConvectionEntry *convection_rect_at_f32(int k)
{
    // prepare() walks every instantiation through this accessor
    static const int shapes[][2] = {{2, 3}, {2, 4}, {3, 4}, {3, 5}, {4, 5}, {4, 6}, {5, 6}, {5, 7}, {5, 8}, {6, 7}, {6, 8}, {6, 9}, {7, 8}, {7, 9}, {7, 11}, {8, 9}, {8, 10}, {8, 12}, {9, 10}, {9, 11}, {9, 14}, {10, 11}, {10, 12}, {10, 15}, {11, 12}, {11, 13}, {12, 13}, {12, 14}};
    return (k >= 0 && k < 28) ? convection_rect_entry_f32(shapes[k][0], shapes[k][1]) : nullptr;
}

}  // namespace tpo

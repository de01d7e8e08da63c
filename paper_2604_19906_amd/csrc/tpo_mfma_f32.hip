// Instantiations of the matrix-core kernel family for float, n = 1 .. 16.
#include "tpo_mfma.hpp"

namespace tpo {

// Elements per workgroup, wavefronts per workgroup and hint bits per n.  The default deals
// at least eight tiles to four wavefronts; the specialisations come from a sweep on MI355X.
template <int N>
struct MfmaTune_f32 {
    static constexpr int TILES = (N * N + 15) / 16;
    static constexpr int G = (8 + TILES - 1) / TILES;
    static constexpr int NW = 4;
    static constexpr int HINT = 2;
    static constexpr bool PERSIST = false;
    static constexpr int WAVES = 1;
    static constexpr bool XCD = false;
};

// n = 14: two elements (26 tiles) per workgroup: 2.11-2.12 against 2.17 ms on 262144 elements
// (n = 15, 16: the default is within 0.5 % of the best of eight wavefronts per workgroup, cached
// or fully non-temporal accesses, two elements per workgroup and die renumbering).
template <>
struct MfmaTune_f32<14> {
    static constexpr int G = 2;
    static constexpr int NW = 4;
    static constexpr int HINT = 2;
    static constexpr bool PERSIST = false;
    static constexpr int WAVES = 1;
    static constexpr bool XCD = false;
};

template <int N>
using Launcher = MfmaLauncher<float, N, MfmaTune_f32<N>::G, MfmaTune_f32<N>::NW, MfmaTune_f32<N>::HINT, MfmaTune_f32<N>::PERSIST,
                              MfmaTune_f32<N>::WAVES, MfmaTune_f32<N>::XCD>;
#define ENTRY(N) KernelEntry { &Launcher<N>::launch, &Launcher<N>::launch_sep, &Launcher<N>::prepare }

const KernelEntry *mfma_entry_f32(int n)
{
    static const KernelEntry table[TPO_MAX_N] = {
        ENTRY(1),  ENTRY(2),  ENTRY(3),  ENTRY(4),  ENTRY(5),  ENTRY(6),  ENTRY(7),  ENTRY(8),
        ENTRY(9),  ENTRY(10), ENTRY(11), ENTRY(12), ENTRY(13), ENTRY(14), ENTRY(15), ENTRY(16),
    };
    return (n >= 1 && n <= TPO_MAX_N) ? &table[n - 1] : nullptr;
}

}  // namespace tpo

// Instantiations of the matrix-core kernel family for double, n = 1 .. 16.
#include "tpo_mfma.hpp"

namespace tpo {

// Elements per workgroup, wavefronts per workgroup and hint bits per n.  The default deals
// at least eight tiles to four wavefronts; the specialisations come from a sweep on MI355X.
template <int N>
struct MfmaTune_f64 {
    static constexpr int TILES = (N * N + 15) / 16;
    static constexpr int G = (8 + TILES - 1) / TILES;
    static constexpr int NW = 4;
    static constexpr int HINT = 2;
    static constexpr bool PERSIST = false;
    static constexpr int WAVES = 1;
    static constexpr bool XCD = false;
};

// n = 16: one workgroup per element, non-temporal stores (on the named workload, alternating
// libraries on one box: 1.115-1.118 ms against 1.139 with cached stores, 1.128 with non-temporal
// loads as well, 1.156 with non-temporal loads only; also ahead on small batches: E = 4096 68.7
// against 76.8 us, 8192 143 against 146; the persistent form measured 0.08 ms slower).
template <>
struct MfmaTune_f64<16> {
    static constexpr int G = 1;
    static constexpr int NW = 4;
    static constexpr int HINT = 2;
    static constexpr bool PERSIST = false;
    static constexpr int WAVES = 1;     // asking for a fourth wavefront per SIMD: 1.127 against 1.117 ms
    static constexpr bool XCD = false;  // die renumbering: 1.123 against 1.117 ms
};
// n = 11: persistent grid with register prefetch of the next element (1.69 ms against 1.87 ms).
template <>
struct MfmaTune_f64<11> {
    static constexpr int G = 1;
    static constexpr int NW = 4;
    static constexpr int HINT = 0;
    static constexpr bool PERSIST = true;
    static constexpr int WAVES = 1;
    static constexpr bool XCD = false;
};

template <int N>
using Launcher = MfmaLauncher<double, N, MfmaTune_f64<N>::G, MfmaTune_f64<N>::NW, MfmaTune_f64<N>::HINT, MfmaTune_f64<N>::PERSIST,
                              MfmaTune_f64<N>::WAVES, MfmaTune_f64<N>::XCD>;
#define ENTRY(N) KernelEntry { &Launcher<N>::launch, &Launcher<N>::launch_sep, &Launcher<N>::prepare }

const KernelEntry *mfma_entry_f64(int n)
{
    static const KernelEntry table[TPO_MAX_N] = {
        ENTRY(1),  ENTRY(2),  ENTRY(3),  ENTRY(4),  ENTRY(5),  ENTRY(6),  ENTRY(7),  ENTRY(8),
        ENTRY(9),  ENTRY(10), ENTRY(11), ENTRY(12), ENTRY(13), ENTRY(14), ENTRY(15), ENTRY(16),
    };
    return (n >= 1 && n <= TPO_MAX_N) ? &table[n - 1] : nullptr;
}

}  // namespace tpo

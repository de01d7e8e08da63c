// fp32 pencil kernels whose mode products run on the matrix cores as 4x4x1 outer products.
//
// Same data movement as the vector-FMA pencil kernels (tpo_pencil.hpp): one lane owns one
// pencil, the cube is re-distributed through LDS between axes, u_e and v_e move coalesced,
// D_e arrives in its axis-2 pencil layout.  Only the arithmetic differs.  With packed fp32
// arithmetic unavailable, a vector FMA retires 64 fp32 FMAs in 4 cycles; the instruction
// v_mfma_f32_4x4x1_16B_f32 retires 256 in 8.  It computes, in each of 16 four-lane blocks, the
// outer product of a 4-vector A with a 4-vector B (one B value per lane) and adds it to four
// accumulator registers per lane.  With the A-broadcast controls (cbsz = 4, abid = k) every
// block takes its A vector from lanes 4k..4k+3 of the A register, so for every lane
//
//     acc[r] += Areg[lane 4k + r] * b        r = 0..3
//
// which is exactly four FMAs of a pencil product y[4*rg + r] += M[4*rg + r][l] * x[l] with
// wavefront-uniform coefficients.  One A register holds 16 such coefficient quadruples; the
// n * ceil(n/4) quadruples of one matrix in one direction fill ceil(n * ceil(n/4) / 16)
// registers (4 for n = 13), built once per workgroup from the matrix in global memory.
// Rows n .. 4*ceil(n/4)-1 have zero coefficients; the padding costs 16/13 at n = 13.
#pragma once
#include <hip/hip_runtime.h>

#include <utility>

#include "tpo_pencil.hpp"

namespace tpo {

typedef float mm_f4 __attribute__((ext_vector_type(4)));

template <int N>
struct MmShape {
    // A single left-over output row (n = 5, 9, 13) is cheaper as n vector FMAs with scalar
    // coefficients (4n cycles) than as n more matrix instructions (8n cycles).
    static constexpr bool REM_VALU = (N % 4 == 1) && (N > 1);
    static constexpr int RG = REM_VALU ? N / 4 : (N + 3) / 4;   // row groups of 4 output rows
    static constexpr int NY = REM_VALU ? N : 4 * RG;            // outputs per pencil (>= N)
    static constexpr int SLOTS = N * RG;              // coefficient quadruples per table
    static constexpr int NTAB = (SLOTS + 15) / 16;    // A registers per table
    static constexpr size_t TAB_LDS_BYTES = (size_t)5 * NTAB * 64 * sizeof(float);
};

// Coefficient tables.  Slot s = l*RG + rg of a table sits in register s/16, lanes 4*(s%16) .. +3;
// lane r of the quadruple holds the coefficient of output row 4*rg + r and input index l:
// S[l][row] forward (transpose applied), S[row][l] backward.  mm_coef is the value of register t
// in lane `lane`.
template <int N>
__device__ __forceinline__ float mm_coef(const float *__restrict__ S, bool fwd, int t, int lane)
{
    using M = MmShape<N>;
    const int s = 16 * t + (lane >> 2);
    const int l = s / M::RG;
    const int row = 4 * (s - l * M::RG) + (lane & 3);
    const bool ok = (l < N) && (row < N);
    const int idx = ok ? (fwd ? l * N + row : row * N + l) : 0;
    const float c = S[idx];
    return ok ? c : 0.0f;
}
// The six tables in the order the kernel uses them: x, y, z forward, then z, y, x backward.
// Table 0 is loaded straight into registers by every wavefront; tables 1..5 are built once per
// workgroup (their 5*NTAB registers dealt round-robin to the wavefronts), parked in LDS as
// [table][register][lane] and fetched after the barrier that precedes their use.
template <int N, int NWAVES>
struct MmStage {
    static constexpr int ROWS = 5 * MmShape<N>::NTAB;
    static constexpr int PER_WAVE = (ROWS + NWAVES - 1) / NWAVES;
    // The loads of the rows this wavefront builds (issued together) ...
    static __device__ __forceinline__ void load(const float *__restrict__ Sx, const float *__restrict__ Sy,
                                                const float *__restrict__ Sz, int wave, int lane,
                                                float (&val)[PER_WAVE])
    {
#pragma unroll
        for (int k = 0; k < PER_WAVE; ++k) {
            int r = wave + k * NWAVES;
            if (r >= ROWS) r = ROWS - 1;                 // duplicate work instead of a branch
            const int tb = r / MmShape<N>::NTAB + 1;
            const int t = r - (tb - 1) * MmShape<N>::NTAB;
            const float *S = (tb == 1 || tb == 4) ? Sy : (tb == 5 ? Sx : Sz);
            val[k] = mm_coef<N>(S, tb <= 2, t, lane);
        }
    }
    // ... and their stores to LDS.
    static __device__ __forceinline__ void store(float *tabs, int wave, int lane,
                                                 const float (&val)[PER_WAVE])
    {
#pragma unroll
        for (int k = 0; k < PER_WAVE; ++k) {
            int r = wave + k * NWAVES;
            if (r >= ROWS) r = ROWS - 1;
            tabs[r * 64 + lane] = val[k];
        }
    }
};
template <int N>
__device__ __forceinline__ void mm_fetch_table(const float *tabs, int tb, int lane,
                                               float (&tab)[MmShape<N>::NTAB])
{
#pragma unroll
    for (int t = 0; t < MmShape<N>::NTAB; ++t) tab[t] = tabs[((tb - 1) * MmShape<N>::NTAB + t) * 64 + lane];
}

template <int N, int I>
__device__ __forceinline__ void mm_step(const float (&tab)[MmShape<N>::NTAB], const float (&x)[N],
                                        mm_f4 (&acc)[MmShape<N>::RG])
{
    constexpr int RG = MmShape<N>::RG;
    constexpr int L = I / RG, R = I % RG;
    if constexpr (L == 0) {
        const mm_f4 zero = {0.0f, 0.0f, 0.0f, 0.0f};
        acc[R] = __builtin_amdgcn_mfma_f32_4x4x1f32(tab[I / 16], x[L], zero, 4, I % 16, 0);
    } else {
        acc[R] = __builtin_amdgcn_mfma_f32_4x4x1f32(tab[I / 16], x[L], acc[R], 4, I % 16, 0);
    }
}
template <int N, int... I>
__device__ __forceinline__ void mm_steps(const float (&tab)[MmShape<N>::NTAB], const float (&x)[N],
                                         mm_f4 (&acc)[MmShape<N>::RG],
                                         std::integer_sequence<int, I...>)
{
    (mm_step<N, I>(tab, x, acc), ...);
}

// y[row] = sum_l coef(row, l) * x[l] for the lane's pencil; rows >= N of y (if any) are 0.
// S is the matrix itself, read through the constant address space for the left-over row.
template <int N, bool FWD>
__device__ __forceinline__ void mode_product_mm(const float (&tab)[MmShape<N>::NTAB],
                                                const TPO_CONSTANT float *S, const float (&x)[N],
                                                float (&y)[MmShape<N>::NY])
{
    using M = MmShape<N>;
    mm_f4 acc[M::RG];
    mm_steps<N>(tab, x, acc, std::make_integer_sequence<int, M::SLOTS>{});
#pragma unroll
    for (int i = 0; i < 4 * M::RG; ++i) y[i] = acc[i / 4][i % 4];
    if constexpr (M::REM_VALU) {
        asm volatile("" : "+s"(S));       // keep the scalar loads of this product to themselves
        constexpr int R = N - 1;
        float r = (FWD ? S[R] : S[R * N]) * x[0];
#pragma unroll
        for (int l = 1; l < N; ++l) r = fma_(FWD ? S[l * N + R] : S[R * N + l], x[l], r);
        y[R] = r;
    }
}

// HINT and XCD as in ihelm_pencil_kernel; D_e is always loaded in its pencil layout.
// The matrix instructions run outside the `on` branches, on whole wavefronts: the broadcast
// coefficient quadruples are read from ACTIVE lanes of the table register only, so a lane that
// is switched off would take its quadruples away from all the others.  Idle lanes compute on
// a shadow pencil or stale LDS words and never store.
// SEP as in ihelm_pencil_kernel: D_e evaluated from lam_x, lam_y, lam_z, mu instead of read
// (1: IEEE division, 2: hardware reciprocal, 1 ulp).
// Wavefronts per SIMD the register allocation must leave room for: up to n = 13 the kernel fits
// 64 registers (eight wavefronts); left to itself the scheduler spends a few more on addresses
// held across the prologue (71 at n = 13: seven wavefronts, 1 % slower).
template <int N> constexpr int mm_waves_per_simd() { return N <= 13 ? 8 : 1; }

template <int N, int G, int HINT, bool XCD, int SEP = 0>
__global__ void __launch_bounds__((PencilShape<float, N, G>::NT))
__attribute__((amdgpu_waves_per_eu(mm_waves_per_simd<N>())))
ihelm_pencil_mm_kernel(const float *u, const float *__restrict__ Sx, const float *__restrict__ Sy,
                       const float *__restrict__ Sz, const float *__restrict__ D, float *v,
                       long long num_elems, const float *__restrict__ lam_x,
                       const float *__restrict__ lam_y, const float *lam_z_,
                       const float *__restrict__ mu)
{
    using Sh = PencilShape<float, N, G>;
    using M = MmShape<N>;
    constexpr int P = Sh::P, PA = Sh::PA, PB = Sh::PB, CUBE = Sh::CUBE, NY = M::NY;
    extern __shared__ __align__(16) unsigned char tpo_lds[];
    float *cube_all = reinterpret_cast<float *>(tpo_lds);
    float *tabs = cube_all + G * CUBE;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const long long nbatch = (num_elems + G - 1) / G;
    const long long batch = pencil_batch<XCD>(nbatch);
    if (XCD && batch >= nbatch) return;
    const int g_ = tid / P;
    const bool on = (tid < G * P) && (batch * G + g_ < num_elems);
    // Lanes without a pencil (past the last pencil of the workgroup, or in element slots past
    // the end of the field) shadow pencil 0 of the batch's first element: they load what its
    // lane loads and compute what it computes, and never write.  No branch around the loads,
    // nothing to initialise for them.
    const int g = on ? g_ : 0;
    const int p = on ? tid - g_ * P : 0;
    const int hi = p / N;
    const int lo = p - hi * N;
    const long long e = batch * G + g;

    float *cube = cube_all + g * CUBE;
    // addresses: one base per workgroup (uniform) plus a 32-bit word offset per lane
    constexpr int N3 = N * N * N;
    const size_t wg_base = (size_t)(batch * G) * (size_t)N3;
    const char *ub = reinterpret_cast<const char *>(u + wg_base);
    char *vb = reinterpret_cast<char *>(v + wg_base);
    // Byte offset of word (l = MID, b, c) of the lane's element: the n accesses of a pencil along
    // axis 0 are then this one offset plus immediates (l - MID) * P * 4, all within the +-4 KB an
    // instruction can carry for n <= 13 (addressed from l = 0 the upper half needs a register
    // and an add each: 19 vector instructions and 14 registers more per wavefront at n = 13;
    // 5.44-5.46 against 5.51-5.53 ms on the n = 13 workload).  Opaque to the compiler so that it
    // keeps this split.
    constexpr int MID = N / 2;
    int off_bc = (g * N3 + p + MID * P) * 4;
    asm volatile("" : "+v"(off_bc));

    float x[N], y[NY], dd[N];
    float tab[M::NTAB];
    float sep_ab = 1.0f, sep_mu = 0.0f;   // lam_x[a] + lam_y[b] of the lane's axis-2 pencil, mu[e]

    // forward, axis 0: lane (b,c) = (hi,lo)
#pragma unroll
    for (int t = 0; t < M::NTAB; ++t) tab[t] = mm_coef<N>(Sx, true, t, lane);
#pragma unroll
    for (int l = 0; l < N; ++l)
        x[l] = gload<(HINT & 1) != 0>(reinterpret_cast<const float *>(ub + off_bc + (l - MID) * P * 4));
    if constexpr (SEP != 0) {
        sep_ab = lam_x[hi] + lam_y[lo];
        sep_mu = mu[e];
    } else {
        load_words<(HINT & 4) != 0>(D + wg_base + (unsigned)(g * N3 + p * N), dd);
    }
    {
        using Stage = MmStage<N, Sh::NT / 64>;
        const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // scalar: table choice per wavefront
        float val[Stage::PER_WAVE];
        Stage::load(Sx, Sy, Sz, wave, lane, val);
        Stage::store(tabs, wave, lane, val);
    }
    mode_product_mm<N, true>(tab, (const TPO_CONSTANT float *)Sx, x, y);
    if (on) {
#pragma unroll
        for (int i = 0; i < N; ++i) cube[i * PA + hi * PB + lo] = y[i];
    }
    __syncthreads();

    // forward, axis 1: lane (a,c) = (hi,lo)
    mm_fetch_table<N>(tabs, 1, lane, tab);
#pragma unroll
    for (int m = 0; m < N; ++m) x[m] = cube[hi * PA + m * PB + lo];
    mode_product_mm<N, true>(tab, (const TPO_CONSTANT float *)Sy, x, y);
    if (on) {
#pragma unroll
        for (int j = 0; j < N; ++j) cube[hi * PA + j * PB + lo] = y[j];
    }
    __syncthreads();

    // forward axis 2, diagonal scale, backward axis 2: lane (a,b) = (hi,lo)
    mm_fetch_table<N>(tabs, 2, lane, tab);
#pragma unroll
    for (int q = 0; q < N; ++q) x[q] = cube[hi * PA + lo * PB + q];
    mode_product_mm<N, true>(tab, (const TPO_CONSTANT float *)Sz, x, y);
    if constexpr (SEP != 0) {
        const TPO_CONSTANT float *lam_z = (const TPO_CONSTANT float *)lam_z_;
#pragma unroll
        for (int k = 0; k < N; ++k) dd[k] = recip_<SEP == 1>((sep_ab + lam_z[k]) + sep_mu);
    }
#pragma unroll
    for (int k = 0; k < N; ++k) x[k] = y[k] * dd[k];
    mm_fetch_table<N>(tabs, 3, lane, tab);
    mode_product_mm<N, false>(tab, (const TPO_CONSTANT float *)Sz, x, y);
    if (on) {
#pragma unroll
        for (int k = 0; k < N; ++k) cube[hi * PA + lo * PB + k] = y[k];
    }
    __syncthreads();

    // backward, axis 1: lane (a,c) = (hi,lo)
    mm_fetch_table<N>(tabs, 4, lane, tab);
#pragma unroll
    for (int m = 0; m < N; ++m) x[m] = cube[hi * PA + m * PB + lo];
    mode_product_mm<N, false>(tab, (const TPO_CONSTANT float *)Sy, x, y);
    if (on) {
#pragma unroll
        for (int j = 0; j < N; ++j) cube[hi * PA + j * PB + lo] = y[j];
    }
    __syncthreads();

    // backward, axis 0: lane (b,c) = (hi,lo)
    mm_fetch_table<N>(tabs, 5, lane, tab);
#pragma unroll
    for (int l = 0; l < N; ++l) x[l] = cube[l * PA + hi * PB + lo];
    mode_product_mm<N, false>(tab, (const TPO_CONSTANT float *)Sx, x, y);
    if (on) {
#pragma unroll
        for (int i = 0; i < N; ++i)
            gstore<(HINT & 2) != 0>(reinterpret_cast<float *>(vb + off_bc + (i - MID) * P * 4), y[i]);
    }
}

// Per n: elements per workgroup, hint bits and die renumbering: the best of the same sweep as
// for the vector-FMA pencil kernels; n = 13 at E = 1048576.  G = 0: the lane-utilisation rule.
struct PencilMmRow { int g, hint, xcd; };
constexpr PencilMmRow kPencilMmTable[TPO_MAX_N + 1] = {
    {0, 0, 0},
    {0, 0, 1}, {0, 0, 0}, {0, 0, 1}, {8, 2, 0}, {12, 0, 0}, {12, 0, 0}, {6, 0, 0}, {1, 3, 0},
    {6, 0, 0}, {3, 0, 1}, {2, 0, 0}, {3, 2, 0}, {3, 0, 0}, {2, 0, 0}, {1, 0, 1}, {1, 3, 0},
};
template <int N>
struct PencilMmTune {
    static constexpr int G = kPencilMmTable[N].g > 0 ? kPencilMmTable[N].g : pencil_group<float, N>();
    static constexpr int HINT = kPencilMmTable[N].hint;
    static constexpr bool XCD = kPencilMmTable[N].xcd != 0;
};
// Settings for large batches, used when num_elems > FROM (FROM < 0: never).  n = 13: with die
// renumbering the lines shared by neighbouring elements (8788 bytes each) stay in one L2; on the
// 1048576 elements of the named workload that is 5.33-5.35 against 5.38-5.39 ms (alternating
// libraries on one box), on 32768 elements it costs 1 % (172.4-173.3 against 170.6 us).
template <int N>
struct PencilMmLargeTune : PencilMmTune<N> {
    static constexpr long long FROM = -1;
};
template <> struct PencilMmLargeTune<13> : PencilMmTune<13> {
    static constexpr bool XCD = true;
    static constexpr long long FROM = 262144;
};

template <int N, typename Tune>
struct PencilMmLauncherT {
    static constexpr int G = Tune::G;
    using Sh = PencilShape<float, N, G>;
    static constexpr size_t LDS = Sh::LDS_BYTES / 2 + MmShape<N>::TAB_LDS_BYTES;

    template <bool SEP>
    static constexpr auto kernel()
    {
        return &ihelm_pencil_mm_kernel<N, G, Tune::HINT, Tune::XCD, SEP ? 2 : 0>;
    }

    template <bool SEP>
    static hipError_t launch_as(const ApplyArgs &a)
    {
        const long long blocks = pencil_grid<Tune::XCD>((a.num_elems + G - 1) / G);
        if (blocks <= 0 || blocks > 0x7fffffffLL) return kGridTooLarge;
        drop_stale_error();
        hipLaunchKernelGGL(kernel<SEP>(), dim3((unsigned)blocks), dim3(Sh::NT), LDS, a.stream,
                           (const float *)a.u, (const float *)a.sx, (const float *)a.sy,
                           (const float *)a.sz, (const float *)a.d, (float *)a.v, a.num_elems,
                           (const float *)a.lam_x, (const float *)a.lam_y,
                           (const float *)a.lam_z, (const float *)a.mu);
        return hipGetLastError();
    }

    static hipError_t prepare()
    {
        if (LDS <= 48 * 1024) return hipSuccess;
        hipError_t rc = hipFuncSetAttribute((const void *)kernel<false>(),
                                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS);
        if (rc != hipSuccess) return rc;
        return hipFuncSetAttribute((const void *)kernel<true>(),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS);
    }
};

template <int N>
struct PencilMmLauncher {
    using Plain = PencilMmLauncherT<N, PencilMmTune<N>>;
    using Large = PencilMmLauncherT<N, PencilMmLargeTune<N>>;
    static constexpr long long FROM = PencilMmLargeTune<N>::FROM;
    static bool large(const ApplyArgs &a) { return FROM >= 0 && a.num_elems > FROM; }
    static hipError_t launch(const ApplyArgs &a)
    {
        return large(a) ? Large::template launch_as<false>(a) : Plain::template launch_as<false>(a);
    }
    static hipError_t launch_sep(const ApplyArgs &a)
    {
        return large(a) ? Large::template launch_as<true>(a) : Plain::template launch_as<true>(a);
    }
    static hipError_t prepare()
    {
        const hipError_t rc = Plain::prepare();
        return rc != hipSuccess ? rc : Large::prepare();
    }
};

#define TPO_PENCIL_MM_ENTRY(N)                                                  \
    KernelEntry { &PencilMmLauncher<N>::launch, &PencilMmLauncher<N>::launch_sep, \
                  &PencilMmLauncher<N>::prepare }

}  // namespace tpo

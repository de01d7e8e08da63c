// Register-blocked vector-FMA kernel family ("pencil" kernels) for the batched
// inverse-Helmholtz tensor-product operator on gfx950.
//
// One lane owns one pencil: the n values of the cube along the axis being contracted, for
// fixed values of the other two indices.  A mode product is then n*n FMAs on registers:
// the lane's n inputs, n accumulators, and the n*n matrix entries, which are uniform over
// the wavefront and are read through the scalar data path (s_load + SGPR operand of
// v_fma), so they cost neither VGPRs nor LDS bandwidth.  Between axes the cube is
// re-distributed through LDS.  A workgroup processes G whole elements at a time (G*n*n
// pencils, padded to a multiple of 64 lanes); all six mode products and the diagonal scale
// run on chip, HBM sees u_e and D_e once (coalesced reads) and v_e once (coalesced store).
//
// Order of the six products (mode products along different axes commute):
//   forward axis 0 (from global, lanes consecutive along (b,c): coalesced)
//   forward axis 1, forward axis 2, scale by D_e, backward axis 2 (same registers),
//   backward axis 1, backward axis 0 (to global, coalesced).
// D_e either arrives in its axis-2 pencil layout (each lane loads the n consecutive words of
// its pencil) or coalesced like u_e and parked in LDS until the scale, or is evaluated in the
// kernel from its separable form; see the template parameters of ihelm_pencil_kernel.
#pragma once
#include <hip/hip_runtime.h>

#include "tpo_internal.h"

namespace tpo {

#define TPO_CONSTANT __attribute__((address_space(4)))

__device__ __forceinline__ double fma_(double a, double b, double c) { return __builtin_fma(a, b, c); }
__device__ __forceinline__ float fma_(float a, float b, float c) { return __builtin_fmaf(a, b, c); }

// 1/x for the separable diagonal.  EXACT: IEEE division.  Otherwise the hardware reciprocal,
// in fp64 followed by two Newton steps (v_rcp_f64 delivers about single precision): within
// 2 ulp for normal x, a third of the instructions of the IEEE sequence.
template <bool EXACT>
__device__ __forceinline__ double recip_(double x)
{
    if constexpr (EXACT) return 1.0 / x;
    double r = __builtin_amdgcn_rcp(x);
    double e = __builtin_fma(-x, r, 1.0);
    r = __builtin_fma(r, e, r);
    e = __builtin_fma(-x, r, 1.0);
    return __builtin_fma(r, e, r);
}
template <bool EXACT>
__device__ __forceinline__ float recip_(float x)
{
    if constexpr (EXACT) return 1.0f / x;
    return __builtin_amdgcn_rcpf(x);
}

template <typename T, int N, int G>
struct PencilShape {
    static constexpr int P = N * N;                         // pencils per element
    static constexpr int NT = ((G * P + 63) / 64) * 64;     // threads per workgroup
    // LDS pitches (in words): row pitch odd, plane pitch odd, so that the three access
    // patterns (lanes consecutive along c, along c with a in the high part, along b)
    // spread over the banks.
    static constexpr int PB = (N & 1) ? N : N + 1;
    static constexpr int PA = ((N * PB) & 1) ? N * PB : N * PB + 1;
    static constexpr int CUBE = N * PA;
    static constexpr size_t LDS_BYTES = (size_t)2 * G * CUBE * sizeof(T);
};

// Number of elements per workgroup: the G (1..64) with the best lane utilisation among
// those with at most 512 threads and at most ~53 KB of LDS (three workgroups per CU);
// G = 1 if nothing fits.
template <typename T, int N>
constexpr int pencil_group()
{
    int best = 1;
    long best_num = 0, best_den = 1;  // utilisation = num/den
    for (int g = 1; g <= 64; ++g) {
        const int p = g * N * N;
        const int nt = ((p + 63) / 64) * 64;
        const int pb = (N & 1) ? N : N + 1;
        const int pa = ((N * pb) & 1) ? N * pb : N * pb + 1;
        const long lds = 2L * g * N * pa * (long)sizeof(T);
        if (nt > 512 || lds > 53 * 1024) break;
        if ((long)p * best_den > best_num * nt) {
            best = g;
            best_num = p;
            best_den = nt;
        }
    }
    return best;
}

// y[i] = sum_l S[l][i] * x[l]   (FWD: the transpose of the stored matrix is applied)
// y[i] = sum_l S[i][l] * x[l]   (!FWD)
// S is read through the constant address space so that its entries arrive in SGPRs.
template <typename T, int N, bool FWD>
__device__ __forceinline__ void mode_product(const TPO_CONSTANT T *S, const T (&x)[N],
                                             T (&y)[N])
{
    // Make the pointer opaque per product: otherwise two products with the same matrix share
    // one set of scalar loads, all n*n entries stay live across both and spill out of the
    // SGPR file.
    asm volatile("" : "+s"(S));
    if constexpr (FWD) {
#pragma unroll
        for (int i = 0; i < N; ++i) y[i] = S[i] * x[0];
#pragma unroll
        for (int l = 1; l < N; ++l) {
#pragma unroll
            for (int i = 0; i < N; ++i) y[i] = fma_(S[l * N + i], x[l], y[i]);
        }
    } else {
#pragma unroll
        for (int i = 0; i < N; ++i) {
            T acc = S[i * N] * x[0];
#pragma unroll
            for (int l = 1; l < N; ++l) acc = fma_(S[i * N + l], x[l], acc);
            y[i] = acc;
        }
    }
}

// Global accesses with or without the non-temporal hint (streamed once, never re-read).
template <bool NT, typename T>
__device__ __forceinline__ T gload(const T *p)
{
    if constexpr (NT) return __builtin_nontemporal_load(p);
    else return *p;
}
template <bool NT, typename T>
__device__ __forceinline__ void gstore(T *p, T x)
{
    if constexpr (NT) __builtin_nontemporal_store(x, p);
    else *p = x;
}

// K consecutive words of type T from/to global memory at word alignment, as the widest
// accesses the hardware takes at that alignment (vectors of 2 and 4 words declared with the
// alignment of one word become dwordx2 / dwordx4 instructions).
template <typename T, int W> struct WordVec {
    typedef T type __attribute__((ext_vector_type(W), aligned(sizeof(T))));
};
template <bool NT, typename T, int K>
__device__ __forceinline__ void load_words(const T *p, T (&out)[K])
{
    typedef typename WordVec<T, 4>::type v4;
    typedef typename WordVec<T, 2>::type v2;
    int q = 0;
#pragma unroll
    for (; q + 4 <= K; q += 4) {
        const v4 *pv = reinterpret_cast<const v4 *>(p + q);
        v4 t;
        if constexpr (NT) t = __builtin_nontemporal_load(pv); else t = *pv;
        out[q] = t[0]; out[q + 1] = t[1]; out[q + 2] = t[2]; out[q + 3] = t[3];
    }
    if (q + 2 <= K) {
        const v2 *pv = reinterpret_cast<const v2 *>(p + q);
        v2 t;
        if constexpr (NT) t = __builtin_nontemporal_load(pv); else t = *pv;
        out[q] = t[0]; out[q + 1] = t[1];
        q += 2;
    }
    if (q < K) out[q] = gload<NT>(p + q);
}
template <bool NT, typename T, int K>
__device__ __forceinline__ void store_words(T *p, const T (&in)[K])
{
    typedef typename WordVec<T, 4>::type v4;
    typedef typename WordVec<T, 2>::type v2;
    int q = 0;
#pragma unroll
    for (; q + 4 <= K; q += 4) {
        v4 t = {in[q], in[q + 1], in[q + 2], in[q + 3]};
        v4 *pv = reinterpret_cast<v4 *>(p + q);
        if constexpr (NT) __builtin_nontemporal_store(t, pv); else *pv = t;
    }
    if (q + 2 <= K) {
        v2 t = {in[q], in[q + 1]};
        v2 *pv = reinterpret_cast<v2 *>(p + q);
        if constexpr (NT) __builtin_nontemporal_store(t, pv); else *pv = t;
        q += 2;
    }
    if (q < K) gstore<NT>(p + q, in[q]);
}

// HINT bit 0: non-temporal coalesced loads (u, and D_e when it is loaded coalesced); bit 1:
// non-temporal stores of v; bit 2: non-temporal loads of D_e's per-lane runs (DDIRECT).
// DDIRECT = false: D_e is loaded coalesced with u_e and parked in LDS until the scale.
// DDIRECT = true : every lane loads, at kernel start, the n consecutive words of D_e that
//                  belong to its axis-2 pencil (no LDS for D_e: half the LDS per workgroup).
// XCD = true : workgroups are renumbered so that each of the 8 accelerator dies (workgroups
//              are dealt to them round-robin) works on one contiguous eighth of the elements;
//              cache lines shared by neighbouring elements then stay within one L2.
//              The grid must be pencil_grid<XCD>(number of batches).
template <bool XCD>
__host__ __device__ inline long long pencil_grid(long long nbatch)
{
    return XCD ? 8 * ((nbatch + 7) / 8) : nbatch;
}
template <bool XCD>
__device__ __forceinline__ long long pencil_batch(long long nbatch)
{
    if constexpr (XCD) {
        const long long per = (nbatch + 7) / 8;
        return (long long)(blockIdx.x & 7) * per + (long long)(blockIdx.x >> 3);
    } else {
        return blockIdx.x;
    }
}

// SEP != 0 : D_e is not read; it is evaluated where it is used from the separable form
//            D_e[a][b][c] = 1 / (lam_x[a] + lam_y[b] + lam_z[c] + mu[e])
//            (sum left to right; SEP = 1: IEEE division, SEP = 2: recip_<false>); D is ignored
//            and may be null.
template <typename T, int N, int G, int HINT, bool DDIRECT = false, bool XCD = false,
          int SEP = 0>
__global__ void __launch_bounds__((PencilShape<T, N, G>::NT))
ihelm_pencil_kernel(const T *u, const T *Sx_, const T *Sy_, const T *Sz_,
                    const T *__restrict__ D, T *v, long long num_elems,
                    const T *__restrict__ lam_x, const T *__restrict__ lam_y,
                    const T *lam_z_, const T *__restrict__ mu)
{
    using Sh = PencilShape<T, N, G>;
    constexpr int P = Sh::P, PA = Sh::PA, PB = Sh::PB, CUBE = Sh::CUBE;
    extern __shared__ __align__(16) unsigned char tpo_lds[];
    T *cube_all = reinterpret_cast<T *>(tpo_lds);
    T *dpark_all = cube_all + G * CUBE;

    const TPO_CONSTANT T *Sx = (const TPO_CONSTANT T *)Sx_;
    const TPO_CONSTANT T *Sy = (const TPO_CONSTANT T *)Sy_;
    const TPO_CONSTANT T *Sz = (const TPO_CONSTANT T *)Sz_;

    const int tid = threadIdx.x;
    const int g = tid / P;          // element slot inside the workgroup
    const int p = tid - g * P;      // pencil id inside the element
    const int hi = p / N;
    const int lo = p - hi * N;
    const long long nbatch = (num_elems + G - 1) / G;
    const long long batch = pencil_batch<XCD>(nbatch);
    if (XCD && batch >= nbatch) return;                 // whole workgroup: no barrier is skipped
    const long long e = batch * G + g;
    const bool on = (tid < G * P) && (e < num_elems);

    T *cube = cube_all + (g < G ? g : 0) * CUBE;
    T *dpark = dpark_all + (g < G ? g : 0) * CUBE;
    const size_t base = (size_t)(on ? e : 0) * (size_t)(N * N * N);

    T x[N], y[N];

    // forward, axis 0: lane (b,c) = (hi,lo); global reads are consecutive over lanes
    T dd[N];
    T sep_ab = T(0), sep_mu = T(0);     // lam_x[a] + lam_y[b] of the lane's axis-2 pencil, mu[e]
    if (on) {
#pragma unroll
        for (int l = 0; l < N; ++l) x[l] = gload<(HINT & 1) != 0>(u + base + (size_t)(l * P + p));
        if constexpr (SEP != 0) {
            sep_ab = lam_x[hi] + lam_y[lo];
            sep_mu = mu[e];
        } else if constexpr (DDIRECT) {
            load_words<(HINT & 4) != 0>(D + base + (size_t)(p * N), dd);   // D_e[a][b][0..n-1]
        } else {
#pragma unroll
            for (int l = 0; l < N; ++l) dd[l] = gload<(HINT & 1) != 0>(D + base + (size_t)(l * P + p));
        }
        mode_product<T, N, true>(Sx, x, y);
#pragma unroll
        for (int i = 0; i < N; ++i) cube[i * PA + hi * PB + lo] = y[i];
        if constexpr (!DDIRECT && SEP == 0) {
#pragma unroll
            for (int l = 0; l < N; ++l) dpark[l * PA + hi * PB + lo] = dd[l];
        }
    }
    __syncthreads();

    // forward, axis 1: lane (a,c) = (hi,lo)
    if (on) {
#pragma unroll
        for (int m = 0; m < N; ++m) x[m] = cube[hi * PA + m * PB + lo];
        mode_product<T, N, true>(Sy, x, y);
#pragma unroll
        for (int j = 0; j < N; ++j) cube[hi * PA + j * PB + lo] = y[j];
    }
    __syncthreads();

    // forward axis 2, diagonal scale, backward axis 2: lane (a,b) = (hi,lo)
    if (on) {
#pragma unroll
        for (int q = 0; q < N; ++q) x[q] = cube[hi * PA + lo * PB + q];
        if constexpr (SEP != 0) {
            const TPO_CONSTANT T *lam_z = (const TPO_CONSTANT T *)lam_z_;
#pragma unroll
            for (int k = 0; k < N; ++k) dd[k] = recip_<SEP == 1>((sep_ab + lam_z[k]) + sep_mu);
        }
        mode_product<T, N, true>(Sz, x, y);
#pragma unroll
        for (int k = 0; k < N; ++k) y[k] *= (DDIRECT || SEP != 0) ? dd[k] : dpark[hi * PA + lo * PB + k];
        mode_product<T, N, false>(Sz, y, x);
#pragma unroll
        for (int k = 0; k < N; ++k) cube[hi * PA + lo * PB + k] = x[k];
    }
    __syncthreads();

    // backward, axis 1: lane (a,c) = (hi,lo)
    if (on) {
#pragma unroll
        for (int m = 0; m < N; ++m) x[m] = cube[hi * PA + m * PB + lo];
        mode_product<T, N, false>(Sy, x, y);
#pragma unroll
        for (int j = 0; j < N; ++j) cube[hi * PA + j * PB + lo] = y[j];
    }
    __syncthreads();

    // backward, axis 0: lane (b,c) = (hi,lo); global stores are consecutive over lanes
    if (on) {
#pragma unroll
        for (int l = 0; l < N; ++l) x[l] = cube[l * PA + hi * PB + lo];
        mode_product<T, N, false>(Sx, x, y);
#pragma unroll
        for (int i = 0; i < N; ++i) gstore<(HINT & 2) != 0>(v + base + (size_t)(i * P + p), y[i]);
    }
}

// Per (type, n): elements per workgroup G, hint bits, how D_e is brought in (1: straight into
// its pencil layout, half the LDS; 0: coalesced and parked in LDS), and whether the workgroups
// are renumbered per accelerator die.  One row per n = 1..16: the best of a sweep on MI355X over
// G in {1,2,3,4,6,8,12,16,32} x hint bits x D mode x renumbering on 1 GiB fields; n = 8, 11
// (fp64) and 13 (fp32) are the sweeps at the sizes of the named workloads, re-checked on the
// named workloads' own data (n = 8: D_e in per-lane runs 0.2501-0.2506 ms against 0.2523-0.2550
// parked in LDS, at 4 elements per workgroup with non-temporal accesses).  n = 1 keeps the
// lane-utilisation rule (G = 0 in the table).
struct PencilRow { int g, hint, ddirect, xcd; };
template <typename T> struct PencilTable;
template <> struct PencilTable<double> {
    static constexpr PencilRow row[TPO_MAX_N + 1] = {
        {0, 2, 1, 0},
        {0, 2, 1, 1},  {16, 0, 1, 0}, {32, 0, 1, 0}, {4, 3, 0, 0},  {16, 0, 1, 0}, {1, 3, 1, 0},
        {1, 3, 1, 0},  {4, 3, 1, 0},  {3, 1, 1, 0},  {1, 3, 1, 0},  {1, 0, 1, 1},  {3, 3, 1, 0},
        {3, 0, 1, 0},  {1, 0, 1, 0},  {1, 0, 1, 0},  {1, 3, 1, 1},
    };
};
template <> struct PencilTable<float> {
    static constexpr PencilRow row[TPO_MAX_N + 1] = {
        {0, 2, 1, 0},
        {0, 2, 1, 1},  {16, 0, 1, 0}, {32, 0, 1, 0}, {8, 2, 1, 0},  {16, 0, 1, 0}, {12, 0, 1, 0},
        {1, 3, 1, 1},  {2, 3, 1, 0},  {3, 0, 1, 0},  {2, 0, 1, 0},  {2, 0, 1, 0},  {3, 2, 1, 0},
        {3, 0, 1, 0},  {2, 0, 1, 0},  {2, 0, 1, 0},  {1, 3, 1, 0},
    };
};
template <typename T, int N>
struct PencilTune {
    static constexpr PencilRow R = PencilTable<T>::row[N];
    static constexpr int G = R.g > 0 ? R.g : pencil_group<T, N>();
    static constexpr int HINT = R.hint;
    static constexpr bool DDIRECT = R.ddirect != 0;
    static constexpr bool XCD = R.xcd != 0;
    static constexpr size_t LDS_MIN = 0;    // LDS requested at least (caps workgroups per CU)
};
// n = 11: two elements per workgroup (242 of 256 lanes), non-temporal loads of u_e, and an LDS
// request of 28 KB (20.8 KB are used), which holds the CU at 5 workgroups = 10 elements instead
// of 7: with fewer loads in flight the memory system runs faster.  Chosen on the named workload
// (E = 262144, full-mantissa values; the settings rank differently on low-entropy data, where
// the clock runs higher), alternating libraries on one box, ms per launch: this setting 1.421-
// 1.424; the same with cached u_e loads 1.450-1.452; 26 KB / 30 KB requests 1.465 / 1.421-1.430;
// one element per workgroup with 18 KB (the earlier choice) 1.441-1.462, with 14 KB 1.469;
// three / four elements per workgroup 1.518 / 1.472.
template <> struct PencilTune<double, 11> {
    static constexpr int G = 2, HINT = 1;
    static constexpr bool DDIRECT = true, XCD = true;
    static constexpr size_t LDS_MIN = 28 * 1024;
};

// Settings for small batches, used when LO < num_elems <= HI (HI = 0: never).  With a few
// thousand workgroups the launch is a handful of rounds of resident workgroups: how the rounds
// divide the batch and how fast a round drains count for more than the steady-state memory
// behaviour the large-batch settings were chosen for.  From sweeps over E = 2048 .. 131072 on
// MI355X (the batch of 8192 elements per call is the one the paper times, Sec. 6.1):
//  * n = 11: up to 6144 elements one element per workgroup without die renumbering and occupancy
//    cap is ahead (us per launch, against the large-batch settings: E = 1024 10.9 / 11.3, 4096
//    27.0 / 29.0, 6144 38.4 / 38.4); beyond, the two leapfrog with the number of rounds of
//    resident workgroups (8192 49.2 / 47.2, 12288 74.0 / 67.0, 16384 97.8 / 99.7, 24576 142.3 /
//    142.3, 49152 277 / 281, 65536 368.5 / 367.1) and the large-batch settings are kept;
//  * n = 9 (fp64): three elements per workgroup; non-temporal u_e loads pay from about 30000
//    elements on (us per launch with / without them: E = 2048 11.6 / 11.1, 8192 28.3 / 27.2, 32768
//    99.4 / 102.6, 184000 547 / 580; two elements per workgroup with cached loads, the earlier
//    choice: 11.0, 28.5, 104.0, 569), so they are left out up to 16384 elements;
//  * n = 8: between 4096 and 24576 elements one element per workgroup with cached accesses and
//    D_e in its pencil layout beats four per workgroup (8192: 19.5 against 20.5 us, 16384: 33.2
//    against 35.9); at 4096 and from 32768 on the large-batch settings win.
template <typename T, int N>
struct PencilSmallTune : PencilTune<T, N> {
    static constexpr long long LO = 0, HI = 0;
};
template <> struct PencilSmallTune<double, 11> : PencilTune<double, 11> {
    static constexpr int G = 1, HINT = 0;
    static constexpr bool XCD = false;
    static constexpr size_t LDS_MIN = 0;
    static constexpr long long LO = 0, HI = 6144;
};
template <> struct PencilSmallTune<double, 9> : PencilTune<double, 9> {
    static constexpr int HINT = 0;
    static constexpr long long LO = 0, HI = 16384;
};
template <> struct PencilSmallTune<double, 8> : PencilTune<double, 8> {
    static constexpr int G = 1, HINT = 0;
    static constexpr bool DDIRECT = true;
    static constexpr long long LO = 4096, HI = 24576;
};

// Tuning of the separable-diagonal form: as the D form unless measured otherwise.  Without the
// D_e stream a workgroup has half the loads in flight, so the D form's occupancy cap at n = 11
// and its four elements per workgroup at n = 8 no longer pay (n = 11: 1.27 against 1.35 ms;
// n = 8: 0.202 against 0.215 ms).
template <typename T, int N>
struct PencilSepTune : PencilTune<T, N> {};
template <> struct PencilSepTune<double, 11> : PencilTune<double, 11> {
    static constexpr int G = 1, HINT = 0;
    static constexpr size_t LDS_MIN = 0;
};
template <> struct PencilSepTune<double, 8> : PencilTune<double, 8> {
    static constexpr int G = 1;
};
template <> struct PencilSepTune<double, 9> : PencilTune<double, 9> {
    static constexpr int G = 2, HINT = 0;       // (the D form's retuning at n = 9 was not repeated here)
};

// SEP: 0 = D read from memory, 1 / 2 = separable diagonal (IEEE division / fast reciprocal).
template <typename T, int N, typename Tune, int SEP>
struct PencilLauncherT {
    static constexpr int G = Tune::G;
    using Sh = PencilShape<T, N, G>;
    static constexpr bool DDIRECT = Tune::DDIRECT || SEP != 0;   // no D_e in LDS either way
    static constexpr size_t LDS_USED = DDIRECT ? Sh::LDS_BYTES / 2 : Sh::LDS_BYTES;
    static constexpr size_t LDS = LDS_USED > Tune::LDS_MIN ? LDS_USED : Tune::LDS_MIN;

    static constexpr auto kernel()
    {
        return &ihelm_pencil_kernel<T, N, G, Tune::HINT, DDIRECT, Tune::XCD, SEP>;
    }

    static hipError_t launch(const ApplyArgs &a)
    {
        const long long blocks = pencil_grid<Tune::XCD>((a.num_elems + G - 1) / G);
        if (blocks <= 0 || blocks > 0x7fffffffLL) return kGridTooLarge;
        drop_stale_error();
        hipLaunchKernelGGL(kernel(), dim3((unsigned)blocks), dim3(Sh::NT), LDS, a.stream,
                           (const T *)a.u, (const T *)a.sx, (const T *)a.sy, (const T *)a.sz,
                           (const T *)a.d, (T *)a.v, a.num_elems, (const T *)a.lam_x,
                           (const T *)a.lam_y, (const T *)a.lam_z, (const T *)a.mu);
        return hipGetLastError();
    }

    static hipError_t prepare()
    {
        if (LDS <= 48 * 1024) return hipSuccess;
        return hipFuncSetAttribute((const void *)kernel(),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)LDS);
    }
};

template <typename T, int N>
struct PencilLauncher {
    using Plain = PencilLauncherT<T, N, PencilTune<T, N>, 0>;
    using Small = PencilLauncherT<T, N, PencilSmallTune<T, N>, 0>;
    using Sep = PencilLauncherT<T, N, PencilSepTune<T, N>, 2>;   // fast reciprocal
    static hipError_t launch(const ApplyArgs &a)
    {
        using St = PencilSmallTune<T, N>;
        if (a.num_elems > St::LO && a.num_elems <= St::HI) return Small::launch(a);
        return Plain::launch(a);
    }
    static hipError_t launch_sep(const ApplyArgs &a) { return Sep::launch(a); }
    static hipError_t prepare()
    {
        hipError_t rc = Plain::prepare();
        if (rc == hipSuccess) rc = Small::prepare();
        return rc != hipSuccess ? rc : Sep::prepare();
    }
};

#define TPO_PENCIL_ENTRY(T, N)                                                        \
    KernelEntry { &PencilLauncher<T, N>::launch, &PencilLauncher<T, N>::launch_sep, \
                  &PencilLauncher<T, N>::prepare }

}  // namespace tpo

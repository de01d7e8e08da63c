// Matrix-core kernel family for the batched inverse-Helmholtz tensor-product operator on
// gfx950 (v_mfma_f64_16x16x4_f64 / v_mfma_f32_16x16x4_f32).
//
// A mode product along one axis of the cube is the matrix product
//     Out[i, X] = sum_l Mat[i, l] * In[l, X],      X = the other two indices, flattened,
// with Mat = S^T (forward) or S (backward).  It is cut into 16-column tiles of X; one tile
// is  D(16x16) = sum over k-steps of  A(16x4) * B(4x16)  with
//     A = Mat[:, 4 values of l]   (the same for every tile: held in registers for the whole
//                                  kernel, zero beyond n),
//     B = In[4 values of l, 16 columns]   (one word per lane per k-step, read from LDS).
// The accumulator leaves lane (x, g) holding Out[row(r,g), X0+x], r = 0..3, with
// row(r,g) = 4r+g for f64 and 4g+r for f32.  A tile overwrites its own columns in LDS, so a
// mode product needs no second buffer, and nothing between the first load of u_e and the
// store of v_e touches HBM.
//
// Order: forward axis 0 (B read straight from HBM: lanes run along X, so rows of 16 words
// are contiguous), forward axis 1, forward axis 2, scale by D_e, backward axis 2, backward
// axis 1, backward axis 0 (accumulators stored straight to HBM).  After forward axis 2 the
// accumulator rows are exactly the l-values a k-step needs when the contraction index is
// numbered row(s,g), so the scaled accumulators are fed back as B operands of backward
// axis 2 without leaving registers.  D_e is copied to LDS (coalesced) while forward axis 0
// runs and is read from there in accumulator layout.
//
// A workgroup of NW wavefronts handles G elements; the G*ceil(n*n/16) tiles of a mode
// product are dealt round-robin to the wavefronts, with a barrier between mode products.
#pragma once
#include <hip/hip_runtime.h>

#include "tpo_internal.h"
#include "tpo_pencil.hpp"   // PencilShape pitches, gload/gstore, lds_index

namespace tpo {

template <typename T> struct Mfma;
template <> struct Mfma<double> {
    typedef double acc_t __attribute__((ext_vector_type(4)));
    static __device__ __forceinline__ acc_t mma(double a, double b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int row(int r, int g) { return 4 * r + g; }
};
template <> struct Mfma<float> {
    typedef float acc_t __attribute__((ext_vector_type(4)));
    static __device__ __forceinline__ acc_t mma(float a, float b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ int row(int r, int g) { return 4 * g + r; }
};

template <typename T, int N, int G, int NW>
struct MfmaShape {
    using Pitch = PencilShape<T, N, G>;
    static constexpr int P2 = N * N;
    static constexpr int N3 = N * N * N;
    static constexpr int TILES = (P2 + 15) / 16;            // column tiles per element
    static constexpr int TT = G * TILES;                    // tiles per workgroup
    static constexpr int TPW = (TT + NW - 1) / NW;          // tiles per wavefront
    static constexpr int KS = (N + 3) / 4;                  // k-steps, l = 4s+g
    // k-steps of the register-fed backward product, l = row(s,g)
    static constexpr int KSF = (sizeof(T) == 8) ? KS : (N < 4 ? N : 4);
    static constexpr int NT = 64 * NW;
    static constexpr int PA = Pitch::PA, PB = Pitch::PB, CUBE = Pitch::CUBE;
    static constexpr size_t LDS_BYTES = (size_t)2 * G * CUBE * sizeof(T);
};

template <typename T, int N, int G, int NW, int HINT>
__global__ void __launch_bounds__((MfmaShape<T, N, G, NW>::NT))
ihelm_mfma_kernel(const T *u, const T *__restrict__ Sx, const T *__restrict__ Sy,
                  const T *__restrict__ Sz, const T *__restrict__ D, T *v,
                  long long num_elems)
{
    using Sh = MfmaShape<T, N, G, NW>;
    using M = Mfma<T>;
    using acc_t = typename M::acc_t;
    constexpr int P2 = Sh::P2, N3 = Sh::N3, TILES = Sh::TILES, TT = Sh::TT, TPW = Sh::TPW;
    constexpr int KS = Sh::KS, KSF = Sh::KSF, NT = Sh::NT;
    constexpr int PA = Sh::PA, PB = Sh::PB, CUBE = Sh::CUBE;
    constexpr bool LD_NT = (HINT & 1) != 0, ST_NT = (HINT & 2) != 0;

    extern __shared__ __align__(16) unsigned char tpo_lds[];
    T *cube = reinterpret_cast<T *>(tpo_lds);
    T *dpark = cube + G * CUBE;

    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const int lane = tid & 63;
    const int x = lane & 15;       // column inside a tile; row of the A operand
    const int g = lane >> 4;       // k index inside a k-step
    const long long e0 = (long long)blockIdx.x * G;
    const long long left = num_elems - e0;
    const int nel = left < G ? (int)left : G;
    const size_t base = (size_t)e0 * N3;

    // ---- A operands: the six matrices, zero-padded to 16 x 4*KS, one word per k-step ------
    T a_fwd[3][KS], a_bwd[3][KS], a_bz[KSF];
    {
        const T *S[3] = {Sx, Sy, Sz};
#pragma unroll
        for (int d = 0; d < 3; ++d) {
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                const int l = 4 * s + g;
                const bool ok = (x < N) && (l < N);
                const int xs = ok ? x : 0, ls = ok ? l : 0;
                const T f = S[d][ls * N + xs];      // forward: Mat[i][l] = S[l][i]
                const T b = S[d][xs * N + ls];      // backward: Mat[i][l] = S[i][l]
                a_fwd[d][s] = ok ? f : T(0);
                a_bwd[d][s] = ok ? b : T(0);
            }
        }
#pragma unroll
        for (int s = 0; s < KSF; ++s) {
            const int l = M::row(s, g);
            const bool ok = (x < N) && (l < N);
            const T b = Sz[(ok ? x : 0) * N + (ok ? l : 0)];
            a_bz[s] = ok ? b : T(0);
        }
    }

    // ---- per-tile column data --------------------------------------------------------------
    int b0[TPW], b1[TPW], b2[TPW];     // LDS offsets of (row 0, column X) for the three axes
    bool colok[TPW];
    size_t gcol[TPW];                  // word offset of (row 0, column X) in u / v
#pragma unroll
    for (int j = 0; j < TPW; ++j) {
        const int tt = wave + NW * j;
        int ge = tt / TILES;
        const int t = tt - ge * TILES;
        int X = 16 * t + x;
        colok[j] = (tt < TT) && (X < P2) && (ge < nel);
        if (!colok[j]) { ge = 0; X = 0; }
        const int hi = X / N, lo = X - hi * N;
        b0[j] = ge * CUBE + hi * PB + lo;
        b1[j] = ge * CUBE + hi * PA + lo;
        b2[j] = ge * CUBE + hi * PA + lo * PB;
        gcol[j] = base + (size_t)ge * N3 + (size_t)X;
    }

    // ---- D_e: HBM -> registers now, -> LDS after forward axis 0 has been issued -----------
    constexpr int DIT = (G * N3 + NT - 1) / NT;
    T dreg[DIT];
#pragma unroll
    for (int k = 0; k < DIT; ++k) {
        const int w = tid + k * NT;
        dreg[k] = (w < nel * N3) ? gload<LD_NT>(D + base + w) : T(0);
    }

    // ---- forward axis 0: B from HBM, result to LDS ----------------------------------------
#pragma unroll
    for (int j = 0; j < TPW; ++j) {
        T bv[KS];
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const int l = 4 * s + g;
            const bool ok = colok[j] && (l < N);
            bv[s] = ok ? gload<LD_NT>(u + gcol[j] + (size_t)((ok ? l : 0) * P2)) : T(0);
        }
        acc_t acc = {0, 0, 0, 0};
#pragma unroll
        for (int s = 0; s < KS; ++s) acc = M::mma(a_fwd[0][s], bv[s], acc);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int i = M::row(r, g);
            if (i < N && colok[j]) cube[b0[j] + i * PA] = acc[r];
        }
    }
#pragma unroll
    for (int k = 0; k < DIT; ++k) {
        const int w = tid + k * NT;
        if (w < G * N3) dpark[lds_index<T, N, G>(w)] = dreg[k];
    }
    __syncthreads();

    // ---- forward axis 1: LDS -> LDS -----------------------------------------------------------
#pragma unroll
    for (int j = 0; j < TPW; ++j) {
        T bv[KS];
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const int l = 4 * s + g;
            bv[s] = (l < N) ? cube[b1[j] + (l < N ? l : 0) * PB] : T(0);
        }
        acc_t acc = {0, 0, 0, 0};
#pragma unroll
        for (int s = 0; s < KS; ++s) acc = M::mma(a_fwd[1][s], bv[s], acc);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int i = M::row(r, g);
            if (i < N && colok[j]) cube[b1[j] + i * PB] = acc[r];
        }
    }
    __syncthreads();

    // ---- forward axis 2, scale by D_e, backward axis 2 (register to register) ---------------
#pragma unroll
    for (int j = 0; j < TPW; ++j) {
        T bv[KS];
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const int l = 4 * s + g;
            bv[s] = (l < N) ? cube[b2[j] + (l < N ? l : 0)] : T(0);
        }
        acc_t acc = {0, 0, 0, 0};
#pragma unroll
        for (int s = 0; s < KS; ++s) acc = M::mma(a_fwd[2][s], bv[s], acc);
        T gv[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int i = M::row(r, g);
            const T dval = (i < N) ? dpark[b2[j] + (i < N ? i : 0)] : T(0);
            gv[r] = acc[r] * dval;      // rows >= n are zero on both sides
        }
        acc_t acc2 = {0, 0, 0, 0};
#pragma unroll
        for (int s = 0; s < KSF; ++s) acc2 = M::mma(a_bz[s], gv[s], acc2);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int i = M::row(r, g);
            if (i < N && colok[j]) cube[b2[j] + i] = acc2[r];
        }
    }
    __syncthreads();

    // ---- backward axis 1: LDS -> LDS ----------------------------------------------------------
#pragma unroll
    for (int j = 0; j < TPW; ++j) {
        T bv[KS];
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const int l = 4 * s + g;
            bv[s] = (l < N) ? cube[b1[j] + (l < N ? l : 0) * PB] : T(0);
        }
        acc_t acc = {0, 0, 0, 0};
#pragma unroll
        for (int s = 0; s < KS; ++s) acc = M::mma(a_bwd[1][s], bv[s], acc);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int i = M::row(r, g);
            if (i < N && colok[j]) cube[b1[j] + i * PB] = acc[r];
        }
    }
    __syncthreads();

    // ---- backward axis 0: LDS -> HBM ------------------------------------------------------------
#pragma unroll
    for (int j = 0; j < TPW; ++j) {
        T bv[KS];
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const int l = 4 * s + g;
            bv[s] = (l < N) ? cube[b0[j] + (l < N ? l : 0) * PA] : T(0);
        }
        acc_t acc = {0, 0, 0, 0};
#pragma unroll
        for (int s = 0; s < KS; ++s) acc = M::mma(a_bwd[0][s], bv[s], acc);
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int i = M::row(r, g);
            if (i < N && colok[j]) gstore<ST_NT>(v + gcol[j] + (size_t)(i * P2), acc[r]);
        }
    }
}

template <typename T, int N, int G, int NW, int HINT>
struct MfmaLauncher {
    using Sh = MfmaShape<T, N, G, NW>;

    static hipError_t launch(const ApplyArgs &a)
    {
        const long long blocks = (a.num_elems + G - 1) / G;
        if (blocks <= 0 || blocks > 0x7fffffffLL) return hipErrorInvalidValue;
        hipLaunchKernelGGL((ihelm_mfma_kernel<T, N, G, NW, HINT>), dim3((unsigned)blocks),
                           dim3(Sh::NT), Sh::LDS_BYTES, a.stream, (const T *)a.u,
                           (const T *)a.sx, (const T *)a.sy, (const T *)a.sz,
                           (const T *)a.d, (T *)a.v, a.num_elems);
        return hipGetLastError();
    }

    static hipError_t prepare()
    {
        if (Sh::LDS_BYTES <= 48 * 1024) return hipSuccess;
        return hipFuncSetAttribute((const void *)ihelm_mfma_kernel<T, N, G, NW, HINT>,
                                   hipFuncAttributeMaxDynamicSharedMemorySize,
                                   (int)Sh::LDS_BYTES);
    }
};

}  // namespace tpo

// Matrix-core kernel family for the batched inverse-Helmholtz tensor-product operator on
// gfx950 (v_mfma_f64_16x16x4_f64 / v_mfma_f32_16x16x4_f32).
//
// A mode product along one axis of the cube is the matrix product
//     Out[i, X] = sum_l Mat[i, l] * In[l, X],      X = the other two indices, flattened,
// with Mat = S^T (forward) or S (backward).  It is cut into 16-column tiles of X; one tile
// is  D(16x16) = sum over KS = ceil(n/4) k-steps of  A(16x4) * B(4x16)  with
//     A = Mat rows x 4 values of l   (the same for every tile: held in registers for the
//                                     whole kernel, zero beyond n),
//     B = In[4 values of l, 16 columns]   (one word per lane per k-step).
// Lane (x, g) of a wavefront (x = lane % 16, g = lane / 16) supplies column x of B and gets
// column x of the result.  The numbering of l over (k-step s, lane group g) and of the
// result rows over (accumulator register r, lane group g) is free, because the rows and
// k-columns of A can be permuted to match; both are chosen as
//     l = off(g) + s,      i = off(g) + r   (r < KS),      off(g) = min(g*KS, n-KS),
// so that a lane always holds KS CONSECUTIVE indices of the contracted axis, all inside the
// cube (the last lane groups slide back and overlap; the overlap is zeroed in A's k-columns).
// Consequences:
//   * along the fastest axis the lane's words are contiguous in memory, so the first product
//     reads u_e and the last product writes v_e straight from/to HBM with every wavefront
//     instruction covering one contiguous run of 16 rows of the [n*n, n] matrix;
//   * the accumulators of a forward product are, unchanged, the B operands of the backward
//     product along the same axis: the diagonal scale and the turn-around need no LDS.
//
// Order: forward axis 2 (B from HBM), forward axis 1, forward axis 0, scale by D_e (loaded
// from HBM in accumulator layout at kernel start), backward axis 0 (registers), backward
// axis 1, backward axis 2 (accumulators to HBM).  Between products the cube lives in LDS, one
// buffer, updated in place: a tile reads and writes only its own columns.  Nothing between
// the load of u_e, D_e and the store of v_e touches HBM.
//
// In fp64 a lane's KS consecutive result words are 32 bytes, stored by two instructions that
// each write half of every row of the tile: every 128-byte line of v_e reaches the L2 as two
// partial writes (measured at n = 16: twice the write requests of a plain stream).  For n >= 8
// the last product therefore runs with its operands swapped, Out^T = In^T * Mat^T: the data
// rows are the A operand (the same registers as before: lane (x, g) holds its row's words
// off(g) .. off(g)+KS-1), the matrix is the B operand in natural row order, and result register
// r of lane (x, g) is Out[row 4r+g of the tile][i = x]: a store instruction writes four whole
// rows (16 lanes x 8 bytes each).  Same products, same order of summation: the results are
// bit-identical to the unswapped form, the write requests are those of a plain stream, and
// the kernel is 0.5-1 % (n = 16, one shared matrix) to 7 % (three matrices) faster.
//
// A workgroup of NW wavefronts handles G elements; the G*ceil(n*n/16) tiles of a product are
// dealt round-robin to the wavefronts, with a barrier between products.
#pragma once
#include <hip/hip_runtime.h>

#include "tpo_internal.h"
#include "tpo_pencil.hpp"   // PencilShape pitches, gload/gstore

namespace tpo {

// Hardware layouts (checked on gfx950): A[m][k] is read from lane 16*k + m, B[k][n] from lane
// 16*k + n, and accumulator register r of lane (x, g) is D[m][x] with m = 4r+g (f64) or
// m = 4g+r (f32).  split() undoes that: hardware row m -> (lane group, register).
template <typename T> struct Mfma;
template <> struct Mfma<double> {
    typedef double acc_t __attribute__((ext_vector_type(4)));
    static __device__ __forceinline__ acc_t mma(double a, double b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ void split(int m, int &grp, int &reg) { grp = m & 3; reg = m >> 2; }
};
template <> struct Mfma<float> {
    typedef float acc_t __attribute__((ext_vector_type(4)));
    static __device__ __forceinline__ acc_t mma(float a, float b, acc_t c)
    {
        return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
    }
    static __device__ __forceinline__ void split(int m, int &grp, int &reg) { grp = m >> 2; reg = m & 3; }
};

template <typename T, int N, int G, int NW>
struct MfmaShape {
    using Pitch = PencilShape<T, N, G>;
    static constexpr int P2 = N * N;
    static constexpr int N3 = N * N * N;
    static constexpr int TILES = (P2 + 15) / 16;            // column tiles per element
    static constexpr int TT = G * TILES;                    // tiles per workgroup
    static constexpr int TPW = (TT + NW - 1) / NW;          // tiles per wavefront
    static constexpr int KS = (N + 3) / 4;                  // k-steps; words per lane
    static constexpr int NT = 64 * NW;
    static constexpr int PA = Pitch::PA, PB = Pitch::PB, CUBE = Pitch::CUBE;
    static constexpr size_t LDS_BYTES = (size_t)G * CUBE * sizeof(T);
};

// PERSIST = false: one workgroup per batch of G elements (grid = number of batches).
// PERSIST = true : a fixed grid of workgroups walks over the batches (batch = blockIdx.x,
// + gridDim.x, ...) and loads the next batch's u_e and D_e into registers while the current
// one is being computed, so that no workgroup ever sits idle waiting for its first loads.
// WAVES: wavefronts per SIMD the register allocation must leave room for (1 = no demand).
// SAMES = true: the caller passed one matrix for all three directions (equal pointers); the A
// operands are then held once instead of three times (n = 16 in fp64: 134 instead of 156
// VGPRs, 1.15 against 1.21 ms on 65536 elements).
// SEP != 0: D is not read; every lane evaluates the D_e entries of its accumulator layout from
// the separable form 1 / (((lam_x[a] + lam_y[b]) + lam_z[c]) + mu[e]) (SEP = 1: IEEE division,
// 2: recip_<false>) where the D form loads them; D is ignored and may be null.
template <typename T, int N, int G, int NW, int HINT, bool PERSIST, bool SAMES, int WAVES,
          bool XCD = false, int SEP = 0>
__global__ void __launch_bounds__((MfmaShape<T, N, G, NW>::NT))
__attribute__((amdgpu_waves_per_eu(WAVES)))
ihelm_mfma_kernel(const T *u, const T *__restrict__ Sx, const T *__restrict__ Sy,
                  const T *__restrict__ Sz, const T *__restrict__ D, T *v,
                  long long num_elems, const T *__restrict__ lam_x = nullptr,
                  const T *__restrict__ lam_y = nullptr, const T *__restrict__ lam_z = nullptr,
                  const T *__restrict__ mu = nullptr)
{
    using Sh = MfmaShape<T, N, G, NW>;
    using M = Mfma<T>;
    using acc_t = typename M::acc_t;
    constexpr int P2 = Sh::P2, N3 = Sh::N3, TILES = Sh::TILES, TT = Sh::TT, TPW = Sh::TPW;
    constexpr int KS = Sh::KS;
    constexpr int PA = Sh::PA, PB = Sh::PB, CUBE = Sh::CUBE;
    constexpr bool LD_NT = (HINT & 1) != 0, ST_NT = (HINT & 2) != 0;

    extern __shared__ __align__(16) unsigned char tpo_lds[];
    T *cube = reinterpret_cast<T *>(tpo_lds);

    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const int lane = tid & 63;
    const int x = lane & 15;       // column inside a tile; hardware row of the A operand
    const int g = lane >> 4;       // lane group
    const long long nbatch = (num_elems + G - 1) / G;

    // Lane group g holds the KS consecutive indices off(g) .. off(g)+KS-1 of the contracted
    // axis, off(g) = min(g*KS, n-KS): the last groups slide back so that every index stays
    // inside the cube.  An index is "owned" by the group whose unslid range contains it; the
    // k-columns of A are zero for indices a group holds but does not own, so nothing is
    // counted twice, while result rows are simply duplicated (equal values, equal addresses).
    const int off = (g * KS < N - KS) ? g * KS : N - KS;

    // ---- A operands: the six matrices with rows and k-columns arranged as above ------------
    constexpr int ND = SAMES ? 1 : 3;           // distinct direction matrices held
    T a_fwd[ND][KS], a_bwd[ND][KS];
    {
        int grp, reg;
        M::split(x, grp, reg);                      // hardware row x -> (lane group, register)
        const int offr = (grp * KS < N - KS) ? grp * KS : N - KS;
        const bool iok = reg < KS;
        const int i = iok ? offr + reg : 0;
        const T *S[3] = {Sx, Sy, Sz};
#pragma unroll
        for (int d = 0; d < ND; ++d) {
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                const int l = off + s;
                const bool ok = iok && (l >= g * KS);
                const T f = S[d][l * N + i];        // forward: Mat[i][l] = S[l][i]
                const T b = S[d][i * N + l];        // backward: Mat[i][l] = S[i][l]
                a_fwd[d][s] = ok ? f : T(0);
                a_bwd[d][s] = ok ? b : T(0);
            }
        }
    }

    // ---- B operand of the swapped last product: Mat[i = x][l = off(g)+s], natural row order --
    constexpr bool SWAP_LAST = sizeof(T) == 8 && N >= 8;
    T b_last[SWAP_LAST ? KS : 1];
    if constexpr (SWAP_LAST) {
        const T *Sl = SAMES ? Sx : Sz;
#pragma unroll
        for (int s = 0; s < KS; ++s) {
            const int l = off + s;
            const bool ok = (x < N) && (l >= g * KS);
            const T b = Sl[(x < N ? x : 0) * N + l];    // backward: Mat[i][l] = S[i][l]
            b_last[s] = ok ? b : T(0);
        }
    }

    // ---- per-tile column data (the same for every batch) -----------------------------------
    int b0[TPW], b1[TPW], b2[TPW];     // LDS offsets of (off, column X) for the three axes
    int o2[TPW], o0[TPW];              // word offsets inside the batch: (a,b,off) / (off,b,c)
    int o2z[TPW], o0z[TPW];            // the same for element 0 of the batch
    int gel[TPW];                      // element slot of the tile (uniform over the wavefront)
    bool colst[TPW];                   // the lane's column exists in a full batch
    T lam_bc[SEP != 0 ? TPW : 1][2];   // lam_y[b], lam_z[c] of the lane's column (b, c), per tile
    T lam_a[SEP != 0 ? KS : 1];        // lam_x[off + r]: the axis-0 indices of the lane's rows
#pragma unroll
    for (int j = 0; j < TPW; ++j) {
        const int tt = wave + NW * j;
        int ge = tt / TILES;
        const int t = tt - ge * TILES;
        int X = 16 * t + x;
        colst[j] = (tt < TT) && (X < P2);
        if (!colst[j]) { ge = 0; X = 0; }           // a valid column whose results are dropped
        gel[j] = ge;
        const int hi = X / N, lo = X - hi * N;
        b0[j] = ge * CUBE + hi * PB + lo + off * PA;
        b1[j] = ge * CUBE + hi * PA + lo + off * PB;
        b2[j] = ge * CUBE + hi * PA + lo * PB + off;
        o2z[j] = X * N + off;
        o0z[j] = X + off * P2;
        o2[j] = ge * N3 + o2z[j];
        o0[j] = ge * N3 + o0z[j];
        if constexpr (SEP != 0) {
            lam_bc[j][0] = lam_y[hi];
            lam_bc[j][1] = lam_z[lo];
        }
    }
    if constexpr (SEP != 0) {
#pragma unroll
        for (int r = 0; r < KS; ++r) lam_a[r] = lam_x[off + r];
    }

    T un[TPW][KS];      // u_e chunks of the batch about to be computed (B operands, axis 2)
    T dreg[TPW][KS];    // D_e in the accumulator layout of the axis-0 products

    // Loads of one batch; tiles of element slots beyond the end of the field read slot 0.
    auto load_u = [&](long long batch) {
        const long long left = num_elems - batch * G;
        const T *ub = u + (size_t)batch * (size_t)(G * N3);
#pragma unroll
        for (int j = 0; j < TPW; ++j)
            load_words<LD_NT>(ub + (gel[j] < left ? o2[j] : o2z[j]), un[j]);
    };
    auto load_d = [&](long long batch) {
        const long long left = num_elems - batch * G;
        if constexpr (SEP != 0) {
#pragma unroll
            for (int j = 0; j < TPW; ++j) {
                const T mu_e = mu[batch * G + (gel[j] < left ? gel[j] : 0)];
#pragma unroll
                for (int r = 0; r < KS; ++r)
                    dreg[j][r] = recip_<SEP == 1>(((lam_a[r] + lam_bc[j][0]) + lam_bc[j][1]) + mu_e);
            }
        } else {
            const T *db = D + (size_t)batch * (size_t)(G * N3);
#pragma unroll
            for (int j = 0; j < TPW; ++j) {
                const T *dp = db + (gel[j] < left ? o0[j] : o0z[j]);
#pragma unroll
                for (int r = 0; r < KS; ++r) dreg[j][r] = gload<LD_NT>(dp + r * P2);
            }
        }
    };

    // Every product below is written as: all B operands of the wavefront's tiles, then the
    // MFMAs with the k-step outermost (so that consecutive MFMAs belong to different tiles and
    // never wait on each other), then all stores.
#define TPO_MMA_ALL(ACC, AOP, BOP)                                            \
    _Pragma("unroll") for (int s = 0; s < KS; ++s)                            \
        _Pragma("unroll") for (int j = 0; j < TPW; ++j)                       \
            ACC[j] = M::mma(AOP[s], BOP, ACC[j]);
#define TPO_ZERO_ACC(ACC) \
    _Pragma("unroll") for (int j = 0; j < TPW; ++j) ACC[j] = acc_t{0, 0, 0, 0};

    // XCD (one-shot grids only): batches renumbered per accelerator die as in tpo_pencil.hpp
    long long batch = PERSIST ? (long long)blockIdx.x : pencil_batch<XCD>(nbatch);
    if (batch >= nbatch) return;
    load_u(batch);
    load_d(batch);

    for (;;) {
        const long long left = num_elems - batch * G;
        const long long next = PERSIST ? batch + gridDim.x : nbatch;
        bool colok[TPW];
#pragma unroll
        for (int j = 0; j < TPW; ++j) colok[j] = colst[j] && (gel[j] < left);

        acc_t acc[TPW];
        T bv[TPW][KS];

        // ---- forward axis 2: B = u_e chunks (registers), result to LDS ----------------------
        TPO_ZERO_ACC(acc)
        TPO_MMA_ALL(acc, a_fwd[SAMES ? 0 : 2], un[j][s])
        if (PERSIST && next < nbatch) load_u(next);     // next batch's u_e, in flight from here
#pragma unroll
        for (int j = 0; j < TPW; ++j)
            if (colok[j]) {
#pragma unroll
                for (int r = 0; r < KS; ++r) cube[b2[j] + r] = acc[j][r];
            }
        __syncthreads();

        // ---- forward axis 1: LDS -> LDS -------------------------------------------------------
#pragma unroll
        for (int j = 0; j < TPW; ++j)
#pragma unroll
            for (int s = 0; s < KS; ++s) bv[j][s] = cube[b1[j] + s * PB];
        TPO_ZERO_ACC(acc)
        TPO_MMA_ALL(acc, a_fwd[SAMES ? 0 : 1], bv[j][s])
#pragma unroll
        for (int j = 0; j < TPW; ++j)
            if (colok[j]) {
#pragma unroll
                for (int r = 0; r < KS; ++r) cube[b1[j] + r * PB] = acc[j][r];
            }
        __syncthreads();

        // ---- forward axis 0, scale by D_e, backward axis 0 (register to register) ------------
#pragma unroll
        for (int j = 0; j < TPW; ++j)
#pragma unroll
            for (int s = 0; s < KS; ++s) bv[j][s] = cube[b0[j] + s * PA];
        TPO_ZERO_ACC(acc)
        TPO_MMA_ALL(acc, a_fwd[SAMES ? 0 : 0], bv[j][s])
#pragma unroll
        for (int j = 0; j < TPW; ++j)
#pragma unroll
            for (int s = 0; s < KS; ++s) bv[j][s] = acc[j][s] * dreg[j][s];
        if (PERSIST && next < nbatch) load_d(next);     // next batch's D_e
        TPO_ZERO_ACC(acc)
        TPO_MMA_ALL(acc, a_bwd[SAMES ? 0 : 0], bv[j][s])
#pragma unroll
        for (int j = 0; j < TPW; ++j)
            if (colok[j]) {
#pragma unroll
                for (int r = 0; r < KS; ++r) cube[b0[j] + r * PA] = acc[j][r];
            }
        __syncthreads();

        // ---- backward axis 1: LDS -> LDS -------------------------------------------------------
#pragma unroll
        for (int j = 0; j < TPW; ++j)
#pragma unroll
            for (int s = 0; s < KS; ++s) bv[j][s] = cube[b1[j] + s * PB];
        TPO_ZERO_ACC(acc)
        TPO_MMA_ALL(acc, a_bwd[SAMES ? 0 : 1], bv[j][s])
#pragma unroll
        for (int j = 0; j < TPW; ++j)
            if (colok[j]) {
#pragma unroll
                for (int r = 0; r < KS; ++r) cube[b1[j] + r * PB] = acc[j][r];
            }
        __syncthreads();

        // ---- backward axis 2: LDS -> HBM (one contiguous chunk per lane) -----------------------
#pragma unroll
        for (int j = 0; j < TPW; ++j)
#pragma unroll
            for (int s = 0; s < KS; ++s) bv[j][s] = cube[b2[j] + s];
        TPO_ZERO_ACC(acc)
        T *vb = v + (size_t)batch * (size_t)(G * N3);
        if constexpr (SWAP_LAST) {
            // A = data rows, B = matrix: register r of lane (x, g) is Out[row 4r+g][i = x]
#pragma unroll
            for (int s = 0; s < KS; ++s)
#pragma unroll
                for (int j = 0; j < TPW; ++j) acc[j] = M::mma(bv[j][s], b_last[s], acc[j]);
#pragma unroll
            for (int j = 0; j < TPW; ++j) {
                // the tile's own element slot and column range (gel[j] is 0 in lanes whose own
                // column lies past the end of the element; here the lane stores ROWS of the tile)
                const int tt = wave + NW * j;
                const int ge = tt / TILES;
                const int t = tt - ge * TILES;
                if (tt < TT && ge < left && x < N) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int m = sizeof(T) == 8 ? 4 * r + g : 4 * g + r;   // hardware row of register r
                        const int X = 16 * t + m;
                        if (X < P2) gstore<ST_NT>(vb + (size_t)(ge * N3 + X * N + x), acc[j][r]);
                    }
                }
            }
        } else {
            TPO_MMA_ALL(acc, a_bwd[SAMES ? 0 : 2], bv[j][s])
#pragma unroll
            for (int j = 0; j < TPW; ++j)
                if (colok[j]) {
                    T vc[KS];
#pragma unroll
                    for (int r = 0; r < KS; ++r) vc[r] = acc[j][r];
                    store_words<ST_NT>(vb + o2[j], vc);
                }
        }

        if (!PERSIST || next >= nbatch) break;
        batch = next;
        __syncthreads();        // all reads of the cube are done before the next batch writes it
    }
#undef TPO_MMA_ALL
#undef TPO_ZERO_ACC
}

// Persistent grids are sized from the occupancy the runtime reports for the kernel.
template <typename T, int N, int G, int NW, int HINT, bool PERSIST, int WAVES, bool XCD = false>
struct MfmaLauncher {
    using Sh = MfmaShape<T, N, G, NW>;
    static inline int wgs_per_device[4] = {0, 0, 0, 0};       // [SAMES + 2 * (SEP != 0)]

    template <bool SAMES, int SEP = 0>
    static hipError_t launch_as(const ApplyArgs &a)
    {
        const long long nbatch = (a.num_elems + G - 1) / G;
        if (nbatch <= 0 || nbatch > 0x7fffffffLL) return kGridTooLarge;
        long long blocks = PERSIST ? nbatch : pencil_grid<XCD>(nbatch);
        if (PERSIST) {
            constexpr int slot = SAMES + 2 * (SEP != 0);
            if (wgs_per_device[slot] <= 0) return hipErrorNotInitialized;
            if (blocks > wgs_per_device[slot]) blocks = wgs_per_device[slot];
        }
        drop_stale_error();
        hipLaunchKernelGGL((ihelm_mfma_kernel<T, N, G, NW, HINT, PERSIST, SAMES, WAVES, XCD, SEP>),
                           dim3((unsigned)blocks), dim3(Sh::NT), Sh::LDS_BYTES, a.stream,
                           (const T *)a.u, (const T *)a.sx, (const T *)a.sy, (const T *)a.sz,
                           (const T *)a.d, (T *)a.v, a.num_elems, (const T *)a.lam_x,
                           (const T *)a.lam_y, (const T *)a.lam_z, (const T *)a.mu);
        return hipGetLastError();
    }

    static hipError_t launch(const ApplyArgs &a)
    {
        return (a.sx == a.sy && a.sy == a.sz) ? launch_as<true>(a) : launch_as<false>(a);
    }
    // separable diagonal, hardware reciprocal (as the pencil families)
    static hipError_t launch_sep(const ApplyArgs &a)
    {
        return (a.sx == a.sy && a.sy == a.sz) ? launch_as<true, 2>(a) : launch_as<false, 2>(a);
    }

    template <bool SAMES, int SEP = 0>
    static hipError_t prepare_as()
    {
        const void *fn = (const void *)ihelm_mfma_kernel<T, N, G, NW, HINT, PERSIST, SAMES, WAVES, XCD, SEP>;
        if (Sh::LDS_BYTES > 48 * 1024) {
            hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize,
                                               (int)Sh::LDS_BYTES);
            if (e != hipSuccess) return e;
        }
        if (PERSIST) {
            int dev = 0, cus = 0, per_cu = 0;
            hipError_t e = hipGetDevice(&dev);
            if (e != hipSuccess) return e;
            e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
            if (e != hipSuccess) return e;
            e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, fn, Sh::NT, Sh::LDS_BYTES);
            if (e != hipSuccess) return e;
            if (per_cu < 1) per_cu = 1;
            wgs_per_device[SAMES + 2 * (SEP != 0)] = cus * per_cu;
        }
        return hipSuccess;
    }

    static hipError_t prepare()
    {
        hipError_t e = prepare_as<false>();
        if (e == hipSuccess) e = prepare_as<true>();
        if (e == hipSuccess) e = prepare_as<false, 2>();
        return e != hipSuccess ? e : prepare_as<true, 2>();
    }
};

}  // namespace tpo

// Device helpers shared by the forward and the backward kernels of the truncated-signature path: the words a lane
// owns as a tree in registers, one step of Horner's scheme (Section 2.3) on them, and the chains over the carried
// prefix.
#pragma once
#include <hip/hip_runtime.h>

#include "sg_plan.h"

namespace sg {

typedef const double __attribute__((address_space(4))) * uniform_ptr;   // constant address space: scalar loads

__host__ __device__ constexpr int ipow(int D, int m)
{
    int p = 1;
    for (int i = 0; i < m; ++i) p *= D;
    return p;
}

// The words a lane owns, level by level: node e of level m has the children e * D + c at level m + 1; level m holds
// S * D^m nodes and starts at off(m).
template <int D, int M, int S>
struct Tree {
    static constexpr int cnt(int m) { return S * ipow(D, m); }
    static constexpr int off(int m)
    {
        int o = 0;
        for (int i = 0; i < m; ++i) o += cnt(i);
        return o;
    }
    static constexpr int TOT = off(M + 1);
    static constexpr int GT = M > 0 ? off(M) : 1;

    // Lead-lag paths (Section 4) move one half of their channels per segment: H = 1, the lead half [0, D/2), H = 2, the
    // lag half [D/2, 2 (D/2)); an odd D has the time channel last, which always moves.  The increments of the other
    // channels are zero, so their multiply-adds are left out (a chain value is then the entry itself).  H = 0: all.
    template <int H>
    static constexpr bool moves(int c)
    {
        return H == 0 || ((D & 1) && c == D - 1) || (H == 1 ? c < D / 2 : (c >= D / 2 && c < 2 * (D / 2)));
    }

    // levels m .. MT of the update of the owned level MT (the word of node e at level MT has length k - 1 + 1 = k)
    template <int MT, int m, int H>
    static __device__ __forceinline__ void descend(double (&A)[TOT], double (&G)[GT], const double (&zz)[D])
    {
        constexpr int np = cnt(m - 1);
#pragma unroll
        for (int e = 0; e < np; ++e) {
            // parent word has |v| = Q + m letters and k = Q + 1 + MT, so k - |v| = MT + 1 - m
            const double gs = (m < MT) ? G[off(m - 1) + e] * (1.0 / (double)(MT + 1 - m)) : G[off(m - 1) + e];
#pragma unroll
            for (int c = 0; c < D; ++c) {
                const int i = off(m) + e * D + c;
                if (moves<H>(c)) {
                    if (m < MT) G[i] = __builtin_fma(gs, zz[c], A[i]);
                    else A[i] = __builtin_fma(gs, zz[c], A[i]);
                } else if (m < MT) {
                    G[i] = A[i];
                }
            }
        }
        if constexpr (m < MT) descend<MT, m + 1, H>(A, G, zz);
    }

    // g = G_k[u] for k = Q + 1 + MT; zc = the increments at the lane's S letters
    template <int MT, int H = 0>
    static __device__ __forceinline__ void level(double (&A)[TOT], double g, const double (&zc)[S], const double (&zz)[D])
    {
        if constexpr (MT == 0) {
#pragma unroll
            for (int s = 0; s < S; ++s) A[s] = __builtin_fma(g, zc[s], A[s]);
        } else {
            double G[GT];
            const double g0 = g * (1.0 / (double)(MT + 1));
#pragma unroll
            for (int s = 0; s < S; ++s) G[s] = __builtin_fma(g0, zc[s], A[s]);
            descend<MT, 1, H>(A, G, zz);
        }
    }

    // ---- the adjoint of the step (used by the backward kernels) ----
    // The chain values of owned level MT >= 1 as the forward step forms them: G[off(m) + i], m = 0 .. MT - 1.
    template <int MT, int m, int H>
    static __device__ __forceinline__ void chain_descend(const double (&A)[TOT], double (&G)[GT], const double (&zz)[D])
    {
        if constexpr (m < MT) {
            constexpr int np = cnt(m - 1);
#pragma unroll
            for (int e = 0; e < np; ++e) {
                const double gs = G[off(m - 1) + e] * (1.0 / (double)(MT + 1 - m));
#pragma unroll
                for (int c = 0; c < D; ++c) {
                    const int i = off(m) + e * D + c;
                    G[i] = moves<H>(c) ? __builtin_fma(gs, zz[c], A[i]) : A[i];
                }
            }
            chain_descend<MT, m + 1, H>(A, G, zz);
        }
    }

    // adjoints from level m up to the roots; Gb[off(m) ..] is complete when this is entered
    // (channels that stand still in a lead-lag segment: their increments are zero and are no variables, so neither
    // their products nor their adjoints are formed)
    template <int MT, int m, int H>
    static __device__ __forceinline__ void ascend_rev(double (&Ab)[TOT], const double (&G)[GT], double (&Gb)[GT],
                                                      const double (&zz)[D], double (&zzb)[D])
    {
        if constexpr (m >= 1) {
            constexpr int np = cnt(m - 1);
            constexpr double f = 1.0 / (double)(MT + 1 - m);
#pragma unroll
            for (int e = 0; e < np; ++e) {
                const double gs = G[off(m - 1) + e] * f;
                double acc = 0.0;
#pragma unroll
                for (int c = 0; c < D; ++c) {
                    const int i = off(m) + e * D + c;
                    Ab[i] += Gb[i];                               // the chain value holds the old entry itself
                    if (moves<H>(c)) {
                        acc = __builtin_fma(Gb[i], zz[c], acc);
                        zzb[c] = __builtin_fma(Gb[i], gs, zzb[c]);
                    }
                }
                Gb[off(m - 1) + e] = acc * f;
            }
            ascend_rev<MT, m - 1, H>(Ab, G, Gb, zz, zzb);
        }
    }

    // Adjoint of the update of owned level MT: A holds the entries before the step, Ab the adjoints (those of level MT
    // are read, those of the lower owned levels receive their share), gP = G_k[u]; returns the adjoint of gP and adds
    // to the adjoints of the increments.
    template <int MT, int H = 0>
    static __device__ __forceinline__ double level_rev(const double (&A)[TOT], double (&Ab)[TOT], double gP,
                                                       const double (&zc)[S], const double (&zz)[D], double (&zcb)[S],
                                                       double (&zzb)[D])
    {
        double gPb = 0.0;
        if constexpr (MT == 0) {
#pragma unroll
            for (int s = 0; s < S; ++s) {
                gPb = __builtin_fma(Ab[s], zc[s], gPb);
                zcb[s] = __builtin_fma(Ab[s], gP, zcb[s]);
            }
        } else {
            constexpr double i0 = 1.0 / (double)(MT + 1);
            double G[GT], Gb[GT];
            const double g0 = gP * i0;
#pragma unroll
            for (int s = 0; s < S; ++s) G[s] = __builtin_fma(g0, zc[s], A[s]);
            chain_descend<MT, 1, H>(A, G, zz);
            // the entries of level MT themselves: A_new = A + G[parent] z[c]
            constexpr int np = cnt(MT - 1);
#pragma unroll
            for (int e = 0; e < np; ++e) {
                const double gs = G[off(MT - 1) + e];
                double acc = 0.0;
#pragma unroll
                for (int c = 0; c < D; ++c) {
                    const int i = off(MT) + e * D + c;
                    if (moves<H>(c)) {
                        acc = __builtin_fma(Ab[i], zz[c], acc);
                        zzb[c] = __builtin_fma(Ab[i], gs, zzb[c]);
                    }
                }
                Gb[off(MT - 1) + e] = acc;
            }
            ascend_rev<MT, MT - 1, H>(Ab, G, Gb, zz, zzb);
#pragma unroll
            for (int s = 0; s < S; ++s) {
                Ab[s] += Gb[s];
                gPb = __builtin_fma(Gb[s], zc[s], gPb);
                zcb[s] = __builtin_fma(Gb[s], g0, zcb[s]);
            }
            gPb *= i0;
        }
        return gPb;
    }
};

// The carried prefix has Q letters.  QC is Q itself when Q <= kQExact (every loop below then has constant bounds and
// no test), else kQMax with a test of r against Q in every iteration.
template <int QC>
__device__ __forceinline__ bool has(int r, int Q)
{
    return QC <= kQExact ? true : r < Q;
}

// G_k[u] for the level that lies E letters beyond the prefix (k = Q + E): the chain over the prefixes of u.
// preR[r] / zuR[r] belong to the prefix of length Q - r (reversed so that every index below is a constant).
template <int E, int QC, int QA>
__device__ __forceinline__ double prefix_chain(int Q, const double (&preR)[QA], const double (&zuR)[QA])
{
    double g = 1.0;
#pragma unroll
    for (int r = QC - 1; r >= 0; --r)
        if (has<QC>(r, Q)) g = __builtin_fma(g, zuR[r] * (1.0 / (double)(r + 1 + E)), preR[r]);   // k - |v| = r + 1 + E
    return g;
}

template <int MT, int D, int M, int S, int QC, int TOT, int QA, int H = 0>
__device__ __forceinline__ void owned_levels(double (&A)[TOT], int Q, const double (&preR)[QA],
                                             const double (&zuR)[QA], const double (&zc)[S], const double (&zz)[D])
{
    Tree<D, M, S>::template level<MT, H>(A, prefix_chain<MT + 1, QC, QA>(Q, preR, zuR), zc, zz);
    if constexpr (MT > 0) owned_levels<MT - 1, D, M, S, QC, TOT, QA, H>(A, Q, preR, zuR, zc, zz);
}

// the carried entries at the prefixes of u: word length Q - r0, longest first
template <int QC, int QA>
__device__ __forceinline__ void prefix_levels(int Q, double (&preR)[QA], const double (&zuR)[QA])
{
#pragma unroll
    for (int r0 = 0; r0 < QC; ++r0) {
        if (has<QC>(r0, Q)) {
            double g = 1.0;
#pragma unroll
            for (int r = QC - 1; r > r0; --r)
                if (has<QC>(r, Q)) g = __builtin_fma(g, zuR[r] * (1.0 / (double)(r - r0 + 1)), preR[r]);
            preR[r0] = __builtin_fma(g, zuR[r0], preR[r0]);
        }
    }
}

// ---- adjoints over the carried prefix (backward kernels) ----
// The chain of prefix_chain<E> with every value kept: h[r] is the value after the prefix of length Q - r, h[QC] = 1.
template <int E, int QC, int QA>
__device__ __forceinline__ double prefix_chain_keep(int Q, const double (&preR)[QA], const double (&zuR)[QA],
                                                    double (&h)[QA + 1])
{
    double g = 1.0;
    h[QC] = 1.0;
#pragma unroll
    for (int r = QC - 1; r >= 0; --r) {
        if (has<QC>(r, Q)) g = __builtin_fma(g, zuR[r] * (1.0 / (double)(r + 1 + E)), preR[r]);
        h[r] = g;
    }
    return g;
}

// hb = adjoint of the chain's result: shares go to the adjoints of the carried entries and of their increments
template <int E, int QC, int QA>
__device__ __forceinline__ void prefix_chain_rev(int Q, const double (&zuR)[QA], const double (&h)[QA + 1], double hb,
                                                 double (&prb)[QA], double (&zub)[QA])
{
#pragma unroll
    for (int r = 0; r < QC; ++r) {
        if (has<QC>(r, Q)) {
            constexpr double one = 1.0;
            const double c = one / (double)(r + 1 + E);
            prb[r] += hb;
            zub[r] = __builtin_fma(hb, h[r + 1] * c, zub[r]);
            hb *= c * zuR[r];
        }
    }
}

// Adjoint of prefix_levels: the statements in the opposite order (shortest word first), each reading the adjoint
// of its own entry before any longer word has added to it.  preR holds the entries before the step.
template <int QC, int QA>
__device__ __forceinline__ void prefix_levels_rev(int Q, const double (&preR)[QA], const double (&zuR)[QA],
                                                  double (&prb)[QA], double (&zub)[QA])
{
#pragma unroll
    for (int r0 = QC - 1; r0 >= 0; --r0) {
        if (has<QC>(r0, Q)) {
            double h[QA + 1];
            double g = 1.0;
            h[QC] = 1.0;
#pragma unroll
            for (int r = QC - 1; r > r0; --r) {
                if (has<QC>(r, Q)) g = __builtin_fma(g, zuR[r] * (1.0 / (double)(r - r0 + 1)), preR[r]);
                h[r] = g;
            }
            const double a = prb[r0];
            zub[r0] = __builtin_fma(a, g, zub[r0]);
            double hb = a * zuR[r0];
#pragma unroll
            for (int r = r0 + 1; r < QC; ++r) {
                if (has<QC>(r, Q)) {
                    const double c = 1.0 / (double)(r - r0 + 1);
                    prb[r] += hb;
                    zub[r] = __builtin_fma(hb, h[r + 1] * c, zub[r]);
                    hb *= c * zuR[r];
                }
            }
        }
    }
}

template <int MT, int D, int M, int S, int QC, int TOT, int QA, int H = 0>
__device__ __forceinline__ void owned_levels_rev(const double (&A)[TOT], double (&Ab)[TOT], int Q,
                                                 const double (&preR)[QA], double (&prb)[QA], const double (&zuR)[QA],
                                                 const double (&zc)[S], const double (&zz)[D], double (&zub)[QA],
                                                 double (&zcb)[S], double (&zzb)[D])
{
    double h[QA + 1];
    const double gP = prefix_chain_keep<MT + 1, QC, QA>(Q, preR, zuR, h);
    const double gPb = Tree<D, M, S>::template level_rev<MT, H>(A, Ab, gP, zc, zz, zcb, zzb);
    prefix_chain_rev<MT + 1, QC, QA>(Q, zuR, h, gPb, prb, zub);
    if constexpr (MT < M) owned_levels_rev<MT + 1, D, M, S, QC, TOT, QA, H>(A, Ab, Q, preR, prb, zuR, zc, zz, zub, zcb, zzb);
}

}  // namespace sg

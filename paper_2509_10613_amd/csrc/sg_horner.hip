// Batched truncated signatures by Horner's scheme (paper Section 2.3) for gfx950.
//
// One step of the scheme for the increment z of a segment, read word by word (v a word, c a letter, |v| its length):
//     G_k[empty] = 1,   G_k[v c] = G_k[v] z[c] / (k - |v|) + A_{|v|+1}[v c]   for |v| + 1 < k,
//     A_k[w c] += G_k[w] z[c]                                                  for |w| = k - 1,
// levels k = N, ..., 1 in that order so that every right-hand side still holds the values before the step
// (G_k[w] is B_k[w] + A_{k-1}[w] of Section 2.3).  Starting from A = (1, 0, 0, ...), the first step gives the tensor
// exponential of the first increment (Proposition 2.1), so no separate initialisation is needed.
//
// A value at a word depends only on values at its prefixes.  A lane therefore owns a prefix u of Q letters, S
// consecutive letters after it, and all continuations by up to M more letters, in registers for the whole path, plus
// its own copies of the Q entries at the prefixes of u.  No lane talks to another one.  All lanes of a wave work on
// the same path: the D increments of a step are wave-uniform and come in by scalar loads into scalar registers, the
// few that a lane selects by its own letters come in by ordinary loads; both are fetched one step ahead.
#include <hip/hip_runtime.h>

#include "sg_dev.h"
#include "sg_kernels.h"

namespace sg {

namespace {

// The owned entries of level Q + 1 + m go to the words u (blk S + s) v: `first` is the number of the word u (blk S) in
// base D, at[m] the start of that level in the flattened signature.
template <int m, int D, int M, int S, int TOT>
__device__ __forceinline__ void store_owned(const double (&A)[TOT], double* out, const long (&at)[M + 1], int Dn,
                                            long first, int c0)
{
    constexpr int pm = ipow(D, m);
#pragma unroll
    for (int s = 0; s < S; ++s) {
        if (c0 + s < Dn) {
            double* o = out + at[m] + (first + s) * pm;
#pragma unroll
            for (int v = 0; v < pm; ++v) o[v] = A[Tree<D, M, S>::off(m) + s * pm + v];
        }
    }
    if constexpr (m < M) store_owned<m + 1, D, M, S, TOT>(A, out, at, Dn, first, c0);
}

// One wave's share of one path, all steps.  DT > 0: D = DT channels, increments of a step in scalar registers.
// DT == 0: any number of channels, M = 0, S = 1 (a lane owns one word of the top level).
// SHARED: a wave holds several short paths (lanes per path at most 32): lane groups of LP lanes, each group a path
// of its own; the increments are then per-lane values and come in by ordinary loads.
// LEADLAG: the rows alternate between a move of the lead half (even rows) and of the lag half (odd rows) of the
// channels; the multiply-adds with the half that stands still are left out.
template <int DT, int M, int S, int QC, bool SHARED, bool LEADLAG>
__device__ __forceinline__ void run(const Args& a)
{
    constexpr int DD = DT > 0 ? DT : 1;
    constexpr int QA = QC > 0 ? QC : 1;
    using T = Tree<DD, M, S>;
    const int D = DT > 0 ? DT : a.D;
    const int Q = QC <= kQExact ? QC : a.Q;
    const int lane = threadIdx.x & (kWave - 1);
    // Workgroups go to the 8 XCDs (each with an L2 of its own) in turn: number them so that the workgroups of one
    // path, which read the same increments, sit on the same XCD.
    long wg = blockIdx.x;
    if (gridDim.x % kXcds == 0) wg = (long)(blockIdx.x % kXcds) * (gridDim.x / kXcds) + blockIdx.x / kXcds;
    const long wt = wg * kWavesPerWG + __builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
    if (wt >= a.NW) return;
    long b, ti;
    bool valid;
    if constexpr (SHARED) {
        const int g = lane / (int)a.LP;
        b = wt * a.PW + g;
        ti = lane - g * (int)a.LP;
        valid = g < a.PW && b < a.B;
        if (!valid) {       // idle lanes follow the wave's first path and write nothing
            b = wt * a.PW;
            ti = 0;
        }
    } else {
        b = wt / a.WP;
        ti = (wt - b * a.WP) * kWave + lane;
        valid = ti < a.LP;
        if (!valid) ti = 0;
    }
    const int blk = (int)(ti % a.NB);
    const long rest = ti / a.NB;      // the prefix u as a number in base D, first letter most significant
    int uR[QA];
    {
        long t = rest;
#pragma unroll
        for (int r = 0; r < QA; ++r) {
            uR[r] = (r < QC && has<QC>(r, Q)) ? (int)(t % D) : 0;
            t /= D;
        }
    }
    int cs[S];
#pragma unroll
    for (int s = 0; s < S; ++s) cs[s] = min(blk * S + s, D - 1);

    double A[T::TOT];
#pragma unroll
    for (int i = 0; i < T::TOT; ++i) A[i] = 0.0;
    double preR[QA];
#pragma unroll
    for (int r = 0; r < QA; ++r) preR[r] = 0.0;

    const double* zrow = a.dz + b * a.np * a.Dpad;
    double zz[DD], zc[S], zuR[QA];
    double zzn[DD], zcn[S], zuRn[QA];
    auto fetch = [&](long step, double (&z_)[DD], double (&zc_)[S], double (&zu_)[QA]) {
        const double* zp = zrow + step * a.Dpad;
        if constexpr (DT > 0 && M > 0 && !SHARED) {
            uniform_ptr zs = (uniform_ptr)(zp);
#pragma unroll
            for (int c = 0; c < DD; ++c) z_[c] = zs[c];
        } else if constexpr (DT > 0 && M > 0) {
#pragma unroll
            for (int c = 0; c < DD; ++c) z_[c] = zp[c];
        }
#pragma unroll
        for (int s = 0; s < S; ++s) zc_[s] = zp[cs[s]];
#pragma unroll
        for (int r = 0; r < QA; ++r) zu_[r] = (r < QC && has<QC>(r, Q)) ? zp[uR[r]] : 0.0;
    };
#pragma unroll
    for (int c = 0; c < DD; ++c) zz[c] = zzn[c] = 0.0;
    // Two steps per iteration with two sets of registers for the increments, each set requested one step before the
    // arithmetic that reads it.  Two things keep the compiler from moving a load next to its use: the body has no
    // branch (loads get moved into the block that uses them), and the set carried round the loop starts as constants,
    // not as a load (a value that is a load on every path into the loop becomes one load at the top of the body).
    // So the first step is a zero increment, which changes nothing, the rows follow in pairs, and the stored row count
    // np is odd with zero rows after the last segment.
#pragma unroll
    for (int s = 0; s < S; ++s) zc[s] = 0.0;
#pragma unroll
    for (int r = 0; r < QA; ++r) zuR[r] = 0.0;
    for (long step = 0; step < a.np; step += 2) {
        // the set carried round the loop holds the odd rows (lag half; the zero increment at the start fits any
        // half), the other set the even rows (lead half)
        fetch(step, zzn, zcn, zuRn);
        owned_levels<M, DD, M, S, QC, T::TOT, QA, LEADLAG ? 2 : 0>(A, Q, preR, zuR, zc, zz);
        prefix_levels<QC, QA>(Q, preR, zuR);
        fetch(step + 1 < a.np ? step + 1 : step, zz, zc, zuR);
        owned_levels<M, DD, M, S, QC, T::TOT, QA, LEADLAG ? 1 : 0>(A, Q, preR, zuRn, zcn, zzn);
        prefix_levels<QC, QA>(Q, preR, zuRn);
    }

    if (!valid) return;
    double* out = a.out + b * a.sig_len;
    // start of level k in the flattened signature: 1 + D + ... + D^(k-1)
    auto lvl = [&](int k) {
        long o = 0, p = 1;
        for (int i = 0; i < k; ++i) {
            o += p;
            p *= D;
        }
        return o;
    };
    if (ti == 0) out[0] = 1.0;
    // carried prefix entries: written by the lane whose remaining letters are all zero
    {
        long pw = 1;
#pragma unroll
        for (int r = 0; r < QC; ++r) {
            if (has<QC>(r, Q) && blk == 0 && rest % pw == 0) out[lvl(Q - r) + rest / pw] = preR[r];
            pw *= D;
        }
    }
    long at[M + 1];
#pragma unroll
    for (int m = 0; m <= M; ++m) at[m] = lvl(Q + 1 + m);
    store_owned<0, DD, M, S, T::TOT>(A, out, at, D, rest * D + blk * S, blk * S);
}

template <int DT, int M, int S, int QC, bool SHARED, bool LEADLAG>
__global__ __launch_bounds__(kWave * kWavesPerWG) void horner_kernel(const Args a)
{
    run<DT, M, S, QC, SHARED, LEADLAG>(a);
}

// Increments of the transformed paths (Section 4), one row of Dpad doubles per segment: channels of the path (after
// the lead-lag transform: lead half, then lag half; a segment of the transformed path moves one half only, the lead
// first), then the time channel 1/n if asked for, then zero padding.  A path is stored as P pieces of np rows: piece p
// holds the segments p Lc .. p Lc + Lc - 1 (those below n), then zero rows.
template <typename TI>
__global__ __launch_bounds__(256) void increments_kernel(const TI* __restrict__ x, double* __restrict__ dz, long B, long L,
                                                         int d, int D, int Dpad, long n, int P, long Lc, long np,
                                                         int time_aug, int lead_lag)
{
    const long total = B * P * np * Dpad;
    for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
        const int c = (int)(i % Dpad);
        const long bs = i / Dpad;
        const long j = bs % np;
        const long bp = bs / np;
        const long piece = bp % P;
        const long b = bp / P;
        const long s = piece * Lc + j;
        double v = 0.0;
        if (j >= Lc || s >= n) {
            // a zero row: past the piece or past the path
        } else if (time_aug && c == D - 1) {
            v = 1.0 / (double)n;
        } else if (c < D) {
            long seg = s;
            int ch = c;
            bool moves = true;
            if (lead_lag) {
                seg = s >> 1;
                const bool lag_half = c >= d;
                ch = lag_half ? c - d : c;
                moves = ((s & 1) != 0) == lag_half;
            }
            if (moves) {
                const TI* xp = x + (b * L + seg) * d + ch;
                v = (double)xp[d] - (double)xp[0];
            }
        }
        dz[i] = v;
    }
}

// Chen's identity (Proposition 2.2) for pairs of neighbouring pieces: out[i] = in[2 i] (x) in[2 i + 1], truncated at
// level N; entry w of level k is sum_{j=0..k} A[first j letters of w] B[last k - j letters of w].  One thread per entry.
__global__ __launch_bounds__(256) void chen_pairs_kernel(const double* __restrict__ in, double* __restrict__ out, long pairs,
                                                         int D, int N, long sig_len)
{
    const unsigned Du = (unsigned)D;
    for (long e = (long)blockIdx.x * blockDim.x + threadIdx.x; e < sig_len; e += (long)gridDim.x * blockDim.x) {
        // level k and word number of entry e (32-bit arithmetic: a signature here has fewer than 2^31 entries)
        int k = 0;
        unsigned at = 0, pw = 1;            // start of level k, D^k
        while ((unsigned)e >= at + pw) {
            at += pw;
            pw *= Du;
            ++k;
        }
        for (long pr = blockIdx.y; pr < pairs; pr += gridDim.y) {
            const double* A = in + 2 * pr * sig_len;
            const double* Bm = A + sig_len;
            // t = 0 .. k letters go to the second factor: the prefix of k - t letters has the number w / D^t, the
            // suffix the number w % D^t; one letter moves over per term
            unsigned pre = (unsigned)e - at, suf = 0, div = 1;
            unsigned at_pre = at;      // start of level k - t
            unsigned pw_pre = pw;      // D^(k - t)
            unsigned at_suf = 0;       // start of level t
            double acc = 0.0;
            for (int t = 0; t <= k; ++t) {
                acc = __builtin_fma(A[at_pre + pre], Bm[at_suf + suf], acc);
                const unsigned q = pre / Du;
                suf += (pre - q * Du) * div;
                pre = q;
                at_suf += div;
                div *= Du;
                pw_pre /= Du;
                at_pre -= pw_pre;
            }
            out[pr * sig_len + e] = acc;
        }
    }
}

template <int DT, int M, int S, int QC, bool SHARED>
hipError_t launch_one(const Args& a, long grid, hipStream_t st)
{
    // kernels that skip the half of the channels a lead-lag segment does not move: where a lane has registers over
    // those channels at all (M >= 1) and at least four channels
    if constexpr (DT >= 4 && M >= 1) {
        if (a.leadlag) {
            hipLaunchKernelGGL((horner_kernel<DT, M, S, QC, SHARED, true>), dim3((unsigned)grid), dim3(kWave * kWavesPerWG), 0, st, a);
            return hipGetLastError();
        }
    }
    hipLaunchKernelGGL((horner_kernel<DT, M, S, QC, SHARED, false>), dim3((unsigned)grid), dim3(kWave * kWavesPerWG), 0, st, a);
    return hipGetLastError();
}

// prefix lengths up to kQExact have kernels of their own; longer ones share the kernel that tests against Q, which
// exists for the channel counts that can reach them (kLongPrefixMaxD).  Kernels whose waves hold several paths exist
// for prefixes up to kSharedMaxQ letters and up to kSharedMaxD channels (beyond that a path fills a wave anyway).
template <int DT, int M, int S>
hipError_t launch_variant(const Args& a, long grid, hipStream_t st)
{
    if (a.PW > 1) {
        if constexpr (DT <= kSharedMaxD) {
            switch (a.Q) {
            case 0: return launch_one<DT, M, S, 0, true>(a, grid, st);
            case 1: return launch_one<DT, M, S, 1, true>(a, grid, st);
            case 2: return launch_one<DT, M, S, 2, true>(a, grid, st);
            default: return hipErrorInvalidValue;
            }
        } else {
            return hipErrorInvalidValue;
        }
    }
    switch (a.Q) {
    case 0: return launch_one<DT, M, S, 0, false>(a, grid, st);
    case 1: return launch_one<DT, M, S, 1, false>(a, grid, st);
    case 2: return launch_one<DT, M, S, 2, false>(a, grid, st);
    case 3: return launch_one<DT, M, S, 3, false>(a, grid, st);
    case 4: return launch_one<DT, M, S, 4, false>(a, grid, st);
    default:
        if constexpr (DT <= kLongPrefixMaxD) return launch_one<DT, M, S, kQMax, false>(a, grid, st);
        else return hipErrorInvalidValue;
    }
}

}  // namespace

hipError_t launch_horner(int DT, int M, int S, const Args& a, long grid, hipStream_t st)
{
    if (grid <= 0) return hipSuccess;
    if ((a.np > 0 && !(a.np & 1)) || a.np < a.n || a.Q < 0 || a.Q > kQMax || a.LP <= 0 || a.WP * kWave < a.LP || a.NB * (long)S < (DT ? DT : a.D))
        return hipErrorInvalidValue;
    if (a.PW < 1 || (a.PW > 1 && (a.WP != 1 || a.PW * a.LP > kWave || a.NW * a.PW < a.B)) || (a.PW == 1 && a.NW != a.B * a.WP) ||
        grid * kWavesPerWG < a.NW)
        return hipErrorInvalidValue;
    if (a.leadlag && (a.n & 1)) return hipErrorInvalidValue;      // pieces of a lead-lag path start with a lead move
    if (DT == 0) return (M == 0 && S == 1) ? launch_variant<0, 0, 1>(a, grid, st) : hipErrorInvalidValue;
#define SG_CASE(D_, M_, S_) \
    if (DT == D_ && M == M_ && S == S_) return launch_variant<D_, M_, S_>(a, grid, st);
    SG_VARIANTS(SG_CASE)
#undef SG_CASE
    return hipErrorInvalidValue;
}

hipError_t launch_chen_pairs(const double* in, double* out, long pairs, int D, int N, long sig_len, hipStream_t st)
{
    if (pairs <= 0 || sig_len <= 0) return hipSuccess;
    if (sig_len >= (1L << 31) || D < 1) return hipErrorInvalidValue;
    long gx = (sig_len + 255) / 256;
    if (gx > 65536) gx = 65536;
    const long gy = pairs < 65535 ? pairs : 65535;
    hipLaunchKernelGGL(chen_pairs_kernel, dim3((unsigned)gx, (unsigned)gy), dim3(256), 0, st, in, out, pairs, D, N, sig_len);
    return hipGetLastError();
}

template <typename TI>
hipError_t launch_increments(const TI* x, double* dz, long B, long L, int d, int D, int Dpad, long n, int P, long Lc,
                             long np, int time_aug, int lead_lag, hipStream_t st)
{
    if (P < 1 || np < Lc || P * Lc < n || (np > 0 && !(np & 1))) return hipErrorInvalidValue;
    const long total = B * P * np * Dpad;
    if (total <= 0) return hipSuccess;
    long grid = (total + 255) / 256;
    if (grid > 65536) grid = 65536;
    hipLaunchKernelGGL((increments_kernel<TI>), dim3((unsigned)grid), dim3(256), 0, st, x, dz, B, L, d, D, Dpad, n, P, Lc,
                       np, time_aug, lead_lag);
    return hipGetLastError();
}

template hipError_t launch_increments<float>(const float*, double*, long, long, int, int, int, long, int, long, long, int, int, hipStream_t);
template hipError_t launch_increments<double>(const double*, double*, long, long, int, int, int, long, int, long, long, int, int, hipStream_t);

}  // namespace sg

// Gradient of batched truncated signatures with respect to the path points (paper Section 2.4) for gfx950.
//
// Section 2.4 walks the path backwards: the signature before a segment is recovered from the one after it,
// S_{l-1} = S_l (x) exp(-z_l), which is Horner's step of Section 2.3 with the increment negated, and the adjoint
// (dF/dS_l -> dF/dS_{l-1}, dF/dz_l) is taken through that one step.  The lanes are those of the forward kernel: a lane
// owns the entries under a prefix u and a block of next letters, in registers, now together with their adjoints.
// The adjoint of the step is linear in the incoming adjoints, so the adjoints of the entries at the prefixes of u,
// which every lane under the prefix carries a copy of, never have to be summed over lanes: each lane carries a share
// (the upstream value starts in one lane, zero in the others) and the shares add up to the adjoint at every step.
// Only dF/dz_l is a sum over all lanes of a path: per step a wave adds its lanes' shares in LDS (each lane a row,
// summed column by column) and issues one global atomic per channel.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "sg_dev.h"
#include "sg_kernels.h"

namespace sg {

namespace {

template <int D, int M, int S, int TOT, int m = 0>
__device__ __forceinline__ void load_owned(double (&A)[TOT], const double* src, const long (&at)[M + 1], int Dn,
                                           long first, int c0, bool valid)
{
    constexpr int pm = ipow(D, m);
#pragma unroll
    for (int s = 0; s < S; ++s) {
        const bool ok = valid && c0 + s < Dn;
        const double* o = src + at[m] + (first + s) * pm;
#pragma unroll
        for (int v = 0; v < pm; ++v) A[Tree<D, M, S>::off(m) + s * pm + v] = ok ? o[v] : 0.0;
    }
    if constexpr (m < M) load_owned<D, M, S, TOT, m + 1>(A, src, at, Dn, first, c0, valid);
}

// SHARED: a wave holds several short paths (lane groups of LP <= 32 lanes, as in the forward kernel); a path then
// lives in one wave, and the sums of dF/dz over its lanes are stored, not added.
// LEADLAG: even rows move the lead half of the channels, odd rows the lag half; the multiply-adds and adjoints of the
// half that stands still are left out, as in the forward kernel.
template <int DT, int M, int S, int QC, bool SHARED, bool LEADLAG>
__device__ __forceinline__ void run_bwd(const BwdArgs& a, double* lds)
{
    constexpr int DD = DT > 0 ? DT : 1;
    constexpr int QA = QC > 0 ? QC : 1;
    constexpr bool kRows = DT > 0 && M > 0;            // the lanes' shares of dF/dz go through rows in LDS
    constexpr bool kUniformZ = kRows && !SHARED;       // increments of a step in scalar registers
    static_assert(!SHARED || kRows, "waves that hold several paths exist for the kernels with rows only");
    using T = Tree<DD, M, S>;
    const int D = DT > 0 ? DT : a.D;
    const int Q = QC <= kQExact ? QC : a.Q;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x / kWave));
    long wg = blockIdx.x;
    if (gridDim.x % kXcds == 0) wg = (long)(blockIdx.x % kXcds) * (gridDim.x / kXcds) + blockIdx.x / kXcds;
    const long wt = wg * kWavesPerWG + wave;
    if (wt >= a.NW) return;
    long b, ti;
    bool valid;
    if constexpr (SHARED) {
        const int g = lane / (int)a.LP;
        b = wt * a.PW + g;
        ti = lane - g * (int)a.LP;
        valid = g < a.PW && b < a.B;
        if (!valid) {       // idle lanes follow the wave's first path with zero adjoints
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
    const long rest = ti / a.NB;
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
    bool cok[S];
#pragma unroll
    for (int s = 0; s < S; ++s) {
        cok[s] = valid && blk * S + s < D;
        cs[s] = min(blk * S + s, D - 1);
    }

    // this wave's LDS: Dpad sums per channel, then (kernels with wave-uniform increments) 64 rows of DS doubles
    const int DS = D | 1;
    double* acc = lds + (size_t)wave * a.lds_wave;
    double* tr = acc + a.Dpad;
    for (int c = lane; c < a.Dpad; c += kWave) acc[c] = 0.0;

    auto lvl = [&](int k) {
        long o = 0, p = 1;
        for (int i = 0; i < k; ++i) {
            o += p;
            p *= D;
        }
        return o;
    };
    long at[M + 1];
#pragma unroll
    for (int m = 0; m <= M; ++m) at[m] = lvl(Q + 1 + m);

    // the signature of the whole path and the upstream gradient, each lane its own entries
    double A[T::TOT], Ab[T::TOT], preR[QA], prb[QA];
    const double* sig = a.sig + b * a.sig_len;
    const double* gout = a.gout + b * a.sig_len;
    load_owned<DD, M, S, T::TOT>(A, sig, at, D, rest * D + blk * S, blk * S, true);
    load_owned<DD, M, S, T::TOT>(Ab, gout, at, D, rest * D + blk * S, blk * S, valid);
    {
        long pw = 1;
#pragma unroll
        for (int r = 0; r < QA; ++r) {
            preR[r] = 0.0;
            prb[r] = 0.0;
            if (r < QC && has<QC>(r, Q)) {
                const long idx = lvl(Q - r) + rest / pw;
                preR[r] = sig[idx];
                if (valid && blk == 0 && rest % pw == 0) prb[r] = gout[idx];   // one lane starts with the upstream value
            }
            pw *= D;
        }
    }

    const double* zrow = a.dz + b * a.np * a.Dpad;
    double* grow = a.gz + b * a.np * a.Dpad;
    double zz[DD], zc[S], zuR[QA];
    double zzn[DD], zcn[S], zuRn[QA];
    auto fetch = [&](long row, double (&z_)[DD], double (&zc_)[S], double (&zu_)[QA]) {
        const double* zp = zrow + row * a.Dpad;
        if constexpr (kUniformZ) {
            uniform_ptr zs = (uniform_ptr)(zp);
#pragma unroll
            for (int c = 0; c < DD; ++c) z_[c] = zs[c];
        } else if constexpr (kRows) {
#pragma unroll
            for (int c = 0; c < DD; ++c) z_[c] = zp[c];
        }
#pragma unroll
        for (int s = 0; s < S; ++s) zc_[s] = zp[cs[s]];
#pragma unroll
        for (int r = 0; r < QA; ++r) zu_[r] = (r < QC && has<QC>(r, Q)) ? zp[uR[r]] : 0.0;
    };

    // The sum of dF/dz[row] over the lanes of the wave takes three hops through LDS, and they are spread over three
    // segments so that no hop waits for the one before it: after segment i the lanes publish their shares of row i
    // (a row of DS doubles per lane: the shares that belong to the wave-uniform increments are written, the shares a
    // lane formed with increments it picked by its own letters are added into the same row by LDS atomics, which never
    // meet another lane's); the rows published after the previous segment are summed column by column by a few lanes
    // per channel into acc; and the sums that reached acc one segment earlier go out as one global atomic per channel.
    // LDS executes a wave's instructions in order, which is all the synchronisation this needs.
    long r1 = -1, r2 = -1;   // row whose shares sit in the lanes' LDS rows / row whose sums sit in acc
    auto publish = [&](const double (&zzb)[DD], const double (&zcb)[S], const double (&zub)[QA]) {
#pragma unroll
        for (int cc = 0; cc < DD; ++cc) tr[lane * DS + cc] = zzb[cc];
#pragma unroll
        for (int s = 0; s < S; ++s)
            if (cok[s]) atomicAdd(&tr[lane * DS + cs[s]], zcb[s]);
#pragma unroll
        for (int r = 0; r < QC; ++r)
            if (has<QC>(r, Q)) atomicAdd(&tr[lane * DS + uR[r]], zub[r]);
    };
    // waves that hold several paths: two hops (rows, then one lane per path and channel sums the rows of its path and
    // stores the result: no other wave has a share of it)
    auto reduce_step_shared = [&](long row_new, const double (&zzb)[DD], const double (&zcb)[S], const double (&zub)[QA]) {
        if (r1 >= 0) {
            const int LPi = (int)a.LP;
            for (int idx = lane; idx < a.PW * DD; idx += kWave) {
                const int g = idx / DD, c = idx - g * DD;
                const long bg = wt * a.PW + g;
                if (bg < a.B) {
                    // all reads issued back to back (rows past the group are read again and not counted)
                    const double* col = tr + g * LPi * DS + c;
                    double s0 = 0.0, s1 = 0.0;
                    auto rows = [&](auto count) {
#pragma unroll
                        for (int i = 0; i < decltype(count)::value; i += 2) {
                            const double v0 = col[min(i, LPi - 1) * DS], v1 = col[min(i + 1, LPi - 1) * DS];
                            s0 += i < LPi ? v0 : 0.0;
                            s1 += i + 1 < LPi ? v1 : 0.0;
                        }
                    };
                    if (LPi <= 2) rows(std::integral_constant<int, 2>());
                    else if (LPi <= 4) rows(std::integral_constant<int, 4>());
                    else if (LPi <= 8) rows(std::integral_constant<int, 8>());
                    else if (LPi <= 16) rows(std::integral_constant<int, 16>());
                    else rows(std::integral_constant<int, 32>());
                    a.gz[(bg * a.np + r1) * a.Dpad + c] = s0 + s1;
                }
            }
        }
        if (row_new >= 0) publish(zzb, zcb, zub);
        r1 = row_new;
    };
    auto reduce_step = [&](long row_new, const double (&zzb)[DD], const double (&zcb)[S], const double (&zub)[QA]) {
        constexpr int P = kWave / DD;                  // lanes per channel
        constexpr int R = (kWave + P - 1) / P;         // LDS rows per lane
        const bool flush = r2 >= 0, coll = r1 >= 0;
        const int c = lane % DD, q = lane / DD;
        double v = 0.0, sum = 0.0;
        if (flush && lane < DD) v = acc[lane];
        if (coll && lane < DD * P) {
#pragma unroll
            for (int i = 0; i < R; ++i) {
                const int rw = q * R + i;
                if (rw < kWave) sum += tr[rw * DS + c];
            }
        }
        if (flush && lane < DD) {
            acc[lane] = 0.0;
            atomicAdd(&grow[r2 * a.Dpad + lane], v);
        }
        if (coll && lane < DD * P) atomicAdd(&acc[c], sum);
        if (row_new >= 0) publish(zzb, zcb, zub);
        r2 = r1;
        r1 = row_new;
    };

    // one segment backwards; row < 0: the zero increment that starts the loop, nothing to add anywhere
    auto segment = [&](auto half, long row, const double (&z_)[DD], const double (&zc_)[S], const double (&zu_)[QA]) {
        constexpr int H = decltype(half)::value;
        // the signature before the segment: the forward step with the increment negated
        double nz[DD], nzc[S], nzu[QA];
#pragma unroll
        for (int c = 0; c < DD; ++c) nz[c] = -z_[c];
#pragma unroll
        for (int s = 0; s < S; ++s) nzc[s] = -zc_[s];
#pragma unroll
        for (int r = 0; r < QA; ++r) nzu[r] = -zu_[r];
        owned_levels<M, DD, M, S, QC, T::TOT, QA, H>(A, Q, preR, nzu, nzc, nz);
        prefix_levels<QC, QA>(Q, preR, nzu);
        // the adjoint of the forward step from that signature with the increment itself
        double zzb[DD], zcb[S], zub[QA];
#pragma unroll
        for (int c = 0; c < DD; ++c) zzb[c] = 0.0;
#pragma unroll
        for (int s = 0; s < S; ++s) zcb[s] = 0.0;
#pragma unroll
        for (int r = 0; r < QA; ++r) zub[r] = 0.0;
        prefix_levels_rev<QC, QA>(Q, preR, zu_, prb, zub);
        owned_levels_rev<0, DD, M, S, QC, T::TOT, QA, H>(A, Ab, Q, preR, prb, zu_, zc_, z_, zub, zcb, zzb);
        if constexpr (SHARED) {
            reduce_step_shared(row, zzb, zcb, zub);
        } else if constexpr (kRows) {
            reduce_step(row, zzb, zcb, zub);
        } else {
            // run-time channel count: the shares go straight to acc by LDS atomics (lanes with equal letters meet)
            if (row < 0) return;
#pragma unroll
            for (int s = 0; s < S; ++s)
                if (cok[s]) atomicAdd(&acc[cs[s]], zcb[s]);
#pragma unroll
            for (int r = 0; r < QC; ++r)
                if (has<QC>(r, Q)) atomicAdd(&acc[uR[r]], zub[r]);
            __builtin_amdgcn_wave_barrier();
            for (int c = lane; c < D; c += kWave) {
                const double v = acc[c];
                acc[c] = 0.0;
                atomicAdd(&grow[row * a.Dpad + c], v);
            }
            __builtin_amdgcn_wave_barrier();
        }
    };

    // Rows np-1 .. 0, two per iteration with two register sets as in the forward kernel; the set carried round the
    // loop starts as a zero increment (constants, not a load), and np is odd.
#pragma unroll
    for (int c = 0; c < DD; ++c) zz[c] = zzn[c] = 0.0;
#pragma unroll
    for (int s = 0; s < S; ++s) zc[s] = 0.0;
#pragma unroll
    for (int r = 0; r < QA; ++r) zuR[r] = 0.0;
    long rowA = -1;
    for (long row = a.np - 1; row >= 0; row -= 2) {
        // `row` is even (np is odd): the lead half moves; the set carried round the loop holds odd rows
        fetch(row, zzn, zcn, zuRn);
        segment(std::integral_constant<int, LEADLAG ? 2 : 0>(), rowA, zz, zc, zuR);
        fetch(row > 0 ? row - 1 : 0, zz, zc, zuR);
        segment(std::integral_constant<int, LEADLAG ? 1 : 0>(), row, zzn, zcn, zuRn);
        rowA = row - 1;
    }
    if constexpr (kRows) {
        double zb0[DD], zb1[S], zb2[QA];
#pragma unroll
        for (int c = 0; c < DD; ++c) zb0[c] = 0.0;
#pragma unroll
        for (int s = 0; s < S; ++s) zb1[s] = 0.0;
#pragma unroll
        for (int r = 0; r < QA; ++r) zb2[r] = 0.0;
        if constexpr (SHARED) {
            reduce_step_shared(-1, zb0, zb1, zb2);
        } else {
            reduce_step(-1, zb0, zb1, zb2);
            reduce_step(-1, zb0, zb1, zb2);
        }
    }
}

template <int DT, int M, int S, int QC, bool SHARED, bool LEADLAG>
__global__ __launch_bounds__(kWave * kWavesPerWG) void horner_bwd_kernel(const BwdArgs a)
{
    extern __shared__ double lds[];
    run_bwd<DT, M, S, QC, SHARED, LEADLAG>(a, lds);
}

// dF/dx from dF/dz (one row per segment of the transformed path): a point gains what the segment before it gives and
// loses what the segment after it gives.  Lead-lag: segment 2k moves the lead half by x[k+1] - x[k], segment 2k + 1
// the lag half by the same difference.  The time channel has no gradient.
template <typename TO>
__global__ __launch_bounds__(256) void point_gradients_kernel(const double* __restrict__ gz, TO* __restrict__ gx, long B,
                                                              long L, int d, int Dpad, int P, long Lc, long np,
                                                              int lead_lag)
{
    const long total = B * L * d;
    for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long)gridDim.x * blockDim.x) {
        const int ch = (int)(i % d);
        const long bp = i / d;
        const long pt = bp % L;
        const long b = bp / L;
        const double* g = gz + b * P * np * Dpad;
        // row of segment s of the transformed path: piece s / Lc, row s % Lc of that piece
        auto row = [&](long s, int c) { return g[((s / Lc) * np + s % Lc) * Dpad + c]; };
        auto seg = [&](long k) { return lead_lag ? row(2 * k, ch) + row(2 * k + 1, d + ch) : row(k, ch); };
        double v = 0.0;
        if (pt > 0) v += seg(pt - 1);
        if (pt < L - 1) v -= seg(pt);
        gx[i] = (TO)v;
    }
}

// Adjoint of chen_pairs_kernel (the product X = Xl (x) Xr of two neighbouring pieces, truncated at level N): from the
// adjoint Gp of X, the adjoint of Xl is Gl[w] = sum_c Gp[w c] Xr[c] and that of Xr is Gr[w] = sum_a Xl[a] Gp[a w], over
// all words c, a with |w| + |c| <= N.  X holds 2 * pairs signatures (Xl, Xr interleaved), Gc receives their adjoints
// in the same order.  The entries of levels k_lo..k_hi are computed by one lane each (lanes == 1) or by one wave each,
// its lanes striding over the terms (lanes == 64): short words have sums of up to the whole signature.
struct LevelTable {
    unsigned lv[24];    // start of level k in a flattened signature
    unsigned pw[24];    // D^k
};

__global__ __launch_bounds__(256) void chen_pairs_adjoint_kernel(const double* __restrict__ X, const double* __restrict__ Gp,
                                                                 double* __restrict__ Gc, long pairs, const LevelTable T,
                                                                 int N, long sig_len, int k_lo, int k_hi, int lanes)
{
    // blockIdx.y walks over the child signatures (2 * pair + child), blockIdx.x and the threads over the entries
    const unsigned e_lo = T.lv[k_lo], e_hi = T.lv[k_hi + 1];      // entries [e_lo, e_hi)
    const unsigned lane = lanes == 1 ? 0u : (threadIdx.x & 63u);
    const unsigned slot = blockIdx.x * blockDim.x + threadIdx.x;
    const unsigned e = e_lo + (lanes == 1 ? slot : slot / 64u);
    if (e >= e_hi) return;                             // whole waves leave together in the wave-per-entry form
    int k = k_lo;
    while (e >= T.lv[k + 1]) ++k;
    const unsigned w = e - T.lv[k];
    for (long sg = blockIdx.y; sg < 2 * pairs; sg += gridDim.y) {
        const long pr = sg >> 1;
        const int child = (int)(sg & 1);
        const double* Gpar = Gp + pr * sig_len;
        const double* Xo = X + (2 * pr + (child ^ 1)) * sig_len;      // the sibling
        double acc = 0.0;
        if (k > 0) {
            for (int j = 0; j <= N - k; ++j) {                         // the other word o has j letters
                const unsigned cnt = T.pw[j];
                const double* xo = Xo + T.lv[j];
                if (child == 0) {                                      // left factor: the word w o
                    const double* g = Gpar + T.lv[k + j] + w * cnt;
                    for (unsigned o = lane; o < cnt; o += (unsigned)lanes) acc = __builtin_fma(g[o], xo[o], acc);
                } else {                                               // right factor: the word o w
                    const double* g = Gpar + T.lv[k + j] + w;
                    const unsigned st = T.pw[k];
                    for (unsigned o = lane; o < cnt; o += (unsigned)lanes) acc = __builtin_fma(g[o * st], xo[o], acc);
                }
            }
        }
        if (lanes != 1) {
#pragma unroll
            for (int sh = 32; sh >= 1; sh >>= 1) acc += __shfl_xor(acc, sh, 64);
        }
        if (lane == 0) Gc[sg * sig_len + e] = acc;
    }
}

template <int DT, int M, int S, int QC, bool SHARED>
hipError_t launch_one(const BwdArgs& a, long grid, size_t lds_bytes, hipStream_t st)
{
    if constexpr (DT >= 4 && M >= 1) {
        if (a.leadlag) {
            hipLaunchKernelGGL((horner_bwd_kernel<DT, M, S, QC, SHARED, true>), dim3((unsigned)grid), dim3(kWave * kWavesPerWG),
                               lds_bytes, st, a);
            return hipGetLastError();
        }
    }
    hipLaunchKernelGGL((horner_bwd_kernel<DT, M, S, QC, SHARED, false>), dim3((unsigned)grid), dim3(kWave * kWavesPerWG),
                       lds_bytes, st, a);
    return hipGetLastError();
}

template <int DT, int M, int S>
hipError_t launch_variant(const BwdArgs& a, long grid, size_t lds_bytes, hipStream_t st)
{
    if (a.PW > 1) {
        if constexpr (DT > 0 && M > 0 && DT <= kSharedMaxD) {
            switch (a.Q) {
            case 0: return launch_one<DT, M, S, 0, true>(a, grid, lds_bytes, st);
            case 1: return launch_one<DT, M, S, 1, true>(a, grid, lds_bytes, st);
            case 2: return launch_one<DT, M, S, 2, true>(a, grid, lds_bytes, st);
            default: return hipErrorInvalidValue;
            }
        } else {
            return hipErrorInvalidValue;
        }
    }
    switch (a.Q) {
    case 0: return launch_one<DT, M, S, 0, false>(a, grid, lds_bytes, st);
    case 1: return launch_one<DT, M, S, 1, false>(a, grid, lds_bytes, st);
    case 2: return launch_one<DT, M, S, 2, false>(a, grid, lds_bytes, st);
    case 3: return launch_one<DT, M, S, 3, false>(a, grid, lds_bytes, st);
    case 4: return launch_one<DT, M, S, 4, false>(a, grid, lds_bytes, st);
    default:
        if constexpr (DT <= kBwdLongPrefixMaxD) return launch_one<DT, M, S, kQMax, false>(a, grid, lds_bytes, st);
        else return hipErrorInvalidValue;
    }
}

}  // namespace

hipError_t launch_horner_bwd(int DT, int M, int S, const BwdArgs& a, long grid, size_t lds_bytes, hipStream_t st)
{
    if (grid <= 0) return hipSuccess;
    const int D = DT ? DT : a.D;
    const bool uniform = DT > 0 && M > 0;
    const size_t need = (size_t)kWavesPerWG * a.lds_wave * sizeof(double);
    if ((a.np > 0 && !(a.np & 1)) || a.np < a.n || a.Q < 0 || a.Q > kQMax || a.LP <= 0 || a.WP * kWave < a.LP ||
        a.NB * (long)S < D || a.Dpad < D || a.lds_wave < (size_t)a.Dpad + (uniform ? (size_t)kWave * (D | 1) : 0) ||
        lds_bytes < need || lds_bytes > 64 * 1024)
        return hipErrorInvalidValue;
    if (a.PW < 1 || (a.PW > 1 && (a.WP != 1 || a.PW * a.LP > kWave || a.NW * a.PW < a.B)) || (a.PW == 1 && a.NW != a.B * a.WP) ||
        grid * kWavesPerWG < a.NW)
        return hipErrorInvalidValue;
    if (a.leadlag && (a.n & 1)) return hipErrorInvalidValue;      // pieces of a lead-lag path start with a lead move
    if (DT == 0) return (M == 0 && S == 1) ? launch_variant<0, 0, 1>(a, grid, lds_bytes, st) : hipErrorInvalidValue;
#define SG_CASE(D_, M_, S_) \
    if (DT == D_ && M == M_ && S == S_) return launch_variant<D_, M_, S_>(a, grid, lds_bytes, st);
    SG_BWD_VARIANTS(SG_CASE)
#undef SG_CASE
    return hipErrorInvalidValue;
}

template <typename TO>
hipError_t launch_point_gradients(const double* gz, TO* gx, long B, long L, int d, int Dpad, int P, long Lc, long np,
                                  int lead_lag, hipStream_t st)
{
    const long total = B * L * d;
    if (total <= 0) return hipSuccess;
    if (P < 1 || (Lc < 1 && L > 1) || np < Lc) return hipErrorInvalidValue;
    long grid = (total + 255) / 256;
    if (grid > 65536) grid = 65536;
    hipLaunchKernelGGL((point_gradients_kernel<TO>), dim3((unsigned)grid), dim3(256), 0, st, gz, gx, B, L, d, Dpad, P, Lc,
                       np, lead_lag);
    return hipGetLastError();
}

template hipError_t launch_point_gradients<float>(const double*, float*, long, long, int, int, int, long, long, int, hipStream_t);
template hipError_t launch_point_gradients<double>(const double*, double*, long, long, int, int, int, long, long, int, hipStream_t);

hipError_t launch_chen_pairs_adjoint(const double* X, const double* Gp, double* Gc, long pairs, int D, int N, long sig_len,
                                     hipStream_t st)
{
    if (pairs <= 0 || sig_len <= 0) return hipSuccess;
    if (sig_len >= (1L << 31) || D < 1 || N < 1 || N > 21) return hipErrorInvalidValue;
    // levels whose sums have more than 64 terms get a wave per entry: words of length k with 1 + D + ... + D^(N-k) > 64
    int k_split = 0;         // first level computed by single lanes
    {
        long terms = 0, pw = 1;
        int j = 0;
        while (j <= N && terms + pw <= 64) {
            terms += pw;
            pw *= D;
            ++j;
        }
        k_split = N - j + 1;           // levels k >= k_split have at most 64 terms
        if (k_split < 0) k_split = 0;
    }
    LevelTable T;
    {
        unsigned o = 0, q = 1;
        for (int k = 0; k < 24; ++k) {
            T.lv[k] = o;
            T.pw[k] = q;
            if (k <= N) {
                o += q;
                q *= (unsigned)D;
            }
        }
    }
    const unsigned gy = (unsigned)(2 * pairs < 65535 ? 2 * pairs : 65535);
    if (k_split <= N) {
        const long entries = (long)T.lv[N + 1] - (long)T.lv[k_split];
        hipLaunchKernelGGL(chen_pairs_adjoint_kernel, dim3((unsigned)((entries + 255) / 256), gy), dim3(256), 0, st, X, Gp, Gc,
                           pairs, T, N, sig_len, k_split, N, 1);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    if (k_split > 0) {
        const long entries = (long)T.lv[k_split];
        hipLaunchKernelGGL(chen_pairs_adjoint_kernel, dim3((unsigned)((entries + 3) / 4), gy), dim3(256), 0, st, X, Gp, Gc,
                           pairs, T, N, sig_len, 0, k_split - 1, 64);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace sg

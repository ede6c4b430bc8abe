// Solo sweeps (gfx950): one wavefront per path pair, for launches with enough pairs to fill the chip (the
// Gram matrices) whose block rows fit one strip of 64 M lanes-rows.  The wavefront does everything itself,
// with the per-lane building blocks of sk_lane.h:
//
//  * M block rows per lane, so a pair of up to 64 M block rows is a single strip: no hand-over rows, and the
//    pipeline skew of 63 macro-steps is paid once per pair instead of once per 64 block rows;
//  * no lane is ever masked (a lane whose column is outside the grid works with p = 0, A = B = 1), and
//    the macro-steps whose 64 columns all lie inside the grid run without clamping or selects;
//  * pairs are handed to the waves in y-major order: a wave works through a contiguous run of the pair
//    sequence, so in a Gram matrix consecutive pairs share the y path, which then stays in LDS together
//    with its gradient accumulator (one flush per run instead of one per pair).
//
// Backward (Section 3.4): forward sweep with a checkpoint of the lane state every 8 macro-steps and the
// pair's bottom row kept in LDS, then the mirrored reverse sweep that recovers the forward values by
// inverting Eq. (1) between checkpoints (see sk_lane.h), with the same drift guard as the other kernels:
// a recovered state that differs from the exact checkpoint (at the left end: from the boundary value 1) by more
// than kDriftTol of the lane's largest forward value disqualifies the pair: nothing of it reaches the gradient
// sums (the y side is collected per pair and merged into the run's sums only when the pair has passed), and
// the pair is listed for the replay kernel, which solves it once more.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "sk_dev.h"
#include "sk_kernels.h"
#include "sk_lane.h"

namespace sk {

// ------------------------------------------------------------------------------------------------
// forward
// ------------------------------------------------------------------------------------------------
template <int BL, int D, int M, int LL>
__global__ __launch_bounds__(kWavesPerWG* kWave, (D * M > 16) ? 2 : 3) void solo_fwd_kernel(SweepArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    using LK = Lock<BL, D, M, LL>;
    constexpr int C = LK::C;
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const long slot = (long)blockIdx.x * kWavesPerWG + w;
    const long nslots = (long)gridDim.x * kWavesPerWG;
    SK_LDS real* ylds = (SK_LDS real*)(smem + (size_t)w * a.lds_wave);
    const long q0 = slot * a.npairs / nslots, q1 = (slot + 1) * a.npairs / nslots;
    const int nb = a.nb;
    const int NT = nb + kWave - 1;
    long cur_y = -1;

    typename LK::Coef cf;
    typename LK::Fwd f;
    for (long q = q0; q < q1; ++q) {
        long xi, yi, pid, pid2;
        gram_pair(a, q, xi, yi, pid, pid2);
        if (yi != cur_y) {
            const real* dyg = a.dy + yi * a.ystride;
            for (int t = lane; t < a.q * LK::DSc; t += kWave) ylds[t] = dyg[t];
            cur_y = yi;
        }
        cf.setup(a, 0, lane, a.dx + xi * a.xstride, ylds);
        f.init();

        auto step = [&](auto edge_c, int J, const real (&y)[D]) {
            constexpr bool EDGE = decltype(edge_c)::value;
            real Ac[M], Bc[M], A0[M], B0[M];
#pragma unroll
            for (int m = 0; m < M; ++m) {
                LK::coef_fwd(cf.template inner<EDGE>(m, J, y), Ac[m], Bc[m]);
                if constexpr (LL == 1) LK::coef_fwd(cf.template inner_off<EDGE>(m, J), A0[m], B0[m]);
                else { A0[m] = Ac[m]; B0[m] = Bc[m]; }
            }
            real recv[C];
#pragma unroll
            for (int cc = 0; cc < C; ++cc) recv[cc] = wave_from_above_or(f.bot[cc], 1.0);
            f.step(recv, Ac, Bc, A0, B0);
        };
        // macro-steps [T0, T1), the y increments fetched one step ahead
        auto run = [&](auto edge_c, int T0, int T1) {
            constexpr bool EDGE = decltype(edge_c)::value;
            if (T0 >= T1) return;
            int Ja, Jb, ba, bb;
            real ya[D], yb[D];
            cf.template fetch<EDGE>(T0, Ja, ba, ya);
            int T = T0;
            for (; T + 2 <= T1; T += 2) {
                cf.template fetch<EDGE>(T + 1, Jb, bb, yb);
                step(edge_c, Ja, ya);
                cf.template fetch<EDGE>(T + 2 < T1 ? T + 2 : T + 1, Ja, ba, ya);
                step(edge_c, Jb, yb);
            }
            if (T < T1) step(edge_c, Ja, ya);
        };
        const int Ti = nb > kWave - 1 ? kWave - 1 : NT;   // end of the leading edge range
        run(std::true_type(), 0, Ti);
        if (nb > kWave - 1) {
            run(std::false_type(), kWave - 1, nb);
            run(std::true_type(), nb, NT);
        }
        if (lane == kWave - 1) {
            a.k_out[pid] = f.bot[C - 1];
            if (pid2 != pid) a.k_out[pid2] = f.bot[C - 1];
        }
    }
}

// ------------------------------------------------------------------------------------------------
// backward
// ------------------------------------------------------------------------------------------------
// (second launch bound: wavefronts per SIMD the register allocation has to leave room for)
// PHASE 0: the whole backward pass.  PHASE 1 / 2: its two halves as launches of their own, for a forward call that
// keeps its sweep and the backward call that takes it over: checkpoints and bottom row then have a place per pair in
// global memory (phase 1 copies the row out of LDS, phase 2 copies it in) instead of one per wave.
// OCC: wavefronts per SIMD the registers are allotted for.  A kernel that could share a SIMD is also built for one
// wave: where the y copy and the sums of a workgroup take more than half of LDS it runs alone whatever its registers,
// and held to 256 of them the kernels with many channels or two block rows per lane spill their lane state.
template <int BL, int D, int M, int PHASE, int LL, int OCC>
__global__ __launch_bounds__(kWavesPerWG* kWave, OCC) void solo_bwd_kernel(SweepArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    using LK = Lock<BL, D, M, LL>;
    constexpr int C = LK::C, RR = LK::RR, NVC = LK::NVC, S = kLockS;
    constexpr int NVS = RR + 1 + C;
    // the macro-steps of a segment are unrolled in pairs (the y buffers alternate) when a lane holds many channels:
    // a full unroll keeps too much alive
    constexpr int kUnroll = D * M > 16 ? 2 : S;
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const long slot = (long)blockIdx.x * kWavesPerWG + w;
    const long nslots = (long)gridDim.x * kWavesPerWG;
    unsigned char* mylds = smem + (size_t)w * a.lds_wave;
    SK_LDS real* ylds = (SK_LDS real*)mylds;
    SK_LDS real* gyl = (SK_LDS real*)(mylds + a.lk_off_gy);    // y-side sums of the run of pairs
    SK_LDS real* gyp = (SK_LDS real*)(mylds + a.lk_off_gyp);   // ... of the pair in work
    SK_LDS real* krow = (SK_LDS real*)(mylds + a.lk_off_krows) + LK::PADF;   // bottom row, by node column
    SK_LDS real* dump = (SK_LDS real*)(mylds + a.lk_off_dump);
    real* ckpt = a.ckpt + slot * a.ckpt_slot + lane;   // PHASE != 0: set per pair below
    const int klen = kWave * C + a.lk_NT * C + 2;      // the bottom row's place in LDS, from krow - PADF
    const long q0 = slot * a.npairs / nslots, q1 = (slot + 1) * a.npairs / nslots;
    const int nb = a.nb;
    const int NT = a.lk_NT;           // macro-steps, a multiple of S
    const int nseg = NT / S;
    const int ny = a.q * LK::DSc;
    const bool plain = a.rs2 == 0;    // 64 lanes at 64 different y rows: plain read-modify-write is safe
    long cur_y = -1;
    real* gdy_cur = nullptr;

    for (int t = lane; t < ny; t += kWave) gyp[t] = 0.0;
    typename LK::Coef cf;
    auto flush_gy = [&]() {
        if (gdy_cur && a.want_gy) {
            for (int t = lane; t < ny; t += kWave) {
                const real v = gyl[t];
                if (v != 0.0) unsafeAtomicAdd(&gdy_cur[t], v);
            }
        }
    };

    for (long q = q0; q < q1; ++q) {
        long xi, yi, pid, pid2;
        gram_pair(a, q, xi, yi, pid, pid2);
        if (yi != cur_y) {
            flush_gy();
            const real* dyg = a.dy + yi * a.ystride;
            for (int t = lane; t < ny; t += kWave) { ylds[t] = dyg[t]; gyl[t] = 0.0; }
            cur_y = yi;
            gdy_cur = a.gdy + yi * a.ystride;
        }
        cf.setup(a, 0, lane, a.dx + xi * a.xstride, ylds);
        const real gk = PHASE == 1 ? 0.0 : gram_weight(a, pid, pid2);
        real* keepq = nullptr;
        if constexpr (PHASE != 0) {
            ckpt = a.ckpt + q * a.ckpt_slot + lane;
            keepq = a.lk_keep + q * a.keep_len;
        }
        if constexpr (PHASE == 2) {
            for (int t = lane; t < klen; t += kWave) krow[t - LK::PADF] = keepq[t];
        }

        // ---- phase 1: forward, a checkpoint every S macro-steps, the bottom row into LDS ----
        if constexpr (PHASE != 2) {
            typename LK::Fwd f;
            f.init();
            for (int t = lane; t < LK::PADF + 1; t += kWave) krow[t - LK::PADF] = 1.0;   // columns left of the grid
            // every lane stores its bottom edge, the last lane into the row, the others into a dump that nobody reads:
            // [c][lane], so that the 64 stores of an instruction are 8 bytes apart (16 apart they collide in pairs)
            SK_LDS real* const op0 = lane == kWave - 1 ? krow + (0 - (kWave - 1)) * C + 1 : dump + lane;
            const int ostep = lane == kWave - 1 ? C : 0;
            const int cstep = lane == kWave - 1 ? 1 : kWave;
            auto seg = [&](auto edge_c, int T0) {
                constexpr bool EDGE = decltype(edge_c)::value;
                SK_LDS real* op = op0 + T0 * ostep;
                int J[2], b[2];
                real y[2][D];
                cf.template fetch<EDGE>(T0, J[0], b[0], y[0]);
#pragma unroll kUnroll
                for (int i = 0; i < S; ++i) {
                    if (i + 1 < S) cf.template fetch<EDGE>(T0 + i + 1, J[(i + 1) & 1], b[(i + 1) & 1], y[(i + 1) & 1]);
                    real Ac[M], Bc[M], A0[M], B0[M];
#pragma unroll
                    for (int m = 0; m < M; ++m) {
                        LK::coef_fwd(cf.template inner<EDGE>(m, J[i & 1], y[i & 1]), Ac[m], Bc[m]);
                        if constexpr (LL == 1) LK::coef_fwd(cf.template inner_off<EDGE>(m, J[i & 1]), A0[m], B0[m]);
                        else { A0[m] = Ac[m]; B0[m] = Bc[m]; }
                    }
                    real recv[C];
#pragma unroll
                    for (int cc = 0; cc < C; ++cc) recv[cc] = wave_from_above_or(f.bot[cc], 1.0);
                    f.step(recv, Ac, Bc, A0, B0);
#pragma unroll
                    for (int cc = 0; cc < C; ++cc) op[i * ostep + cc * cstep] = f.bot[cc];
                }
            };
            for (int g = 0; g < nseg; ++g) {
                f.store_ckpt(ckpt + (long)g * NVC * kWave);
                if (cf.interior(g * S, S)) seg(std::false_type(), g * S);
                else seg(std::true_type(), g * S);
            }
            f.store_ckpt(ckpt + (long)nseg * NVC * kWave);
        }
        if (a.k_out && lane == 0) {
            a.k_out[pid] = krow[nb * C];
            if (pid2 != pid) a.k_out[pid2] = krow[nb * C];
        }
        if constexpr (PHASE == 1) {
            for (int t = lane; t < klen; t += kWave) keepq[t] = krow[t - LK::PADF];
            continue;
        }
        scratch_fence();   // the checkpoints are read back below

        // ---- phase 2: the mirror image ----
        {
            typename LK::Rev rv;
            rv.init();
            real gacc[M][D];
#pragma unroll
            for (int m = 0; m < M; ++m)
#pragma unroll
                for (int c = 0; c < D; ++c) gacc[m][c] = 0.0;
            real kscale = 1.0;
            bool drift = false;
            const int up1 = lane > 0 ? -1 : 0;   // the bottom edge of the lane above travels with this lane's top edge
            real cpn[NVS];
            auto load_ckpt = [&](int idx) {
                const real* cp = ckpt + (long)idx * NVC * kWave;
#pragma unroll
                for (int i = 0; i <= RR; ++i) cpn[i] = ld_scratch(cp + i * kWave);
                cpn[RR + 1] = ld_scratch(cp + (RR + 1 + C) * kWave + up1);
#pragma unroll
                for (int i = 1; i < C; ++i) cpn[RR + 1 + i] = ld_scratch(cp + (RR + 1 + i - 1) * kWave + up1);
            };
            const int Tseed = nb - 1 + kWave - 1;   // macro-step in which the last lane is at the last column
            auto seg = [&](auto edge_c, int T0) {
                constexpr bool EDGE = decltype(edge_c)::value;
                const SK_LDS real* kp = krow + (T0 - (kWave - 1)) * C;
                int J[2], b[2];
                real y[2][D];
                cf.template fetch<EDGE>(T0 + S - 1, J[(S - 1) & 1], b[(S - 1) & 1], y[(S - 1) & 1]);
#pragma unroll kUnroll
                for (int i = S - 1; i >= 0; --i) {
                    if (i >= 1) cf.template fetch<EDGE>(T0 + i - 1, J[(i - 1) & 1], b[(i - 1) & 1], y[(i - 1) & 1]);
                    real Ac[M], Bc[M], iB[M], p6[M], A0[M], B0[M], iB0[M], accP[M];
#pragma unroll
                    for (int m = 0; m < M; ++m) {
                        const real p = cf.template inner<EDGE>(m, J[i & 1], y[i & 1]);
                        LK::coef_rev(p, Ac[m], Bc[m], iB[m]);
                        p6[m] = p * (1.0 / 6.0);
                        if constexpr (LL == 1) LK::coef_rev(cf.template inner_off<EDGE>(m, J[i & 1]), A0[m], B0[m], iB0[m]);
                        else { A0[m] = Ac[m]; B0[m] = Bc[m]; iB0[m] = iB[m]; }
                    }
                    // dF/dk[m, n] enters under the last lane at the last column
                    const real seed = (T0 + i == Tseed) ? gk : 0.0;
                    real recv[C], recvk[C];
#pragma unroll
                    for (int cc = 0; cc < C; ++cc) {
                        recv[cc] = wave_from_below_or(rv.up[cc], cc == C - 1 ? seed : 0.0);
                        recvk[cc] = wave_from_below_or(rv.ktop[cc], kp[i * C + cc]);
                    }
                    rv.step(recv, recvk, Ac, Bc, iB, p6, A0, B0, iB0, accP);
                    // the linear map of Section 3.4 (lead-lag: blocks off the diagonal of that level have no increment)
                    real gp[M];
#pragma unroll
                    for (int m = 0; m < M; ++m)
                        gp[m] = ((!EDGE || (unsigned)J[i & 1] < (unsigned)cf.nbl[m]) && !cf.off_block(m, J[i & 1])) ? accP[m] : 0.0;
                    // (both sides are always formed: a call that wants one gradient only is rare, and two uniform
                    // branches per macro-step cost every call; the flushes below look at what is wanted)
#pragma unroll
                    for (int m = 0; m < M; ++m)
#pragma unroll
                        for (int c = 0; c < D; ++c) gacc[m][c] = fma(gp[m], y[i & 1][c], gacc[m][c]);
                    {
                        SK_LDS real* gq = gyp + __mul24(b[i & 1], LK::DSc);
                        real t[D];
#pragma unroll
                        for (int c = 0; c < D; ++c) {
                            real v = gp[0] * cf.dxr[0][c];
#pragma unroll
                            for (int m = 1; m < M; ++m) v = fma(gp[m], cf.dxr[m][c], v);
                            t[c] = v;
                        }
                        if (plain) {
                            if (!EDGE || (unsigned)J[i & 1] < (unsigned)nb) {
                                if constexpr (D <= 8) {
                                    real o[D];   // every read before the first write: one wait instead of one per channel
#pragma unroll
                                    for (int c = 0; c < D; ++c) o[c] = gq[c];
#pragma unroll
                                    for (int c = 0; c < D; ++c) gq[c] = o[c] + t[c];
                                } else {
                                    // (sixteen channels: the registers for that are not there, and spilling the lane
                                    // state costs a factor of four)
#pragma unroll
                                    for (int c = 0; c < D; ++c) gq[c] += t[c];
                                }
                            }
                        } else {
#pragma unroll
                            for (int c = 0; c < D; ++c) lds_atomic_add(gq + c, t[c]);
                        }
                    }
                }
            };
            load_ckpt(nseg);
            for (int g = nseg - 1; g >= 0; --g) {
#pragma unroll
                for (int i = 0; i <= RR; ++i) kscale = fmax(kscale, fabs(cpn[i]));
                if (g < nseg - 1) {
#pragma unroll
                    for (int i = 0; i <= RR; ++i)   // written so that a NaN counts as drift
                        if (!(fabs(rv.kR[i] - cpn[i]) <= kDriftTol * kscale)) drift = true;
                }
#pragma unroll
                for (int i = 0; i <= RR; ++i) rv.kR[i] = cpn[i];
#pragma unroll
                for (int i = 0; i < C; ++i) rv.ktop[i] = cpn[RR + 1 + i];
                if (g >= 1) load_ckpt(g);   // for the next segment (to the left)
                if (cf.interior(g * S, S)) seg(std::false_type(), g * S);
                else seg(std::true_type(), g * S);
            }
            // the left end: the sweep started from the boundary value 1 in every lane
#pragma unroll
            for (int i = 0; i <= RR; ++i)
                if (!(fabs(rv.kR[i] - 1.0) <= kDriftTol * kscale)) drift = true;
            if (__ballot(drift) == 0ull) {
                if (a.want_gx) {
#pragma unroll
                    for (int m = 0; m < M; ++m) {
                        const int I = lane * M + m - a.lk_padb;
                        if (I >= 0) {
                            real* gq = a.gdx + xi * a.xstride + (long)(I >> a.rs1) * LK::DSc;
#pragma unroll
                            for (int c = 0; c < D; ++c) unsafeAtomicAdd(gq + c, gacc[m][c] * a.sc);
                        }
                    }
                }
                for (int t = lane; t < ny; t += kWave) { gyl[t] += gyp[t]; gyp[t] = 0.0; }
            } else {
                // nothing of this pair is kept: the replay kernel solves it once more
                for (int t = lane; t < ny; t += kWave) gyp[t] = 0.0;
                if (lane == 0) list_drifted(a, pid, pid2);
            }
        }
        scratch_fence();   // the next pair overwrites the checkpoints
    }
    flush_gy();
}

// ------------------------------------------------------------------------------------------------
// launchers
// ------------------------------------------------------------------------------------------------
template <int BL, int D, int M, int LL>
static hipError_t launch_solo_fwd(const SweepArgs& a, int grid, size_t lds, hipStream_t st)
{
    if (hipError_t e = allow_full_lds(reinterpret_cast<const void*>(&solo_fwd_kernel<BL, D, M, LL>)); e != hipSuccess) return e;
    hipLaunchKernelGGL((solo_fwd_kernel<BL, D, M, LL>), dim3(grid), dim3(kWavesPerWG * kWave), lds, st, a);
    return hipGetLastError();
}

template <int BL, int D, int M, int PHASE, int LL, int OCC>
static hipError_t launch_solo_bwd_occ(const SweepArgs& a, int grid, size_t lds, hipStream_t st)
{
    if (hipError_t e = allow_full_lds(reinterpret_cast<const void*>(&solo_bwd_kernel<BL, D, M, PHASE, LL, OCC>)); e != hipSuccess) return e;
    hipLaunchKernelGGL((solo_bwd_kernel<BL, D, M, PHASE, LL, OCC>), dim3(grid), dim3(kWavesPerWG * kWave), lds, st, a);
    return hipGetLastError();
}

// (The launcher templates below have internal linkage: the two translation units define them differently.)
// This file is compiled twice (the kernels take minutes): sk_solo.hip holds the forward kernels and every backward
// kernel at the occupancy the launch plan allows it at most, sk_solo_one.hip (SK_SOLO_ONE) the one-wave builds of the
// backward kernels that could share a SIMD, for launches whose LDS leaves room for one workgroup per compute unit.
#ifdef SK_SOLO_ONE
#define SK_SOLO_ENTRY launch_sweep_solo_one
#else
#define SK_SOLO_ENTRY launch_sweep_solo
#endif

template <int BL, int D, int M, int PHASE, int LL>
static hipError_t launch_solo_bwd_phase(int DT, const SweepArgs& a, int grid, size_t lds, hipStream_t st)
{
    constexpr int occ = solo_bwd_waves_per_simd(BL, M, D);
#ifdef SK_SOLO_ONE
    if constexpr (occ >= 2) return launch_solo_bwd_occ<BL, D, M, PHASE, LL, 1>(a, grid, lds, st);
    else return hipErrorInvalidValue;
#else
    if constexpr (occ >= 2) {
        if (!solo_bwd_shares_simd(BL, M, D, lds)) return launch_sweep_solo_one(true, BL, DT, a, grid, lds, st);
    }
    return launch_solo_bwd_occ<BL, D, M, PHASE, LL, occ>(a, grid, lds, st);
#endif
}

template <int BL, int D, int M, int LL>
static hipError_t launch_solo_bwd(const SweepArgs& a, int grid, size_t lds, hipStream_t st)
{
    constexpr int DT = D;
    if (a.lk_phase == 0) return launch_solo_bwd_phase<BL, D, M, 0, LL>(DT, a, grid, lds, st);
    // the halves need the per-pair places of checkpoints and bottom rows
    if (!a.lk_keep || a.keep_len != (long)kWave * (1 << BL) + (long)a.lk_NT * (1 << BL) + 2) return hipErrorInvalidValue;
    if (a.lk_phase == 1) return launch_solo_bwd_phase<BL, D, M, 1, LL>(DT, a, grid, lds, st);
    if (a.lk_phase == 2) return launch_solo_bwd_phase<BL, D, M, 2, LL>(DT, a, grid, lds, st);
    return hipErrorInvalidValue;
}

template <int BL, int D, int LL>
static hipError_t launch_solo_m(bool backward, const SweepArgs& a, int grid, size_t lds, hipStream_t st)
{
    if (a.lk_M > solo_max_rows(backward, BL, D)) return hipErrorInvalidValue;
    if (backward) {
        if (a.lk_M == 1) return launch_solo_bwd<BL, D, 1, LL>(a, grid, lds, st);
        if constexpr (solo_max_rows(true, BL, D) >= 2) return launch_solo_bwd<BL, D, 2, LL>(a, grid, lds, st);
    } else {
#ifndef SK_SOLO_ONE
        if (a.lk_M == 1) return launch_solo_fwd<BL, D, 1, LL>(a, grid, lds, st);
        if constexpr (solo_max_rows(false, BL, D) >= 2) return launch_solo_fwd<BL, D, 2, LL>(a, grid, lds, st);
#endif
    }
    return hipErrorInvalidValue;
}

// lead-lag form of the sweep (SweepArgs::ll): inside the blocks (1) for blocks that hold every refined cell of a pair
// of increments, above them (2) otherwise
template <int BL, int D>
static hipError_t launch_solo_ll(bool backward, const SweepArgs& a, int grid, size_t lds, hipStream_t st)
{
    if (a.ll == 0) return launch_solo_m<BL, D, 0>(backward, a, grid, lds, st);
    if constexpr (BL >= 1) {
        if (a.ll == 1 && a.rs1 == 0 && a.rs2 == 0) return launch_solo_m<BL, D, 1>(backward, a, grid, lds, st);
    }
    if (a.ll == 2 && a.rs1 >= 1 && a.rs2 >= 1) return launch_solo_m<BL, D, 2>(backward, a, grid, lds, st);
    return hipErrorInvalidValue;
}

template <int BL>
static hipError_t launch_solo_bl(bool backward, int DT, const SweepArgs& a, int grid, size_t lds, hipStream_t st)
{
    switch (DT) {
#ifndef SK_ONLY_C2   /* development builds instantiate a single shape */
        case 2: return launch_solo_ll<BL, 2>(backward, a, grid, lds, st);
        case 4: return launch_solo_ll<BL, 4>(backward, a, grid, lds, st);
        case 5: return launch_solo_ll<BL, 5>(backward, a, grid, lds, st);
        case 6: return launch_solo_ll<BL, 6>(backward, a, grid, lds, st);
        case 8: return launch_solo_ll<BL, 8>(backward, a, grid, lds, st);
#endif
        case 3: return launch_solo_ll<BL, 3>(backward, a, grid, lds, st);
        case 16: return launch_solo_ll<BL, 16>(backward, a, grid, lds, st);
        default: return hipErrorInvalidValue;
    }
}

hipError_t SK_SOLO_ENTRY(bool backward, int BL, int DT, const SweepArgs& a, int grid, size_t lds, hipStream_t st)
{
    if (a.lk_M < 1 || (backward && ((a.lk_NT % kLockS) != 0 || !a.bad_list || !a.bad_count))) return hipErrorInvalidValue;
    switch (BL) {
        case 0: return launch_solo_bl<0>(backward, DT, a, grid, lds, st);
        case 1: return launch_solo_bl<1>(backward, DT, a, grid, lds, st);
#ifndef SK_ONLY_C2
        case 2: return launch_solo_bl<2>(backward, DT, a, grid, lds, st);
#endif
        default: return hipErrorInvalidValue;
    }
}

}  // namespace sk

// Tile sweeps (gfx950): one wavefront per path pair, for many pairs of short paths with many channels and no
// dyadic refinement (at most 64 x 64 cells per pair, 8 or 16 channels: the large Gram matrices).
//
// With d = 16 channels and one cell per block the contraction over the channels (Eq. (1), third line) is most
// of the arithmetic, and a lane that reads its column's y increments from LDS at every step of the skewed
// sweep is bound by LDS bandwidth (128 bytes per lane and step).  Here the contractions run on the matrix
// cores and the sweep only moves one number per cell:
//
//  * The increment Gram matrix of the pair, Delta[a, b] = <dx[a], dy[b]>, is formed as 4 x 4 tiles of
//    16 x 16 entries by v_mfma_f64_16x16x4_f64 (the operands live in registers in the instruction's own
//    layout; the y side stays there over a run of pairs that share the y path) and written once to a
//    64 x 64 array P in the wave's LDS.  It never goes to HBM.
//  * The forward sweep (Eq. (1)) walks the anti-diagonals as in the other kernels: lane = grid row, one
//    column per macro-step, the edge of the lane above by DPP; p is one LDS read per cell.
//  * The reverse sweep (Section 3.4) recovers the forward values by inverting Eq. (1) between checkpoints
//    (see sk_lane.h), and overwrites P in place with G = dF/dp of every cell.
//  * The linear map of Section 3.4, dF/d(dx) = G dy and dF/d(dy) = G^T dx, is again two sets of MFMA tiles
//    with G read from LDS as the A operand.  The y-side sums stay in the accumulator registers over the run
//    of pairs and are flushed once per run.
//
// P is addressed as P[(b + 1) * 66 + a] (a = lane-space row, b = column): the even column stride keeps the
// three access patterns (row-contiguous, skewed by the sweep, and transposed for G^T) at most two-way bank
// conflicted.  Columns -1 and nb hold zeros: a lane whose column T - lane is outside the grid is clamped
// onto them and works with p = 0, A = B = 1, which carries the boundary value 1 forward and a zero adjoint
// backward; no lane is ever masked.  The rows of a pair are aligned to the bottom of the wave (row a of the
// pair sits in lane a + 64 - mb), so the result leaves through lane 63.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "sk_dev.h"
#include "sk_kernels.h"
#include "sk_lane.h"

namespace sk {

typedef double real4 __attribute__((ext_vector_type(4)));

// Pair q of the launch's sequence: y-major in Gram mode (q = m N + n), the identity for pair batches.
__device__ __forceinline__ void tile_pair(const SweepArgs& a, long q, long& xi, long& yi, long& pid)
{
    if (a.gramM) {
        const long N = a.npairs / a.gramM;
        yi = q / N;
        xi = q - yi * N;
        pid = xi * a.gramM + yi;
    } else {
        xi = yi = pid = q;
    }
}

__device__ __forceinline__ int clamp_range(int J, int lo, int hi)
{
    int r;
    asm("v_med3_i32 %0, %1, %2, %3" : "=v"(r) : "v"(J), "v"(lo), "v"(hi));
    return r;
}

template <int KC>
struct Tile {
    static constexpr int D = 4 * KC;   // channels the operand registers hold

    // Operand layout of the increment Gram tiles: v[T][kc] = inc[16 T + lane % 16 - rowoff][4 kc + lane / 16]
    // (zero for rows above the grid).  A tile of Delta^T is sum_kc mfma(yb[J][kc], xb[I][kc]).
    static __device__ __forceinline__ void load_b(const real* inc, int DS, int rowoff, int lane, real (&v)[4][KC])
    {
        const int n16 = lane & 15, g16 = lane >> 4;
#pragma unroll
        for (int T = 0; T < 4; ++T) {
            const int row = 16 * T + n16 - rowoff;
            const real* rp = inc + (long)(row >= 0 ? row : 0) * DS + g16;
#pragma unroll
            for (int kc = 0; kc < KC; ++kc) v[T][kc] = row >= 0 ? rp[4 * kc] : 0.0;
        }
    }
    // Operand layout of the linear map: v[kk] = inc[4 kk + lane / 16 - rowoff][lane % 16] (B operand, the
    // contraction runs over the rows of the path, the 16 output columns are the channels).
    static __device__ __forceinline__ void load_c(const real* inc, int DS, int rowoff, int lane, real (&v)[16])
    {
        const int n16 = lane & 15, g16 = lane >> 4;
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            const int row = 4 * kk + g16 - rowoff;
            v[kk] = (row >= 0 && n16 < D) ? inc[(long)(row >= 0 ? row : 0) * DS + (n16 < D ? n16 : 0)] : 0.0;
        }
    }
    // Delta tiles into P.  Result register r of lane l of tile (J, I) is Delta[a = 16 I + l % 16][b = 16 J + l / 16 + 4 r].
    // The time channel adds its constant product inside the grid only.
    static __device__ __forceinline__ void gram_tiles(SK_LDS real* P, const real (&yb)[4][KC], const real (&xb)[4][KC],
                                                      int lane, int padb, int nb, real tc)
    {
        const int n16 = lane & 15, g16 = lane >> 4;
#pragma unroll
        for (int J = 0; J < 4; ++J) {
#pragma unroll
            for (int I = 0; I < 4; ++I) {
                real4 acc = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
                for (int kc = 0; kc < KC; ++kc)
                    acc = __builtin_amdgcn_mfma_f64_16x16x4f64(yb[J][kc], xb[I][kc], acc, 0, 0, 0);
                const int al = 16 * I + n16;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int b = 16 * J + g16 + 4 * r;
                    const real v = acc[r] + ((al >= padb && b < nb) ? tc : 0.0);
                    P[(b + 1) * kTileStride + al] = v;
                }
            }
        }
    }
    static __device__ __forceinline__ void coef_fwd(real p, real& Ac, real& Bc)
    {
        const real q2 = p * p;
        Bc = fma(q2, -1.0 / 12.0, 1.0);
        Ac = fma(p, 0.5, fma(q2, 1.0 / 12.0, 1.0));
    }
};

// ------------------------------------------------------------------------------------------------
// forward
// ------------------------------------------------------------------------------------------------
template <int KC>
__global__ __launch_bounds__(kWavesPerWG* kWave, 1) void tile_fwd_kernel(SweepArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    using TL = Tile<KC>;
    using LK = Lock<0, 4 * KC, 1>;
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const long slot = (long)blockIdx.x * kWavesPerWG + w;
    const long nslots = (long)gridDim.x * kWavesPerWG;
    SK_LDS real* P = (SK_LDS real*)(smem + (size_t)w * a.lds_wave);
    const long q0 = slot * a.npairs / nslots, q1 = (slot + 1) * a.npairs / nslots;
    const int nb = a.nb, padb = a.lk_padb;
    const int NT = nb + kWave - 1;
    const int pbase = kTileStride + lane;
    long cur_y = -1;
    real yb[4][KC];

    // guard columns -1 and 64
    P[lane] = 0.0;
    P[(kTileCols - 1) * kTileStride + lane] = 0.0;

    typename LK::Fwd f;
    for (long q = q0; q < q1; ++q) {
        long xi, yi, pid;
        tile_pair(a, q, xi, yi, pid);
        if (yi != cur_y) {
            TL::load_b(a.dy + yi * a.ystride, a.DS, 0, lane, yb);
            cur_y = yi;
        }
        real xb[4][KC];
        TL::load_b(a.dx + xi * a.xstride, a.DS, padb, lane, xb);
        TL::gram_tiles(P, yb, xb, lane, padb, nb, a.tc);

        f.init();
        auto readp = [&](int T) { return P[__mul24(clamp_range(T - lane, -1, nb), kTileStride) + pbase]; };
        real pn = readp(0);
#pragma unroll 2
        for (int T = 0; T < NT; ++T) {
            const real p = pn;
            pn = readp(T + 1);
            real Ac[1], Bc[1], recv[1];
            TL::coef_fwd(p, Ac[0], Bc[0]);
            recv[0] = wave_from_above_or(f.bot[0], 1.0);
            f.step(recv, Ac, Bc);
        }
        if (lane == kWave - 1) a.k_out[pid] = f.bot[0];
    }
}

// ------------------------------------------------------------------------------------------------
// backward
// ------------------------------------------------------------------------------------------------
template <int KC>
__global__ __launch_bounds__(kWavesPerWG* kWave, 1) void tile_bwd_kernel(SweepArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    using TL = Tile<KC>;
    using LK = Lock<0, 4 * KC, 1>;
    constexpr int C = 1, RR = 1, NVC = LK::NVC, S = kLockS;
    constexpr int NVS = RR + 1 + C;
    const int lane = threadIdx.x & 63;
    const int n16 = lane & 15, g16 = lane >> 4;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const long slot = (long)blockIdx.x * kWavesPerWG + w;
    const long nslots = (long)gridDim.x * kWavesPerWG;
    unsigned char* mylds = smem + (size_t)w * a.lds_wave;
    SK_LDS real* P = (SK_LDS real*)mylds;
    SK_LDS real* krow = (SK_LDS real*)(mylds + a.lk_off_krows) + LK::PADF;   // bottom row, by node column
    SK_LDS real* dump = (SK_LDS real*)(mylds + a.lk_off_dump);
    real* ckpt = a.ckpt + slot * a.ckpt_slot + lane;
    const long q0 = slot * a.npairs / nslots, q1 = (slot + 1) * a.npairs / nslots;
    const int nb = a.nb, padb = a.lk_padb;
    const int NT = a.lk_NT;           // macro-steps, a multiple of S
    const int nseg = NT / S;
    const int pbase = kTileStride + lane;
    long cur_y = -1;
    real* gdy_cur = nullptr;
    bool drift = false;

    P[lane] = 0.0;
    P[(kTileCols - 1) * kTileStride + lane] = 0.0;

    real yb[4][KC], yc[16];
    real4 gy[4];
    // y-side sums of the run: result register r of lane l of tile J is row b = 16 J + l / 16 + 4 r, channel l % 16
    auto flush_gy = [&]() {
        if (gdy_cur && a.want_gy) {
#pragma unroll
            for (int J = 0; J < 4; ++J)
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int b = 16 * J + g16 + 4 * r;
                    if (b < a.q && n16 < a.d) unsafeAtomicAdd(&gdy_cur[(long)b * a.DS + n16], gy[J][r]);
                }
        }
    };
    auto readp = [&](int T) { return P[__mul24(clamp_range(T - lane, -1, nb), kTileStride) + pbase]; };

    for (long q = q0; q < q1; ++q) {
        long xi, yi, pid;
        tile_pair(a, q, xi, yi, pid);
        if (yi != cur_y) {
            flush_gy();
            const real* dyg = a.dy + yi * a.ystride;
            TL::load_b(dyg, a.DS, 0, lane, yb);
            TL::load_c(dyg, a.DS, 0, lane, yc);
#pragma unroll
            for (int J = 0; J < 4; ++J) gy[J] = real4{0.0, 0.0, 0.0, 0.0};
            cur_y = yi;
            gdy_cur = a.gdy + yi * a.ystride;
        }
        const real* dxg = a.dx + xi * a.xstride;
        {
            real xb[4][KC];
            TL::load_b(dxg, a.DS, padb, lane, xb);
            TL::gram_tiles(P, yb, xb, lane, padb, nb, a.tc);
        }
        const real gk = a.grad_k[pid];

        // ---- phase 1: forward, a checkpoint every S macro-steps, the bottom row into LDS ----
        {
            typename LK::Fwd f;
            f.init();
            for (int t = lane; t < LK::PADF + 1; t += kWave) krow[t - LK::PADF] = 1.0;   // columns left of the grid
            SK_LDS real* const op0 = lane == kWave - 1 ? krow + (0 - (kWave - 1)) * C + 1 : dump + lane * C;
            const int ostep = lane == kWave - 1 ? C : 0;
            real pn = readp(0);
            for (int g = 0; g < nseg; ++g) {
                f.store_ckpt(ckpt + (long)g * NVC * kWave);
                SK_LDS real* op = op0 + g * S * ostep;
#pragma unroll
                for (int i = 0; i < S; ++i) {
                    const real p = pn;
                    pn = readp(g * S + i + 1);
                    real Ac[1], Bc[1], recv[1];
                    TL::coef_fwd(p, Ac[0], Bc[0]);
                    recv[0] = wave_from_above_or(f.bot[0], 1.0);
                    f.step(recv, Ac, Bc);
                    op[i * ostep] = f.bot[0];
                }
            }
            f.store_ckpt(ckpt + (long)nseg * NVC * kWave);
        }
        if (a.k_out && lane == 0) a.k_out[pid] = krow[nb * C];
        scratch_fence();   // the checkpoints are read back below

        // ---- phase 2: the mirror image; G = dF/dp replaces p in place ----
        {
            typename LK::Rev rv;
            rv.init();
            real kscale = 1.0;
            const int up1 = lane > 0 ? -1 : 0;   // the bottom edge of the lane above travels with this lane's top edge
            real cpn[NVS];
            auto load_ckpt = [&](int idx) {
                const real* cp = ckpt + (long)idx * NVC * kWave;
#pragma unroll
                for (int i = 0; i <= RR; ++i) cpn[i] = ld_scratch(cp + i * kWave);
                cpn[RR + 1] = ld_scratch(cp + (RR + 1 + C) * kWave + up1);
            };
            const int Tseed = nb - 1 + kWave - 1;   // macro-step in which the last lane is at the last column
            load_ckpt(nseg);
            for (int g = nseg - 1; g >= 0; --g) {
#pragma unroll
                for (int i = 0; i <= RR; ++i) kscale = fmax(kscale, fabs(cpn[i]));
                if (g < nseg - 1) {
#pragma unroll
                    for (int i = 0; i <= RR; ++i)   // written so that a NaN counts as drift
                        if (!(fabs(rv.kR[i] - cpn[i]) <= 1e-9 * kscale)) drift = true;
                }
#pragma unroll
                for (int i = 0; i <= RR; ++i) rv.kR[i] = cpn[i];
                rv.ktop[0] = cpn[RR + 1];
                if (g >= 1) load_ckpt(g);   // for the next segment (to the left)
                const int T0 = g * S;
                const SK_LDS real* kp = krow + (T0 - (kWave - 1)) * C;
                real pn = readp(T0 + S - 1);
#pragma unroll
                for (int i = S - 1; i >= 0; --i) {
                    const int J = T0 + i - lane;
                    const real p = pn;
                    if (i >= 1) pn = readp(T0 + i - 1);
                    real Ac[1], Bc[1], iB[1], p6[1], accP[1];
                    TL::coef_fwd(p, Ac[0], Bc[0]);
                    const real r = __builtin_amdgcn_rcp(Bc[0]);
                    iB[0] = fma(fma(-Bc[0], r, 1.0), r, r);
                    p6[0] = p * (1.0 / 6.0);
                    // dF/dk[m, n] enters under the last lane at the last column
                    const real seed = (T0 + i == Tseed) ? gk : 0.0;
                    real recv[1], recvk[1];
                    recv[0] = wave_from_below_or(rv.up[0], seed);
                    recvk[0] = wave_from_below_or(rv.ktop[0], kp[i * C]);
                    rv.step(recv, recvk, Ac, Bc, iB, p6, accP);
                    // outside the grid the zeros of the guard columns stay; to the left of the grid dF/dp is not
                    // zero (the adjoint has left the grid there) and must not be kept
                    if ((unsigned)J < (unsigned)nb) P[__mul24(J, kTileStride) + pbase] = accP[0];
                }
            }
        }

        // ---- the linear map of Section 3.4 on the matrix cores ----
        if (a.want_gx) {
            // dF/d(dx)[a, c] = sum_b G[a, b] dy[b, c]: A operand G[16 I + l % 16][4 kb + l / 16], B operand yc[kb]
            real* gq = a.gdx + xi * a.xstride;
#pragma unroll
            for (int I = 0; I < 4; ++I) {
                real4 acc = {0.0, 0.0, 0.0, 0.0};
                const SK_LDS real* gp = P + (g16 + 1) * kTileStride + 16 * I + n16;
#pragma unroll
                for (int kb = 0; kb < 16; ++kb)
                    acc = __builtin_amdgcn_mfma_f64_16x16x4f64(gp[4 * kb * kTileStride], yc[kb], acc, 0, 0, 0);
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int arow = 16 * I + g16 + 4 * r - padb;
                    if (arow >= 0 && n16 < a.d) unsafeAtomicAdd(&gq[(long)arow * a.DS + n16], acc[r]);
                }
            }
        }
        if (a.want_gy) {
            // dF/d(dy)[b, c] = sum_a G[a, b] dx[a, c]: A operand G[4 ka + l / 16][16 J + l % 16], B operand xc[ka]
            real xc[16];
            TL::load_c(dxg, a.DS, padb, lane, xc);
#pragma unroll
            for (int J = 0; J < 4; ++J) {
                const SK_LDS real* gp = P + (16 * J + n16 + 1) * kTileStride + g16;
#pragma unroll
                for (int ka = 0; ka < 16; ++ka)
                    gy[J] = __builtin_amdgcn_mfma_f64_16x16x4f64(gp[4 * ka], xc[ka], gy[J], 0, 0, 0);
            }
        }
        scratch_fence();   // the next pair overwrites the checkpoints
    }
    flush_gy();
    if (drift) atomicExch(a.err, 2);
}

// ------------------------------------------------------------------------------------------------
// launchers
// ------------------------------------------------------------------------------------------------
template <int KC>
hipError_t launch_tile_k(bool backward, const SweepArgs& a, int grid, size_t lds, hipStream_t st)
{
    static bool attr_done[2] = {false, false};
    const void* fn = backward ? reinterpret_cast<const void*>(&tile_bwd_kernel<KC>)
                              : reinterpret_cast<const void*>(&tile_fwd_kernel<KC>);
    if (!attr_done[backward]) {
        hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsPerCU);
        if (e != hipSuccess) return e;
        attr_done[backward] = true;
    }
    if (backward) hipLaunchKernelGGL((tile_bwd_kernel<KC>), dim3(grid), dim3(kWavesPerWG * kWave), lds, st, a);
    else hipLaunchKernelGGL((tile_fwd_kernel<KC>), dim3(grid), dim3(kWavesPerWG * kWave), lds, st, a);
    return hipGetLastError();
}

hipError_t launch_sweep_tile(bool backward, int DT, const SweepArgs& a, int grid, size_t lds, hipStream_t st)
{
    // what the kernels assume about the launch
    if (a.lk_M != 1 || a.rs1 != 0 || a.rs2 != 0 || a.mb > kWave || a.nb > kWave || a.mb < 1 || a.nb < 1 ||
        a.lk_padb != kWave - a.mb || a.rpad < kWave || a.qpad < kWave || a.DS <= DT || a.d > DT ||
        (backward && ((a.lk_NT % kLockS) != 0 || a.lk_NT < a.nb + kWave - 1)))
        return hipErrorInvalidValue;
    switch (DT) {
        case 8: return launch_tile_k<2>(backward, a, grid, lds, st);
        case 16: return launch_tile_k<4>(backward, a, grid, lds, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace sk

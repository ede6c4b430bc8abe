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
//    (see sk_lane.h), and overwrites P in place with 6 G, G = dF/dp of every cell (the factor goes into the map).
//  * The linear map of Section 3.4, dF/d(dx) = G dy and dF/d(dy) = G^T dx, is again two sets of MFMA tiles
//    with G read from LDS as the A operand.  The y-side sums stay in the accumulator registers over the run
//    of pairs and are flushed once per run.
//
// P is addressed as P[(b + 1) * 66 + a] (a = lane-space row, b = column): the even column stride keeps the
// three access patterns (row-contiguous, skewed by the sweep, and transposed for G^T) at most two-way bank
// conflicted.  Column nb holds zeros: a lane whose column J = T - lane is outside the grid on either side
// reads it (min of J as an unsigned number and nb) and works with p = 0, A = B = 1, which carries the
// boundary value 1 forward and a zero adjoint backward; no lane is ever masked.  Column -1 takes the dF/dp
// of lanes left of the grid, which nobody reads.  The rows of a pair are aligned to the bottom of the wave (row a of the
// pair sits in lane a + 64 - mb), so the result leaves through lane 63.
#include "sk_tile.h"

namespace sk {

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

    P[(kTileCols - 1) * kTileStride + lane] = 0.0;   // column 64: the zero column of a pair with 64 columns

    typename LK::Fwd f;
    for (long q = q0; q < q1; ++q) {
        long xi, yi, pid, pid2;
        gram_pair(a, q, xi, yi, pid, pid2);
        if (yi != cur_y) {
            TL::load_b(a.dy + yi * a.ystride, a.DS, 0, lane, yb);
            cur_y = yi;
        }
        real xb[4][KC];
        TL::load_b(a.dx + xi * a.xstride, a.DS, padb, lane, xb);
        if (a.tc != 0.0) TL::template gram_tiles<true>(P, yb, xb, lane, padb, nb, a.tc);
        else TL::template gram_tiles<false>(P, yb, xb, lane, padb, nb, 0.0);

        f.init();
        auto readp = [&](int J) { return P[__mul24(read_col(J, nb), kTileStride) + pbase]; };
        auto step = [&](real p) {
            real Ac[1], Bc[1], recv[1];
            TL::coef_fwd(p, Ac[0], Bc[0]);
            recv[0] = wave_from_above_or(f.bot[0], 1.0);
            f.step(recv, Ac, Bc);
        };
        real pq[kTilePF];
        int Jn = -lane;   // column of the next macro-step to fetch p for
#pragma unroll
        for (int i = 0; i < kTilePF; ++i) pq[i] = readp(Jn + i);
        Jn += kTilePF;
        int T0 = 0;
        for (; T0 + kTilePF <= NT; T0 += kTilePF, Jn += kTilePF) {
#pragma unroll
            for (int i = 0; i < kTilePF; ++i) {
                const real p = pq[i];
                pq[i] = readp(Jn + i);   // past the last step: the zero column, unused
                step(p);
            }
        }
#pragma unroll
        for (int i = 0; i < kTilePF; ++i)
            if (T0 + i < NT) step(pq[i]);
        if (lane == kWave - 1) {
            a.k_out[pid] = f.bot[0];
            if (pid2 != pid) a.k_out[pid2] = f.bot[0];
        }
    }
}

// ------------------------------------------------------------------------------------------------
// launchers
// ------------------------------------------------------------------------------------------------
template <int KC>
hipError_t launch_tile_fwd(const SweepArgs& a, int grid, size_t lds, hipStream_t st)
{
    if (hipError_t e = allow_full_lds(reinterpret_cast<const void*>(&tile_fwd_kernel<KC>)); e != hipSuccess) return e;
    hipLaunchKernelGGL((tile_fwd_kernel<KC>), dim3(grid), dim3(kWavesPerWG * kWave), lds, st, a);
    return hipGetLastError();
}

hipError_t launch_sweep_tile(bool backward, int DT, const SweepArgs& a, int grid, size_t lds, hipStream_t st)
{
    // what the kernels assume about the launch
    if (a.lk_M != 1 || a.rs1 != 0 || a.rs2 != 0 || a.mb > kWave || a.nb > kWave || a.mb < 1 || a.nb < 1 ||
        a.lk_padb != kWave - a.mb || a.lk_padb > kWave / 2 || a.rpad < kWave || a.qpad < kWave || a.DS <= DT || a.d > DT ||
        (backward && (!a.bad_list || !a.bad_count || (a.lk_NT % kLockS) != 0 || a.lk_NT < a.nb + kWave - 1 || a.lk_NT >= a.nb + kWave - 1 + kLockS ||
                      (size_t)a.lk_off_ck + (size_t)((a.lk_NT / kLockS - 1) / kTileCkChunks) * 2 * kWave * sizeof(real) >
                          a.lk_off_krows ||
                      (size_t)a.lk_off_krows + (size_t)(kTileRowPad + kWave + 8) * sizeof(real) > a.lds_wave)))
        return hipErrorInvalidValue;
    if (backward) return launch_tile_bwd(DT, a, grid, st);
    switch (DT) {
        case 8: return launch_tile_fwd<2>(a, grid, lds, st);
        case 16: return launch_tile_fwd<4>(a, grid, lds, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace sk

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
// conflicted.  Column nb holds zeros: a lane whose column J = T - lane is outside the grid on either side
// reads it (min of J as an unsigned number and nb) and works with p = 0, A = B = 1, which carries the
// boundary value 1 forward and a zero adjoint backward; no lane is ever masked.  Column -1 takes the dF/dp
// of lanes left of the grid, which nobody reads.  The rows of a pair are aligned to the bottom of the wave (row a of the
// pair sits in lane a + 64 - mb), so the result leaves through lane 63.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "sk_dev.h"
#include "sk_kernels.h"
#include "sk_lane.h"

namespace sk {

typedef double real4 __attribute__((ext_vector_type(4)));

// Column a lane reads p from: J inside the grid, else the zero column nb (J < 0 is a huge unsigned number).
__device__ __forceinline__ int read_col(int J, int nb) { return (int)min((unsigned)J, (unsigned)nb); }
// Column a lane writes dF/dp to: J inside the grid, the zero column nb to its right (the value is zero
// there), the unread column -1 to its left.
__device__ __forceinline__ int write_col(int J, int nb)
{
    int r;
    asm("v_med3_i32 %0, %1, -1, %2" : "=v"(r) : "v"(J), "s"(nb));
    return r;
}

constexpr int kTilePF = 8;   // the sweeps read p this many macro-steps ahead (LDS latency off the serial chain)

template <int KC>
struct Tile {
    static constexpr int D = 4 * KC;   // channels the operand registers hold

    // Operand layout of the increment Gram tiles: v[T][kc] = inc[16 T + lane % 16 - rowoff][4 kc + lane / 16]
    // (zero for rows above the grid).  A tile of Delta^T is sum_kc mfma(yb[J][kc], xb[I][kc]).
    static __device__ __forceinline__ void load_b(const real* inc, int DS, int rowoff, int lane, real (&v)[4][KC])
    {
        int n16 = lane & 15;
        const int g16 = lane >> 4;
        asm volatile("" : "+v"(n16));   // addresses are formed per call, not kept alive as loop invariants
#pragma unroll
        for (int T = 0; T < 4; ++T) {
            const int row = 16 * T + n16 - rowoff;
            const real* rp = inc + (long)(row >= 0 ? row : 0) * DS + g16;
            real t[KC];
#pragma unroll
            for (int kc = 0; kc < KC; ++kc) t[kc] = rp[4 * kc];
#pragma unroll
            for (int kc = 0; kc < KC; ++kc) v[T][kc] = row >= 0 ? t[kc] : 0.0;
        }
    }
    // Operand layout of the linear map: v[kk] = inc[4 kk + lane / 16 - rowoff][lane % 16] (B operand, the
    // contraction runs over the rows of the path, the 16 output columns are the channels).
    static __device__ __forceinline__ void load_c(const real* inc, int DS, int rowoff, int lane, real (&v)[16])
    {
        const int n16 = lane & 15;
        int g16 = lane >> 4;
        asm volatile("" : "+v"(g16));   // addresses are formed per call, not kept alive as loop invariants
        const int ch = n16 < D ? n16 : 0;
        real t[16];
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            const int row = 4 * kk + g16 - rowoff;
            t[kk] = inc[(long)(row >= 0 ? row : 0) * DS + ch];
        }
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            const int row = 4 * kk + g16 - rowoff;
            v[kk] = (row >= 0 && n16 < D) ? t[kk] : 0.0;
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
        TL::gram_tiles(P, yb, xb, lane, padb, nb, a.tc);

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
// backward
// ------------------------------------------------------------------------------------------------
template <int KC>
__global__ __launch_bounds__(kWavesPerWG* kWave, 1) void tile_bwd_kernel(SweepArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    using TL = Tile<KC>;
    using LK = Lock<0, 4 * KC, 1>;
    constexpr int S = kLockS;          // macro-steps per unrolled chunk
    constexpr int CK = kTileCkChunks;  // chunks between checkpoints
    const int lane = threadIdx.x & 63;
    const int n16 = lane & 15, g16 = lane >> 4;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const long slot = (long)blockIdx.x * kWavesPerWG + w;
    const long nslots = (long)gridDim.x * kWavesPerWG;
    unsigned char* mylds = smem + (size_t)w * a.lds_wave;
    SK_LDS real* P = (SK_LDS real*)mylds;
    // Checkpoints of the forward sweep, in LDS: per lane the last two values of its row, k[a + 1][J] and
    // k[a + 1][J - 1] (J the column the lane is about to process); the row above is the neighbouring lane's.
    SK_LDS real* ckl = (SK_LDS real*)(mylds + a.lk_off_ck) + lane;
    // The bottom row of the pair (the last lane's outputs, which no lane recovers in the reverse sweep) sits
    // in the spare slot 64 of P's columns, by node column c = -1 .. 64 (every node left of the grid is 1).
    SK_LDS real* const krow = P + kTileStride + kWave;
    // Macro-steps run from 0 to NT - 1 with NT a multiple of S; the sweep proper ends at the last one (the last lane at
    // the last column), so that the reverse sweep starts with the seed in place, and begins tpad steps late.
    const int NT = a.lk_NT;
    const int tpad = NT - (a.nb + kWave - 1);   // 0 .. S - 1
    const long q0 = slot * a.npairs / nslots, q1 = (slot + 1) * a.npairs / nslots;
    const int nb = a.nb, padb = a.lk_padb;
    const int nch = NT / S;
    const int pbase = kTileStride + lane;
    const bool last = lane == kWave - 1;
    long cur_y = -1;
    real* gdy_cur = nullptr;

    P[(kTileCols - 1) * kTileStride + lane] = 0.0;   // column 64: the zero column of a pair with 64 columns
    if (last) krow[-kTileStride] = 1.0;              // node column -1 (stands for all nodes left of the grid)

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
    auto readp = [&](int J) { return P[__mul24(read_col(J, nb), kTileStride) + pbase]; };

    // Operands of the pair in work, loaded while the previous pair was in the linear map.
    real xb[4][KC];
    real gk = 0.0;
    if (q0 < q1) {
        long xi, yi, pid, pid2;
        gram_pair(a, q0, xi, yi, pid, pid2);
        TL::load_b(a.dx + xi * a.xstride, a.DS, padb, lane, xb);
        gk = gram_weight(a, pid, pid2);
    }
    for (long q = q0; q < q1; ++q) {
        long xi, yi, pid, pid2;
        gram_pair(a, q, xi, yi, pid, pid2);
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
        TL::gram_tiles(P, yb, xb, lane, padb, nb, a.tc);

        // ---- phase 1: forward; a checkpoint every CK chunks and the bottom row into LDS ----
        real kR0, kR1;   // exact state the reverse sweep starts from: k[a][J], k[a + 1][J]
        {
            typename LK::Fwd f;
            f.init();
            real pq[S];
            int Jn = -tpad - lane;   // column of the next macro-step to fetch p for
#pragma unroll
            for (int i = 0; i < S; ++i) pq[i] = readp(Jn + i);
            Jn += S;
            int cl = -tpad - (kWave - 1) + 1;   // node column the last lane writes in the chunk's first macro-step
            for (int g = 0; g < nch; ++g, Jn += S, cl += S) {
                if (g > 0 && g % CK == 0) {
                    SK_LDS real* cp = ckl + (g / CK - 1) * (2 * kWave);
                    cp[0] = f.left[1];
                    cp[kWave] = f.blc;
                }
                real kb[S];   // the lane's bottom values of the chunk; the last lane's are the pair's bottom row
#pragma unroll
                for (int i = 0; i < S; ++i) {
                    const real p = pq[i];
                    pq[i] = readp(Jn + i);   // past the last step: the zero column, unused
                    real Ac[1], Bc[1], recv[1];
                    TL::coef_fwd(p, Ac[0], Bc[0]);
                    recv[0] = wave_from_above_or(f.bot[0], 1.0);
                    f.step(recv, Ac, Bc);
                    kb[i] = f.bot[0];
                }
                if (last) {   // node columns left of the grid all go to the one slot that stands for them
                    if (cl >= -1) {
                        SK_LDS real* kp = krow + cl * kTileStride;
#pragma unroll
                        for (int i = 0; i < S; ++i) kp[i * kTileStride] = kb[i];
                    } else {
#pragma unroll
                        for (int i = 0; i < S; ++i) krow[(cl + i > -1 ? cl + i : -1) * kTileStride] = kb[i];
                    }
                }
            }
            kR0 = f.left[0];
            kR1 = f.left[1];
        }
        if (a.k_out && lane == 0) {
            a.k_out[pid] = krow[nb * kTileStride];
            if (pid2 != pid) a.k_out[pid2] = krow[nb * kTileStride];
        }

        // ---- phase 2: the mirror image; G = dF/dp replaces p in place ----
        bool drift = false;
        {
            typename LK::Rev rv;
            rv.init();
            // dF/dk[m, n] is the adjoint of the bottom right node of the last lane's first block in this direction
            if (last) rv.accL[1] = gk;
            rv.kR[0] = kR0;
            rv.kR[1] = kR1;
            rv.ktop[0] = kR0;
            real kscale = 1.0;
            // p of the macro-steps of a chunk is read one chunk ahead (P is overwritten with G behind the sweep
            // only: a lane writes column J after it has read columns J - S .. J)
            real pq[S], kq[S];
            int Jb = (nch - 1) * S - tpad - lane;   // column of this lane in the first macro-step of the chunk
#pragma unroll
            for (int i = 0; i < S; ++i) pq[i] = readp(Jb + i);
            int cl = (nch - 1) * S - tpad - (kWave - 1);   // node column under the last lane's block, first macro-step
            for (int g = nch - 1; g >= 0; --g, Jb -= S, cl -= S) {
                // the last lane's bottom edge, before any store of this chunk
                if (cl >= -1) {
                    const SK_LDS real* kp = krow + cl * kTileStride;
#pragma unroll
                    for (int i = 0; i < S; ++i) kq[i] = kp[i * kTileStride];
                } else {
#pragma unroll
                    for (int i = 0; i < S; ++i) kq[i] = krow[(cl + i > -1 ? cl + i : -1) * kTileStride];
                }
#pragma unroll
                for (int i = S - 1; i >= 0; --i) {
                    const int J = Jb + i;
                    const real p = pq[i];
                    pq[i] = readp(J - S);   // left of the grid: the zero column
                    real Ac[1], Bc[1], iB[1], p6[1], accP[1];
                    TL::coef_fwd(p, Ac[0], Bc[0]);
                    const real r = __builtin_amdgcn_rcp(Bc[0]);
                    iB[0] = fma(fma(-Bc[0], r, 1.0), r, r);
                    p6[0] = p * (1.0 / 6.0);
                    real recv[1], recvk[1];
                    recv[0] = wave_shift_down(rv.up[0]);   // nothing enters under the last lane
                    recvk[0] = wave_from_below_or(rv.ktop[0], kq[i]);
                    rv.step(recv, recvk, Ac, Bc, iB, p6, accP);
                    // right of the grid dF/dp is an exact zero (the adjoint is zero there) and lands in the zero
                    // column; left of the grid it is not zero (the adjoint has left the grid) and lands in the
                    // column nobody reads
                    P[__mul24(write_col(J, nb), kTileStride) + pbase] = accP[0];
                }
                if (g > 0 && g % CK == 0) {
                    // the recovered state against the exact one, which replaces it: rounding errors of the inverse
                    // recurrence cannot build up over more than CK chunks, and a drift disqualifies the pair
                    const SK_LDS real* cp = ckl + (g / CK - 1) * (2 * kWave);
                    const real e1 = cp[0];
                    const real e0 = wave_from_above_or(cp[kWave], 1.0);   // the lane above's k[a][J]; row 0 has the boundary above it
                    kscale = fmax(kscale, fmax(fabs(e0), fabs(e1)));
                    // written so that a NaN counts as drift
                    if (!(fabs(rv.kR[0] - e0) <= kDriftTol * kscale) || !(fabs(rv.kR[1] - e1) <= kDriftTol * kscale)) drift = true;
                    rv.kR[0] = e0;
                    rv.kR[1] = e1;
                    rv.ktop[0] = e0;
                }
            }
            // the left end: the sweep started from the boundary value 1 in every lane
            if (!(fabs(rv.kR[0] - 1.0) <= kDriftTol * kscale) || !(fabs(rv.kR[1] - 1.0) <= kDriftTol * kscale)) drift = true;
        }
        // A pair whose inverse recurrence drifted adds nothing to the gradient sums (its G is not mapped) and is
        // listed for the replay kernel, which solves it once more.
        const bool passed = __ballot(drift) == 0ull;
        if (!passed && lane == 0) list_drifted(a, pid, pid2);

        // Loads for the second half of the linear map and for the next pair, issued here so that the first half
        // of the map covers their latency (during the sweeps the registers are needed elsewhere).
        const real* dxg = a.dx + xi * a.xstride;
        real xc[16], xbn[4][KC], gkn = 0.0;
        if (a.want_gy && passed) TL::load_c(dxg, a.DS, padb, lane, xc);
        if (q + 1 < q1) {
            long xin, yin, pidn, pidn2;
            gram_pair(a, q + 1, xin, yin, pidn, pidn2);
            TL::load_b(a.dx + xin * a.xstride, a.DS, padb, lane, xbn);
            gkn = gram_weight(a, pidn, pidn2);
        }

        // ---- the linear map of Section 3.4 on the matrix cores ----
        if (a.want_gx && passed) {
            // dF/d(dx)[a, c] = sum_b G[a, b] dy[b, c]: A operand G[16 I + l % 16][4 kb + l / 16], B operand yc[kb]
            // (the lane's part of the address goes through an opaque move: computed here, once per pair, from one
            // register, instead of sixteen loop-invariant addresses kept alive over the whole pair loop)
            int lrow = g16 - padb;
            asm volatile("" : "+v"(lrow));
            real* gq = a.gdx + xi * a.xstride + (long)lrow * a.DS + n16;
#pragma unroll
            for (int I = 0; I < 4; ++I) {
                real4 acc = {0.0, 0.0, 0.0, 0.0};
                const SK_LDS real* gp = P + (g16 + 1) * kTileStride + 16 * I + n16;
#pragma unroll
                for (int kb = 0; kb < 16; ++kb)
                    acc = __builtin_amdgcn_mfma_f64_16x16x4f64(gp[4 * kb * kTileStride], yc[kb], acc, 0, 0, 0);
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int up = 16 * I + 4 * r;   // rows above the lane's first one
                    if (lrow + up >= 0 && n16 < a.d) unsafeAtomicAdd(&gq[(long)up * a.DS], acc[r]);
                }
            }
        }
        if (a.want_gy && passed) {
            // dF/d(dy)[b, c] = sum_a G[a, b] dx[a, c]: A operand G[4 ka + l / 16][16 J + l % 16], B operand xc[ka]
#pragma unroll
            for (int J = 0; J < 4; ++J) {
                const SK_LDS real* gp = P + (16 * J + n16 + 1) * kTileStride + g16;
#pragma unroll
                for (int ka = 0; ka < 16; ++ka)
                    gy[J] = __builtin_amdgcn_mfma_f64_16x16x4f64(gp[4 * ka], xc[ka], gy[J], 0, 0, 0);
            }
        }
#pragma unroll
        for (int T = 0; T < 4; ++T)
#pragma unroll
            for (int kc = 0; kc < KC; ++kc) xb[T][kc] = xbn[T][kc];
        gk = gkn;
    }
    flush_gy();
}

// ------------------------------------------------------------------------------------------------
// launchers
// ------------------------------------------------------------------------------------------------
template <int KC>
hipError_t launch_tile_k(bool backward, const SweepArgs& a, int grid, size_t lds, hipStream_t st)
{
    const void* fn = backward ? reinterpret_cast<const void*>(&tile_bwd_kernel<KC>)
                              : reinterpret_cast<const void*>(&tile_fwd_kernel<KC>);
    if (hipError_t e = allow_full_lds(fn); e != hipSuccess) return e;
    if (backward) hipLaunchKernelGGL((tile_bwd_kernel<KC>), dim3(grid), dim3(kWavesPerWG * kWave), lds, st, a);
    else hipLaunchKernelGGL((tile_fwd_kernel<KC>), dim3(grid), dim3(kWavesPerWG * kWave), lds, st, a);
    return hipGetLastError();
}

hipError_t launch_sweep_tile(bool backward, int DT, const SweepArgs& a, int grid, size_t lds, hipStream_t st)
{
    // what the kernels assume about the launch
    if (a.lk_M != 1 || a.rs1 != 0 || a.rs2 != 0 || a.mb > kWave || a.nb > kWave || a.mb < 1 || a.nb < 1 ||
        a.lk_padb != kWave - a.mb || a.rpad < kWave || a.qpad < kWave || a.DS <= DT || a.d > DT ||
        (backward && (!a.bad_list || !a.bad_count || (a.lk_NT % kLockS) != 0 || a.lk_NT < a.nb + kWave - 1 || a.lk_NT >= a.nb + kWave - 1 + kLockS ||
                      (size_t)a.lk_off_ck + (size_t)((a.lk_NT / kLockS - 1) / kTileCkChunks) * 2 * kWave * sizeof(real) >
                          a.lds_wave)))
        return hipErrorInvalidValue;
    switch (DT) {
        case 8: return launch_tile_k<2>(backward, a, grid, lds, st);
        case 16: return launch_tile_k<4>(backward, a, grid, lds, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace sk

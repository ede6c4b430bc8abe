// Per-lane building blocks of the lean sweeps (shared by the lock-step kernels, one workgroup per pair, and
// the solo kernels, one wavefront per pair): the increment inner product and coefficients of Eq. (1), the
// forward update of a lane's column of blocks, and its mirror image with the adjoint recurrence of
// Section 3.4.  A lane owns M block rows of 2^BL refined rows each and processes one block column per
// macro-step.  Nothing here masks lanes: a lane whose column lies outside the grid works with p = 0, i.e.
// A = B = 1, which keeps the boundary value 1 forward and a zero adjoint backward.
#pragma once
#include <hip/hip_runtime.h>

#include "sk_dev.h"
#include "sk_kernels.h"

namespace sk {

typedef double real2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ int clamp_col(int J, int hi)
{
    int r;
    asm("v_med3_i32 %0, %1, 0, %2" : "=v"(r) : "v"(J), "v"(hi));
    return r;
}

//
// LL (lead-lag paths, Section 4): the two transformed paths move their lead and their lag halves in turn, so
// their increment Gram matrix is a checkerboard: the 2 x 2 steps that come from one pair of original increments
// (a, b) hold <dx[a], dy[b]> on the diagonal (lead with lead, lag with lag) and nothing off it.  The transformed
// paths are never formed: the grid of the original increments is swept with one more level of refinement, whose
// cells take the coefficients of p on the diagonal quadrants of that level and those of p0 (the time channel's
// constant product alone, 0 without time augmentation) on the others.
//   LL = 0: no transform;  LL = 1: that level lies inside a block (block = all refined cells of one (a, b));
//   LL = 2: it lies above the blocks (a block is uniform: diagonal or not by the parity of its row and column).
template <int BL, int D, int M, int LL = 0>
struct Lock {
    static_assert(LL != 1 || BL >= 1, "a lead-lag level inside the blocks needs blocks of at least 2 x 2 cells");
    static constexpr int C = 1 << BL;
    static constexpr int HB = BL > 0 ? BL - 1 : 0;   // LL = 1: log2 of a quadrant's side
    // LL = 1: whether cell (rr, cc) of a lane's block column lies off the diagonal quadrants of its block
    static __device__ __forceinline__ constexpr bool cell_off(int rr, int cc)
    {
        return LL == 1 && ((((rr & (C - 1)) >> HB) ^ (cc >> HB)) & 1) != 0;
    }
    static constexpr int RR = M << BL;        // refined rows per lane
    static constexpr int DSc = D | 1;         // row stride of the increment arrays (doubles)
    static constexpr int NVC = RR + C + 2;    // checkpoint: right edge (RR+1), bottom edge (C), bottom-left corner
    static constexpr int PADF = kWave * C;    // doubles in front of node column 0 of a hand-over row
    static constexpr int CH1 = kLockCH1, CH2 = kLockCH2;
    static constexpr int CR1 = CH1 * M * kWave * 2;   // doubles per half of the coefficient ring, forward
    static constexpr int CR2 = CH2 * M * kWave * 4;   // ... reverse sweep
    static constexpr int GPH = CH2 * M * kWave;       // doubles per half of the dF/dp ring

    // A(p), B(p) of Eq. (1), and 1 / B(p) for the reverse sweep
    static __device__ __forceinline__ void coef_fwd(real p, real& Ac, real& Bc)
    {
        const real q2 = p * p;
        Bc = fma(q2, -1.0 / 12.0, 1.0);
        Ac = fma(p, 0.5, fma(q2, 1.0 / 12.0, 1.0));
    }
    // 1 / B without the hardware estimate (v_rcp_f64 issues at a quarter of the rate of an FMA: 20 clocks against 5
    // in a lone wave).  With q = p^2 / 12, B = 1 - q and the inner term of A is r0 = 1 + q = (1 - q^2) / B, so
    // e = 1 - B r0 = q^2 and 1 / B = r0 (1 + e + e^2 + ...): cut after e^2 the relative error is q^6, below one
    // rounding error for |p| < 0.17 and below 1e-12 up to |p| = 0.35, far beyond the increments for which the inverse
    // recurrence holds at all; a pair outside that range fails the drift check and is solved by replay.
    static __device__ __forceinline__ void coef_rev(real p, real& Ac, real& Bc, real& iB)
    {
        const real q2 = p * p;
        Bc = fma(q2, -1.0 / 12.0, 1.0);
        const real r0 = fma(q2, 1.0 / 12.0, 1.0);
        Ac = fma(p, 0.5, r0);
        const real e = fma(-Bc, r0, 1.0);
        iB = fma(fma(e, e, e), r0, r0);
    }

    // dF/dp ring: [macro-step][lane][M], so that a lane's M values move in one LDS instruction
    static __device__ __forceinline__ void gp_store(SK_LDS real* half, int i, int lane, const real (&v)[M])
    {
        SK_LDS real* q = half + (i * kWave + lane) * M;
        if constexpr (M == 2) {
            *(SK_LDS real2*)q = real2{v[0], v[1]};
        } else {
#pragma unroll
            for (int m = 0; m < M; ++m) q[m] = v[m];
        }
    }
    static __device__ __forceinline__ void gp_load(const SK_LDS real* half, int i, int lane, real (&v)[M])
    {
        const SK_LDS real* q = half + (i * kWave + lane) * M;
        if constexpr (M == 2) {
            const real2 t = *(const SK_LDS real2*)q;
            v[0] = t.x; v[1] = t.y;
        } else {
#pragma unroll
            for (int m = 0; m < M; ++m) v[m] = q[m];
        }
    }

    // ---------------- coefficient wave ----------------
    struct Coef {
        real dxr[M][D];
        int nbl[M];
        int lane, nb, nbm1, rs2;
        real tcm[M];   // the time channel's constant product; 0 for block rows above the grid
        int rowpar[M]; // LL = 2: parity of the lead-lag step the block row belongs to
        int rs2h;      // LL = 2: block columns per lead-lag step, log2
        const SK_LDS real* ylds;

        __device__ __forceinline__ void setup(const SweepArgs& a, int strip, int lane_, const real* dxp,
                                              const SK_LDS real* y)
        {
            lane = lane_; nb = a.nb; nbm1 = a.nb - 1; rs2 = a.rs2; ylds = y;
            rs2h = a.rs2 - 1;
#pragma unroll
            for (int m = 0; m < M; ++m) {
                const int I = (strip * kWave + lane) * M + m - a.lk_padb;   // block row; < 0: above the grid
                nbl[m] = I >= 0 ? a.nb : 0;
                tcm[m] = I >= 0 ? a.tc : 0.0;
                rowpar[m] = LL == 2 ? ((I >= 0 ? I : 0) >> (a.rs1 - 1)) & 1 : 0;
                const int arow = (I >= 0 ? I : 0) >> a.rs1;
                if (a.fused) {   // dxp: the pair's points [L1][d]; increments are formed here
                    const real* xp = dxp + (long)arow * a.d;
#pragma unroll
                    for (int c = 0; c < D; ++c) dxr[m][c] = (I >= 0 && c < a.d) ? a.sc * (xp[a.d + c] - xp[c]) : 0.0;
                } else {
                    const real* xp = dxp + (long)arow * DSc;
#pragma unroll
                    for (int c = 0; c < D; ++c) dxr[m][c] = I >= 0 ? a.sc * xp[c] : 0.0;
                }
            }
        }
        // A chunk of macro-steps [T0, T0 + n) is interior if every lane's column T - lane lies inside the grid:
        // then no clamping and no masking is needed (rows above the grid have zero increments and a zero
        // time constant, hence p = 0 anyway).
        __device__ __forceinline__ bool interior(int T0, int n) const { return T0 >= kWave - 1 && T0 + n <= nb; }
        // y increments of the block column this lane is at in macro-step T
        template <bool EDGE>
        __device__ __forceinline__ void fetch(int T, int& J, int& b, real (&y)[D]) const
        {
            J = T - lane;
            b = (EDGE ? clamp_col(J, nbm1) : J) >> rs2;
            const SK_LDS real* yp = ylds + __mul24(b, DSc);
#pragma unroll
            for (int c = 0; c < D; ++c) y[c] = yp[c];
        }
        // p of block m (Eq. (1), third line); 0 outside the grid
        template <bool EDGE>
        __device__ __forceinline__ real inner(int m, int J, const real (&y)[D]) const
        {
            real p = tcm[m];
#pragma unroll
            for (int c = 0; c < D; ++c) p = fma(dxr[m][c], y[c], p);
            if constexpr (LL == 2) p = off_block(m, J) ? tcm[m] : p;
            if constexpr (EDGE) return (unsigned)J < (unsigned)nbl[m] ? p : 0.0;
            else return p;
        }
        // LL = 2: whether block (m, J) lies off the diagonal of its lead-lag level (then p is the constant alone
        // and the block's dF/dp belongs to no increment)
        __device__ __forceinline__ bool off_block(int m, int J) const
        {
            if constexpr (LL == 2) return (((J >> rs2h) ^ rowpar[m]) & 1) != 0;
            else return false;
        }
        // LL = 1: p0 of the off-diagonal quadrants of block m in column J
        template <bool EDGE>
        __device__ __forceinline__ real inner_off(int m, int J) const
        {
            if constexpr (EDGE) return (unsigned)J < (unsigned)nbl[m] ? tcm[m] : 0.0;
            else return tcm[m];
        }
        // forward: (A, B) of the chunk of CH1 macro-steps starting at T0
        // part 0: every macro-step of the chunk; part 1 / 2: the even / odd ones (two coefficient waves share a
        // strip).  The y reads of all steps are issued before the arithmetic (PFY steps at a time).
        __device__ __forceinline__ void produce_fwd(int T0, SK_LDS real* half, int part) const
        {
            const bool in = interior(T0, CH1);
            if (part == 0) {
                if (in) produce_fwd_t<false, 0, 1>(T0, half); else produce_fwd_t<true, 0, 1>(T0, half);
            } else if (part == 1) {
                if (in) produce_fwd_t<false, 0, 2>(T0, half); else produce_fwd_t<true, 0, 2>(T0, half);
            } else {
                if (in) produce_fwd_t<false, 1, 2>(T0, half); else produce_fwd_t<true, 1, 2>(T0, half);
            }
        }
        template <bool EDGE, int I0, int IS>
        __device__ __forceinline__ void produce_fwd_t(int T0, SK_LDS real* half) const
        {
            SK_LDS real* wp = half + lane * 2;
            constexpr int NSTEP = (CH1 - I0 + IS - 1) / IS;   // steps handled by this wave
            constexpr int PFY = D <= 8 ? 4 : 2;               // steps whose y reads are in flight together
#pragma unroll
            for (int g0 = 0; g0 < NSTEP; g0 += PFY) {
                int J[PFY], b[PFY];
                real y[PFY][D];
#pragma unroll
                for (int u = 0; u < PFY; ++u)
                    if (g0 + u < NSTEP) fetch<EDGE>(T0 + I0 + (g0 + u) * IS, J[u], b[u], y[u]);
#pragma unroll
                for (int u = 0; u < PFY; ++u) {
                    if (g0 + u < NSTEP) {
                        const int i = I0 + (g0 + u) * IS;
#pragma unroll
                        for (int m = 0; m < M; ++m) {
                            const real p = inner<EDGE>(m, J[u], y[u]);
                            const real q2 = p * p;
                            const real Bc = fma(q2, -1.0 / 12.0, 1.0);
                            const real Ac = fma(p, 0.5, fma(q2, 1.0 / 12.0, 1.0));
                            *(SK_LDS real2*)(wp + (i * M + m) * (kWave * 2)) = real2{Ac, Bc};
                        }
                    }
                }
            }
        }
        // reverse: (A, B, 1/B, p/6) of the chunk of CH2 macro-steps starting at T0
        __device__ __forceinline__ void produce_rev(int T0, SK_LDS real* half) const
        {
            if (interior(T0, CH2)) produce_rev_t<false>(T0, half);
            else produce_rev_t<true>(T0, half);
        }
        template <bool EDGE>
        __device__ __forceinline__ void produce_rev_t(int T0, SK_LDS real* half) const
        {
            // two planes of 16 bytes per lane, (A, B) and (1/B, p/6): consecutive lanes at consecutive 16 bytes
            SK_LDS real* wp = half + lane * 2;
            int J[2], b[2];
            real y[2][D];
            fetch<EDGE>(T0, J[0], b[0], y[0]);
#pragma unroll
            for (int i = 0; i < CH2; ++i) {
                if (i + 1 < CH2) fetch<EDGE>(T0 + i + 1, J[(i + 1) & 1], b[(i + 1) & 1], y[(i + 1) & 1]);
#pragma unroll
                for (int m = 0; m < M; ++m) {
                    const real p = inner<EDGE>(m, J[i & 1], y[i & 1]);
                    real Ac, Bc, invB;
                    coef_rev(p, Ac, Bc, invB);
                    SK_LDS real* ep = wp + (i * M + m) * (kWave * 2);
                    *(SK_LDS real2*)(ep) = real2{Ac, Bc};
                    *(SK_LDS real2*)(ep + CR2 / 2) = real2{invB, p * (1.0 / 6.0)};
                }
            }
        }
        // reverse: the linear map of Section 3.4 for the chunk starting at T0, from the dF/dp ring.
        // x side: this lane's rows accumulate in registers.
        __device__ __forceinline__ void consume_gx(int T0, const SK_LDS real* half, real (&gacc)[M][D]) const
        {
            if (interior(T0, CH2)) consume_gx_t<false>(T0, half, gacc);
            else consume_gx_t<true>(T0, half, gacc);
        }
        template <bool EDGE>
        __device__ __forceinline__ void consume_gx_t(int T0, const SK_LDS real* half, real (&gacc)[M][D]) const
        {
            constexpr int PFY = D <= 8 ? CH2 : 2;
#pragma unroll
            for (int g0 = 0; g0 < CH2; g0 += PFY) {
                int J[PFY], b[PFY];
                real y[PFY][D], gv[PFY][M];
#pragma unroll
                for (int u = 0; u < PFY; ++u) {
                    fetch<EDGE>(T0 + g0 + u, J[u], b[u], y[u]);
                    gp_load(half, g0 + u, lane, gv[u]);
                }
#pragma unroll
                for (int u = 0; u < PFY; ++u)
#pragma unroll
                    for (int m = 0; m < M; ++m) {
                        // outside the grid dF/dp is not zero on the left (the adjoint has left the grid there);
                        // rows above the grid are never flushed
                        const real gp = ((!EDGE || (unsigned)J[u] < (unsigned)nbl[m]) && !off_block(m, J[u])) ? gv[u][m] : 0.0;
#pragma unroll
                        for (int c = 0; c < D; ++c) gacc[m][c] = fma(gp, y[u][c], gacc[m][c]);
                    }
            }
        }
        // y side: the column's accumulator row in LDS.
        __device__ __forceinline__ void consume_gy(int T0, const SK_LDS real* half, SK_LDS real* gy) const
        {
            // rs2 == 0: the 64 lanes are at 64 different columns, so a plain read-modify-write of the column's
            // accumulator row cannot collide inside the wave; the wave of the neighbouring strip works
            // kLockLag2 columns away in the same chunk.
            const bool plain = rs2 == 0;
            if (interior(T0, CH2)) {
                if (plain) consume_gy_t<false, true>(T0, half, gy); else consume_gy_t<false, false>(T0, half, gy);
            } else {
                if (plain) consume_gy_t<true, true>(T0, half, gy); else consume_gy_t<true, false>(T0, half, gy);
            }
        }
        template <bool EDGE, bool PLAIN>
        __device__ __forceinline__ void consume_gy_t(int T0, const SK_LDS real* half, SK_LDS real* gy) const
        {
            real gv[CH2][M];
#pragma unroll
            for (int i = 0; i < CH2; ++i) gp_load(half, i, lane, gv[i]);
#pragma unroll
            for (int i = 0; i < CH2; ++i) {
                const int J = T0 + i - lane;
                const int b = (EDGE ? clamp_col(J, nbm1) : J) >> rs2;
                SK_LDS real* gq = gy + __mul24(b, DSc);
                real t[D];
#pragma unroll
                for (int c = 0; c < D; ++c) {
                    // rows above the grid have zero increments
                    real v = 0.0;
#pragma unroll
                    for (int m = 0; m < M; ++m) {
                        const real gp = ((!EDGE || (unsigned)J < (unsigned)nbl[m]) && !off_block(m, J)) ? gv[i][m] : 0.0;
                        v = m == 0 ? gp * dxr[0][c] : fma(gp, dxr[m][c], v);
                    }
                    t[c] = v;
                }
                if constexpr (PLAIN) {
                    // lanes whose column was clamped into the grid must not touch a row that another lane owns;
                    // the step after this one reads what this one wrote (the lane above moves to this column)
                    if (!EDGE || (unsigned)J < (unsigned)nb) {
                        real o[D];
#pragma unroll
                        for (int c = 0; c < D; ++c) o[c] = gq[c];
#pragma unroll
                        for (int c = 0; c < D; ++c) gq[c] = o[c] + t[c];
                    }
                } else {
#pragma unroll
                    for (int c = 0; c < D; ++c) lds_atomic_add(gq + c, t[c]);
                }
            }
        }
    };

    // ---------------- LL = 1: coefficients of the off-diagonal quadrants, kept by the stencil wave ----------------
    // Their p is the time channel's constant inside the grid and 0 outside it, where A = B = 1 keep the boundary
    // value: above the grid (block rows that pad the first strip) and left of it (a lane that has not started).
    // Right of the grid nothing depends on them (both sweeps use the same ones there).
    struct Off {
        real A0c, B0c, iB0c;
        int tmin[M];   // first macro-step of the strip in which the lane's block m is inside the grid

        __device__ __forceinline__ void setup(const SweepArgs& a, int strip, int lane)
        {
            coef_rev(a.tc, A0c, B0c, iB0c);
#pragma unroll
            for (int m = 0; m < M; ++m) {
                const int I = (strip * kWave + lane) * M + m - a.lk_padb;
                tmin[m] = I >= 0 ? lane : 0x7fffffff;
            }
        }
        __device__ __forceinline__ void at(int T, real (&A0)[M], real (&B0)[M]) const
        {
#pragma unroll
            for (int m = 0; m < M; ++m) {
                const bool in = T >= tmin[m];
                A0[m] = in ? A0c : 1.0;
                B0[m] = in ? B0c : 1.0;
            }
        }
        __device__ __forceinline__ void at(int T, real (&A0)[M], real (&B0)[M], real (&iB0)[M]) const
        {
            at(T, A0, B0);
#pragma unroll
            for (int m = 0; m < M; ++m) iB0[m] = T >= tmin[m] ? iB0c : 1.0;
        }
    };

    // ---------------- stencil wave, forward ----------------
    struct Fwd {
        real left[RR + 1];   // right edge of the last block column, left[0] its top corner
        real bot[C];         // bottom edge (without the left corner)
        real blc;            // bottom-left corner

        __device__ __forceinline__ void init()
        {
#pragma unroll
            for (int i = 0; i <= RR; ++i) left[i] = 1.0;
#pragma unroll
            for (int i = 0; i < C; ++i) bot[i] = 1.0;
            blc = 1.0;
        }
        // one macro-step: Eq. (1) on the RR x C cells of this lane's block column
        __device__ __forceinline__ void step(const real (&recv)[C], const real (&Ac)[M], const real (&Bc)[M])
        {
            static_assert(LL != 1, "lead-lag blocks take the coefficients of their off-diagonal quadrants too");
            step(recv, Ac, Bc, Ac, Bc);
        }
        // A0, B0: coefficients of the off-diagonal quadrants (LL = 1; unused otherwise)
        __device__ __forceinline__ void step(const real (&recv)[C], const real (&Ac)[M], const real (&Bc)[M],
                                             const real (&A0)[M], const real (&B0)[M])
        {
            real top[C + 1];
            top[0] = left[0];
#pragma unroll
            for (int cc = 0; cc < C; ++cc) top[cc + 1] = recv[cc];
#pragma unroll
            for (int rr = 0; rr < RR; ++rr) {
                const int m = rr >> BL;
                real cur[C + 1];
                cur[0] = left[rr + 1];
#pragma unroll
                for (int cc = 0; cc < C; ++cc) {
                    const real Aq = cell_off(rr, cc) ? A0[m] : Ac[m], Bq = cell_off(rr, cc) ? B0[m] : Bc[m];
                    cur[cc + 1] = fma(cur[cc] + top[cc + 1], Aq, -(top[cc] * Bq));
                }
                left[rr + 1] = cur[C];
#pragma unroll
                for (int cc = 0; cc <= C; ++cc) top[cc] = cur[cc];
            }
            blc = top[0];
#pragma unroll
            for (int cc = 0; cc < C; ++cc) bot[cc] = top[cc + 1];
            left[0] = recv[C - 1];
        }
        // chunk of CH1 macro-steps starting at T0
        __device__ __forceinline__ void chunk(int T0, int lane, const SK_LDS real* half, const SK_LDS real* rowprev,
                                              SK_LDS real* rowcur, SK_LDS real* dump, const Off& off)
        {
            const SK_LDS real* cp = half + lane * 2;
            const SK_LDS real* ip = rowprev + T0 * C + 1;                          // lane 0's top edge
            SK_LDS real* op = lane == kWave - 1 ? rowcur + (T0 - (kWave - 1)) * C + 1 : dump + lane * C;
            constexpr int PF = 2;   // coefficient and edge reads are issued PF macro-steps ahead
            real2 ab[CH1][M];
            real edge[CH1][C];
            auto load = [&](int i) {
#pragma unroll
                for (int m = 0; m < M; ++m) ab[i][m] = *(const SK_LDS real2*)(cp + (i * M + m) * (kWave * 2));
#pragma unroll
                for (int cc = 0; cc < C; ++cc) edge[i][cc] = ip[i * C + cc];
            };
#pragma unroll
            for (int i = 0; i < PF; ++i) load(i);
#pragma unroll
            for (int i = 0; i < CH1; ++i) {
                if (i + PF < CH1) load(i + PF);
                real Ac[M], Bc[M];
#pragma unroll
                for (int m = 0; m < M; ++m) { Ac[m] = ab[i][m].x; Bc[m] = ab[i][m].y; }
                real recv[C];
#pragma unroll
                for (int cc = 0; cc < C; ++cc) recv[cc] = wave_from_above_or(bot[cc], edge[i][cc]);
                if constexpr (LL == 1) {
                    real A0[M], B0[M];
                    off.at(T0 + i, A0, B0);
                    step(recv, Ac, Bc, A0, B0);
                } else {
                    step(recv, Ac, Bc);
                }
#pragma unroll
                for (int cc = 0; cc < C; ++cc) op[i * C + cc] = bot[cc];
            }
        }
        __device__ __forceinline__ void store_ckpt(real* cp) const
        {
#pragma unroll
            for (int i = 0; i <= RR; ++i) cp[i * kWave] = left[i];
#pragma unroll
            for (int i = 0; i < C; ++i) cp[(RR + 1 + i) * kWave] = bot[i];
            cp[(RR + 1 + C) * kWave] = blc;
        }
    };

    // ---------------- stencil wave, reverse ----------------
    struct Rev {
        real kR[RR + 1];     // forward values on the right edge of the block column to un-compute next
        real ktop[C];        // recovered top edge, handed to the lane above
        real accL[RR + 1];   // partial adjoints of the left edge nodes (index 0 unused)
        real corner;         // partial adjoint of the top-left node
        real up[C];          // adjoint contributions to the top edge nodes, handed to the lane above

        __device__ __forceinline__ void init()
        {
#pragma unroll
            for (int i = 0; i <= RR; ++i) { kR[i] = 1.0; accL[i] = 0.0; }
#pragma unroll
            for (int i = 0; i < C; ++i) { ktop[i] = 1.0; up[i] = 0.0; }
            corner = 0.0;
        }
        __device__ __forceinline__ void step(const real (&recv)[C], const real (&recvk)[C], const real (&Ac)[M],
                                             const real (&Bc)[M], const real (&iB)[M], const real (&p6)[M],
                                             real (&accP)[M])
        {
            static_assert(LL != 1, "lead-lag blocks take the coefficients of their off-diagonal quadrants too");
            step(recv, recvk, Ac, Bc, iB, p6, Ac, Bc, iB, accP);
        }
        // A0, B0, iB0: coefficients of the off-diagonal quadrants (LL = 1; unused otherwise), whose cells take part in
        // the recurrences but not in dF/dp: their p is a constant
        __device__ __forceinline__ void step(const real (&recv)[C], const real (&recvk)[C], const real (&Ac)[M],
                                             const real (&Bc)[M], const real (&iB)[M], const real (&p6)[M],
                                             const real (&A0)[M], const real (&B0)[M], const real (&iB0)[M],
                                             real (&accP)[M])
        {
            real e[RR + 1][C + 1], gn[RR + 1][C + 1];
#pragma unroll
            for (int rr = 0; rr <= RR; ++rr) e[rr][C] = kR[rr];
#pragma unroll
            for (int cc = 0; cc < C; ++cc) e[RR][cc] = recvk[cc];
#pragma unroll
            for (int rr = 0; rr <= RR; ++rr)
#pragma unroll
                for (int cc = 0; cc <= C; ++cc) gn[rr][cc] = 0.0;
#pragma unroll
            for (int rr = 1; rr <= RR; ++rr) gn[rr][C] = accL[rr];
#pragma unroll
            for (int cc = 0; cc < C; ++cc) gn[RR][cc + 1] += recv[cc];
            gn[0][C] = corner;
            // dF/dp of a block: sum over its cells of g (s A'(p) - k B'(p)); p is the block's, so the two sums over the
            // cells are formed first and the derivatives of the coefficients applied once
            real gs[M], gk[M];
#pragma unroll
            for (int rr = RR - 1; rr >= 0; --rr) {
                const int m = rr >> BL;
#pragma unroll
                for (int cc = C - 1; cc >= 0; --cc) {
                    const bool off = cell_off(rr, cc);
                    const real Aq = off ? A0[m] : Ac[m], Bq = off ? B0[m] : Bc[m], iBq = off ? iB0[m] : iB[m];
                    const real s = e[rr + 1][cc] + e[rr][cc + 1];
                    e[rr][cc] = fma(s, Aq, -e[rr + 1][cc + 1]) * iBq;   // Eq. (1) solved for its oldest term
                    const real go = gn[rr + 1][cc + 1];
                    gn[rr + 1][cc] = fma(go, Aq, gn[rr + 1][cc]);
                    gn[rr][cc + 1] = fma(go, Aq, gn[rr][cc + 1]);
                    gn[rr][cc] = fma(-go, Bq, gn[rr][cc]);
                    if (off) continue;
                    const bool first = (rr & (C - 1)) == C - 1 && cc == C - 1;   // the block's first cell in this order
                    gs[m] = first ? go * s : fma(go, s, gs[m]);
                    gk[m] = first ? go * e[rr][cc] : fma(go, e[rr][cc], gk[m]);
                }
            }
#pragma unroll
            for (int m = 0; m < M; ++m) accP[m] = fma(gs[m], p6[m] + 0.5, gk[m] * p6[m]);   // A'(p) = p/6 + 1/2, -B'(p) = p/6
#pragma unroll
            for (int cc = 0; cc < C; ++cc) { up[cc] = gn[0][cc + 1]; ktop[cc] = e[0][cc]; }
            corner = gn[0][0];
#pragma unroll
            for (int rr = 1; rr <= RR; ++rr) accL[rr] = gn[rr][0];
#pragma unroll
            for (int rr = 0; rr <= RR; ++rr) kR[rr] = e[rr][0];
        }
        // chunk of CH2 mirrored macro-steps T0 + CH2 - 1 down to T0
        __device__ __forceinline__ void chunk(int T0, int lane, const SK_LDS real* half, const SK_LDS real* arow_in,
                                              const SK_LDS real* krow, SK_LDS real* arow_out, SK_LDS real* dump,
                                              SK_LDS real* gphalf, const Off& off)
        {
            const SK_LDS real* cp = half + lane * 2;                    // see produce_rev_t for the layout
            const SK_LDS real* ap = arow_in + (T0 - (kWave - 1)) * C;   // feeds of the strip's last lane
            const SK_LDS real* kp = krow + (T0 - (kWave - 1)) * C;
            SK_LDS real* op = lane == 0 ? arow_out + T0 * C : dump + lane * C;
            constexpr int PF = 1;   // reads one macro-step ahead: deeper prefetch costs more registers than it hides
            real2 ab[CH2][M], ip6[CH2][M];
            real ea[CH2][C], ek[CH2][C];
            auto load = [&](int i) {
#pragma unroll
                for (int m = 0; m < M; ++m) {
                    const SK_LDS real* ep = cp + (i * M + m) * (kWave * 2);
                    ab[i][m] = *(const SK_LDS real2*)(ep);
                    ip6[i][m] = *(const SK_LDS real2*)(ep + CR2 / 2);
                }
#pragma unroll
                for (int cc = 0; cc < C; ++cc) { ea[i][cc] = ap[i * C + cc]; ek[i][cc] = kp[i * C + cc]; }
            };
#pragma unroll
            for (int i = CH2 - 1; i > CH2 - 1 - PF; --i) load(i);
#pragma unroll
            for (int i = CH2 - 1; i >= 0; --i) {
                if (i - PF >= 0) load(i - PF);
                real Ac[M], Bc[M], iB[M], p6[M], accP[M];
#pragma unroll
                for (int m = 0; m < M; ++m) { Ac[m] = ab[i][m].x; Bc[m] = ab[i][m].y; iB[m] = ip6[i][m].x; p6[m] = ip6[i][m].y; }
                real recv[C], recvk[C];
#pragma unroll
                for (int cc = 0; cc < C; ++cc) {
                    recv[cc] = wave_from_below_or(up[cc], ea[i][cc]);
                    recvk[cc] = wave_from_below_or(ktop[cc], ek[i][cc]);
                }
                if constexpr (LL == 1) {
                    real A0[M], B0[M], iB0[M];
                    off.at(T0 + i, A0, B0, iB0);
                    step(recv, recvk, Ac, Bc, iB, p6, A0, B0, iB0, accP);
                } else {
                    step(recv, recvk, Ac, Bc, iB, p6, accP);
                }
#pragma unroll
                for (int cc = 0; cc < C; ++cc) op[i * C + cc] = up[cc];
                gp_store(gphalf, i, lane, accP);
            }
        }
    };
};

}  // namespace sk

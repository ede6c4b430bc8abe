// Tile kernels (gfx950), backward: see sk_tile.hip for the scheme; this file holds the kernel that sweeps forward with
// checkpoints, then backward by inverting Eq. (1), and maps dF/dp to the increment gradients on the matrix cores.
#include "sk_tile.h"

namespace sk {

// ------------------------------------------------------------------------------------------------
// backward
// ------------------------------------------------------------------------------------------------
// PAIRS: the sweeps move p and dF/dp two columns per LDS instruction (grids of at most 63 columns: the zero column
// then has another one behind it).
template <int KC, bool PAIRS>
__global__ __launch_bounds__(kWave, 1) void tile_bwd_kernel(SweepArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    using TL = Tile<KC>;
    using LK = Lock<0, 4 * KC, 1>;
    constexpr int S = kLockS;          // macro-steps per unrolled chunk
    constexpr int CK = kTileCkChunks;  // chunks between checkpoints
    const int lane = threadIdx.x;
    const int n16 = lane & 15, g16 = lane >> 4;
    const long slot = blockIdx.x;        // one wave per workgroup
    const long nslots = gridDim.x;
    // The workgroup's LDS is all dynamic (this kernel has no static __shared__ data), so it starts at LDS address 0.
    // Written as the constant, because the symbol's address is only known at link time and would cost an addition in
    // every address formed from it; should a toolchain ever place it elsewhere, the call reports a failed launch
    // (error flag 1: NaN outputs) instead of computing on the wrong memory.
    if ((unsigned)(size_t)(SK_LDS unsigned char*)smem != 0u) {
        if (lane == 0) atomicExch(a.err, 1);
        return;
    }
    SK_LDS unsigned char* const mylds = (SK_LDS unsigned char*)(size_t)0;
    SK_LDS real* P = (SK_LDS real*)mylds;
    // Checkpoints of the forward sweep, in LDS: per lane the last two values of its row, k[a + 1][J] and
    // k[a + 1][J - 1] (J the column the lane is about to process); the row above is the neighbouring lane's.
    SK_LDS real* ckl = (SK_LDS real*)(mylds + a.lk_off_ck) + lane;
    // The bottom row of the pair (the last lane's outputs, which no lane recovers in the reverse sweep) has an array
    // of its own, by node column: krow[c] for c = -8 .. 64 (every node left of the grid is 1, and a chunk of eight
    // macro-steps that lies wholly left of column -8 neither writes nor reads).  Contiguous, so that the eight values
    // of a chunk move two per LDS instruction.
    // Macro-steps run from 0 to NT - 1 with NT a multiple of S; the sweep proper ends at the last one (the last lane at
    // the last column), so that the reverse sweep starts with the seed in place, and begins tpad steps late.
    const int NT = a.lk_NT;
    const int tpad = NT - (a.nb + kWave - 1);   // 0 .. S - 1
    SK_LDS real* const krow = (SK_LDS real*)(mylds + a.lk_off_krows) + kTileRowPad;
    const long q0 = slot * a.npairs / nslots, q1 = (slot + 1) * a.npairs / nslots;
    const int nb = a.nb, padb = a.lk_padb;
    const int nch = NT / S;
    const bool last = lane == kWave - 1;
    long cur_y = -1;
    real* gdy_cur = nullptr;

    P[(kTileCols - 1) * kTileStride + lane] = 0.0;   // column 64: the zero column of a pair with 64 columns
    if (lane < kTileRowPad) krow[lane - kTileRowPad] = 1.0;   // node columns -8 .. -1
    if constexpr (PAIRS) P[lane] = 0.0;                        // column -1 (reads as zero in the sweeps)

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
                    if (b < a.q && n16 < a.d) unsafeAtomicAdd(&gdy_cur[(long)b * a.DS + n16], gy[J][r] * (1.0 / 6.0));   // (6 dF/dp: see the reverse sweep)
                }
        }
    };
    // p of column J is read, and dF/dp written, at byte offset kColBytes (J + 1) + 8 lane of P, which starts at LDS
    // address 0 (one wave per workgroup).  With t = kColBytes J + 8 lane the two clamps (reads: J inside the grid, else the zero column nb; writes: the
    // zero column to the right, where the value is zero, the unread column -1 to the left) become one instruction on t
    // (t < 0 exactly when J < 0, since 8 lane < kColBytes), and the rest is the instruction's offset.
    constexpr int kColBytes = kTileStride * (int)sizeof(real);
    const int lane8 = lane * (int)sizeof(real);
    const unsigned t_zero = (unsigned)(nb * kColBytes + lane8);   // the zero column
    const int t_unread = lane8 - kColBytes;                       // column -1
    auto readp = [&](int t) {
        return *(const SK_LDS real*)((const SK_LDS char*)P + kColBytes + min((unsigned)t, t_zero));
    };
    auto writep = [&](int t, real v) {
        int o;
        asm("v_med3_i32 %0, %1, %2, %3" : "=v"(o) : "v"(t), "v"(t_unread), "v"((int)t_zero));
        *(SK_LDS real*)((SK_LDS char*)P + kColBytes + o) = v;
    };
    // Two columns at once (PAIRS), J and J + 1, with one clamp on the byte offset u = t + kColBytes of (J, lane) from
    // column -1.  Reads: J from -1 to nb as it is (column -1 reads as zero: it is cleared before every pair, and a lane
    // writes there only after its last read of it; columns nb and nb + 1 are zero), anything else the zero columns.
    // Writes: the same, except that a pair wholly left of the grid (u < 0) goes to two spare slots (slot 64 of the
    // columns lane and lane + 1, which no one reads).
    const unsigned u_zero = t_zero + kColBytes;
    const unsigned u_dump = (unsigned)(lane * kColBytes + kWave * (int)sizeof(real));
    auto readp2 = [&](int t, real& lo, real& hi) {
        const SK_LDS real* bp = (const SK_LDS real*)((const SK_LDS char*)P + min((unsigned)(t + kColBytes), u_zero));
        lo = bp[0];
        hi = bp[kTileStride];
    };
    auto writep2 = [&](int t, real lo, real hi) {
        const int u = t + kColBytes;
        const unsigned o = u < 0 ? u_dump : min((unsigned)u, u_zero);
        SK_LDS real* bp = (SK_LDS real*)((SK_LDS char*)P + o);
        bp[0] = lo;
        bp[kTileStride] = hi;
    };

    // Operands of the pair in work, loaded while the previous pair was in the linear map.
    real xb[4][KC];
    real gk = 0.0;
    PairCursor cur;
    if (q0 < q1) {
        cur.locate(a, q0);
        TL::load_b(a.dx + cur.xi * a.xstride, a.DS, padb, lane, xb);
        gk = gram_weight(a, cur.pid, cur.pid2);
    }
    for (long q = q0; q < q1; ++q) {
        const long xi = cur.xi, yi = cur.yi, pid = cur.pid, pid2 = cur.pid2;
        if (yi != cur_y) {
            flush_gy();
            const real* dyg = a.dy + yi * a.ystride;
            TL::load_b(dyg, a.DS, 0, lane, yb);
            TL::load_c(dyg, a.DS, 0, lane, yc);
#pragma unroll
            for (int kb = 0; kb < 16; ++kb) yc[kb] *= 1.0 / 6.0;   // P holds 6 dF/dp after the reverse sweep
#pragma unroll
            for (int J = 0; J < 4; ++J) gy[J] = real4{0.0, 0.0, 0.0, 0.0};
            cur_y = yi;
            gdy_cur = a.gdy + yi * a.ystride;
        }
        if (a.tc != 0.0) TL::template gram_tiles<true>(P, yb, xb, lane, padb, nb, a.tc);
        else TL::template gram_tiles<false>(P, yb, xb, lane, padb, nb, 0.0);

        // ---- phase 1: forward; a checkpoint every CK chunks and the bottom row into LDS ----
        real kR0, kR1;   // exact state the reverse sweep starts from: k[a][J], k[a + 1][J]
        {
            typename LK::Fwd f;
            f.init();
            real pq[S];
            int tn = (-tpad - lane) * kColBytes + lane8;   // t of the next macro-step to fetch p for
#pragma unroll
            for (int i = 0; i < S; ++i) {
                if constexpr (!PAIRS) pq[i] = readp(tn + i * kColBytes);
                else if (i % 2 == 0) readp2(tn + i * kColBytes, pq[i], pq[i + 1]);
            }
            tn += S * kColBytes;
            int cl = -tpad - (kWave - 1) + 1;   // node column the last lane writes in the chunk's first macro-step
            // (chunks in groups of CK, a checkpoint in front of every group but the first)
            int g = 0;
            for (int k = 0; g < nch; ++k) {
                if (k > 0) {
                    SK_LDS real* cp = ckl + (k - 1) * (2 * kWave);
                    cp[0] = f.left[1];
                    cp[kWave] = f.blc;
                }
                const int gend = min((k + 1) * CK, nch);
                auto chunk = [&]() __attribute__((always_inline)) {
                    real kb[S];   // the lane's bottom values of the chunk; the last lane's are the pair's bottom row
                    real pnext = 0.0;
#pragma unroll
                    for (int i = 0; i < S; ++i) {
                        const real p = pq[i];
                        // the next chunk's p (past the last step: the zero column, unused)
                        if constexpr (!PAIRS) pq[i] = readp(tn + i * kColBytes);
                        else if (i % 2 == 0) readp2(tn + i * kColBytes, pq[i], pnext);
                        else pq[i] = pnext;
                        real Ac[1], Bc[1], recv[1];
                        TL::coef_fwd(p, Ac[0], Bc[0]);
                        recv[0] = wave_from_above_or(f.bot[0], 1.0);
                        f.step(recv, Ac, Bc);
                        kb[i] = f.bot[0];
                    }
                    if (last && cl >= -kTileRowPad) {   // (further left every value is the boundary value 1)
                        SK_LDS real* kp = krow + cl;
#pragma unroll
                        for (int i = 0; i < S; ++i) kp[i] = kb[i];
                    }
                    ++g;
                    tn += S * kColBytes;
                    cl += S;
                };
                if (gend - g == CK) {   // a full group: straight-line code (see the reverse sweep)
#pragma unroll
                    for (int c = 0; c < CK; ++c) chunk();
                } else {
                    while (g < gend) chunk();
                }
            }
            kR0 = f.left[0];
            kR1 = f.left[1];
        }
        if (a.k_out && lane == 0) {
            a.k_out[pid] = krow[nb];
            if (pid2 != pid) a.k_out[pid2] = krow[nb];
        }

        // ---- phase 2: the mirror image; 6 G = 6 dF/dp replaces p in place ----
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
            // t of this lane's column in the first macro-step of the chunk
            int tb = ((nch - 1) * S - tpad - lane) * kColBytes + lane8;
#pragma unroll
            for (int i = 0; i < S; ++i) {
                if constexpr (!PAIRS) pq[i] = readp(tb + i * kColBytes);
                else if (i % 2 == 0) readp2(tb + i * kColBytes, pq[i], pq[i + 1]);
            }
            int cl = (nch - 1) * S - tpad - (kWave - 1);   // node column under the last lane's block, first macro-step
            // (chunks in groups of CK from the right, a checkpoint behind every group but the leftmost)
            int g = nch - 1;
            for (int k = (nch - 1) / CK; k >= 0; --k) {
                // (a full group of CK chunks runs as straight-line code: values that live from chunk to chunk then need
                // no moves into fixed registers at every chunk's end)
                auto chunk = [&]() __attribute__((always_inline)) {
                    // the last lane's bottom edge
                    if (cl >= -kTileRowPad) {
                        const SK_LDS real* kp = krow + cl;
#pragma unroll
                        for (int i = 0; i < S; ++i) kq[i] = kp[i];
                    } else {
#pragma unroll
                        for (int i = 0; i < S; ++i) kq[i] = 1.0;
                    }
                    real pnext = 0.0, ghold = 0.0;
#pragma unroll
                    for (int i = S - 1; i >= 0; --i) {
                        const real p = pq[i];
                        // the next chunk's p (left of the grid: the zero column)
                        if constexpr (!PAIRS) pq[i] = readp(tb + (i - S) * kColBytes);
                        else if (i % 2 == 1) readp2(tb + (i - 1 - S) * kColBytes, pnext, pq[i]);
                        else pq[i] = pnext;
                        real Ac, Bc, iB;
                        LK::coef_rev(p, Ac, Bc, iB);
                        const real recv = wave_shift_down(rv.up[0]);   // nothing enters under the last lane
                        const real recvk = wave_from_below_or(rv.ktop[0], kq[i]);
                        // The mirror image of the step for a lane's single cell (LK::Rev::step written out), with
                        // 6 dF/dp = g ((k[i+1,j] + k[i,j+1]) (p + 3) + k[i,j] p) in place of dF/dp: two instructions
                        // fewer, and the factor 1/6 goes into the operands of the linear map below.
                        const real s01 = recvk + rv.kR[0];
                        const real e00 = fma(s01, Ac, -rv.kR[1]) * iB;   // Eq. (1) solved for its oldest term
                        const real go = rv.accL[1] + recv;
                        rv.accL[1] = go * Ac;
                        rv.up[0] = fma(go, Ac, rv.corner);
                        rv.corner = -(go * Bc);
                        const real accP6 = go * fma(s01, p + 3.0, e00 * p);
                        rv.kR[1] = recvk;
                        rv.kR[0] = e00;
                        rv.ktop[0] = e00;
                        // right of the grid dF/dp is an exact zero (the adjoint is zero there) and lands in the zero
                        // column; left of the grid it is not zero (the adjoint has left the grid) and lands in the
                        // column nobody reads
                        if constexpr (!PAIRS) writep(tb + i * kColBytes, accP6);
                        else if (i % 2 == 1) ghold = accP6;
                        else writep2(tb + i * kColBytes, accP6, ghold);
                    }
                    --g;
                    tb -= S * kColBytes;
                    cl -= S;
                };
                if (g - k * CK + 1 == CK) {
#pragma unroll
                    for (int c = 0; c < CK; ++c) chunk();
                } else {
                    while (g >= k * CK) chunk();
                }
                if (k > 0) {
                    // the recovered state against the exact one, which replaces it: rounding errors of the inverse
                    // recurrence cannot build up over more than CK chunks, and a drift disqualifies the pair
                    const SK_LDS real* cp = ckl + (k - 1) * (2 * kWave);
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
        if constexpr (PAIRS) P[lane] = 0.0;   // column -1 took the dF/dp of lanes left of the grid
        // A pair whose inverse recurrence drifted adds nothing to the gradient sums (its G is not mapped) and is
        // listed for the replay kernel, which solves it once more.
        const bool passed = __ballot(drift) == 0ull;
        if (!passed && lane == 0) list_drifted(a, pid, pid2);

        // Loads for the second half of the linear map and for the next pair, issued here so that the first half
        // of the map covers their latency (during the sweeps the registers are needed elsewhere).
        const real* dxg = a.dx + xi * a.xstride;
        real xc[16], xbn[4][KC], gkn = 0.0;
        if (a.want_gy && passed) TL::load_c(dxg, a.DS, padb, lane, xc);
        cur.next(a);
        if (q + 1 < q1) {
            TL::load_b(a.dx + cur.xi * a.xstride, a.DS, padb, lane, xbn);
            gkn = gram_weight(a, cur.pid, cur.pid2);
        }

        // ---- the linear map of Section 3.4 on the matrix cores ----
        if (a.want_gx && passed) {
            // dF/d(dx)[a, c] = sum_b G[a, b] dy[b, c]: A operand G[16 I + l % 16][4 kb + l / 16], B operand yc[kb]
            // (the lane's part of the address goes through an opaque move: computed here, once per pair, from one
            // register, instead of sixteen loop-invariant addresses kept alive over the whole pair loop)
            int lrow = g16 - padb;
            asm volatile("" : "+v"(lrow));
            real* gq = a.gdx + xi * a.xstride + (long)lrow * a.DS + n16;
            // (the four row tiles advance together: four independent accumulators keep the matrix core busy while the
            // operands of the next step are on their way, and two operands 16 rows apart come with one LDS instruction)
            real4 acc[4];
#pragma unroll
            for (int I = 0; I < 4; ++I) acc[I] = real4{0.0, 0.0, 0.0, 0.0};
            const SK_LDS real* gp = P + (g16 + 1) * kTileStride + n16;
#pragma unroll
            for (int kb = 0; kb < 16; ++kb)
#pragma unroll
                for (int I = 0; I < 4; ++I)
                    acc[I] = __builtin_amdgcn_mfma_f64_16x16x4f64(gp[4 * kb * kTileStride + 16 * I], yc[kb], acc[I], 0, 0, 0);
            // (up: rows above the lane's first one, which is row g16 - padb of the pair.  With at most four rows of
            // padding and every channel in use only the first of the sixteen sums can lie outside the grid.)
            if (padb <= 4 && a.d == 4 * KC) {
#pragma unroll
                for (int I = 0; I < 4; ++I)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int up = 16 * I + 4 * r;
                        if (up > 0 || lrow >= 0) unsafeAtomicAdd(&gq[(long)up * a.DS], acc[I][r]);
                    }
            } else {
#pragma unroll
                for (int I = 0; I < 4; ++I)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const int up = 16 * I + 4 * r;
                        if (lrow + up >= 0 && n16 < a.d) unsafeAtomicAdd(&gq[(long)up * a.DS], acc[I][r]);
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
// launcher
// ------------------------------------------------------------------------------------------------
// The plan counts workgroups of kWavesPerWG independent waves.  The backward kernel runs each of those waves as a
// workgroup of its own (its registers leave room for one wave per SIMD, so four of them share a compute unit all the
// same, and the workgroup's LDS starts at address 0: no base to add); the forward kernel, with fewer registers, would be
// packed unevenly onto the SIMDs that way (measured: 12.5 ms instead of 7.4) and keeps four waves per workgroup.
template <int KC, bool PAIRS>
static hipError_t launch_tile_bwd_p(const SweepArgs& a, int grid, hipStream_t st)
{
    if (hipError_t e = allow_full_lds(reinterpret_cast<const void*>(&tile_bwd_kernel<KC, PAIRS>)); e != hipSuccess) return e;
    hipLaunchKernelGGL((tile_bwd_kernel<KC, PAIRS>), dim3((unsigned)grid * kWavesPerWG), dim3(kWave), a.lds_wave, st, a);
    return hipGetLastError();
}

template <int KC>
static hipError_t launch_tile_bwd_k(const SweepArgs& a, int grid, hipStream_t st)
{
    // two columns per LDS instruction need a zero column behind the zero column nb: P has columns up to 64
    return a.nb + 1 < kTileCols - 1 ? launch_tile_bwd_p<KC, true>(a, grid, st) : launch_tile_bwd_p<KC, false>(a, grid, st);
}

hipError_t launch_tile_bwd(int DT, const SweepArgs& a, int grid, hipStream_t st)
{
    switch (DT) {
        case 8: return launch_tile_bwd_k<2>(a, grid, st);
        case 16: return launch_tile_bwd_k<4>(a, grid, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace sk

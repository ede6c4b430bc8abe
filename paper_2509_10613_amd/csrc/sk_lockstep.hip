// Lock-step cooperative sweeps (gfx950): one workgroup per path pair, used when the batch is too small to
// fill the chip, so that the time of a call is the latency of one pair's chain of macro-steps.
//
// Same decomposition of Eq. (1) as the other sweep kernels (blocks of 2^BL x 2^BL refined cells sharing
// one increment inner product p, a lane per block row, lanes on an anti-diagonal, bottom edges handed from
// lane to lane by DPP; Section 3.3), with three changes that shorten the chain:
//
//  * Two waves per strip.  The stencil wave carries the recurrence and nothing else: per macro-step it reads
//    the coefficients A(p), B(p) of its blocks from a ring in LDS, receives the edge of the lane above, and
//    applies Eq. (1).  The coefficient wave of the strip computes p (the contraction of the lane's x
//    increments with the column's y increments, Eq. (1) third line), A and B one chunk of macro-steps ahead
//    and, in the reverse sweep, also maps dF/dp to the increment gradients one chunk behind (the linear map
//    of Section 3.4).  Nothing on the coefficient wave's side depends on the recurrence.
//  * M block rows per lane (a lane's column of M blocks is swept top to bottom inside one macro-step), so
//    a strip covers 64 M block rows: fewer strips, fewer lane exchanges per cell.
//  * No flags and no waits.  All waves of the workgroup advance in chunks of CH macro-steps separated by
//    workgroup barriers; strip s + 1 runs LAG >= 63 + CH macro-steps behind strip s, so every value it reads
//    from the hand-over row of strip s was written in an earlier chunk.  Hand-over rows hold a whole row
//    of the grid in LDS (this mode is only planned when that fits).
//
// Every lane computes at every macro-step; there is no activity mask.  A lane whose column index
// J = T - lane is outside [0, nb) gets p = 0 from the coefficient wave, i.e. A = B = 1: with the boundary
// value 1 on all its inputs Eq. (1) returns exactly 1, so a lane that has not started yet carries the
// boundary condition k = 1 by itself; a lane that has run past the last column computes values nobody
// uses.  The strips are aligned to the bottom of the grid: the block rows that pad the first strip sit
// above row 0, get p = 0 as well, and so hand the boundary row k[0, .] = 1 down to the first real row.
//
// Backward (Section 3.4): phase 1 is the forward sweep with a checkpoint of the lane state every 8
// macro-steps; the hand-over rows stay in LDS.  Phase 2 is its exact mirror image in time: at mirrored step
// T a lane recovers the nodes of its block column by inverting Eq. (1) from the right and bottom edges
// (bottom edge: the top edge the lane below recovered one step earlier; for the strip's last lane the
// exact row kept from phase 1), scatters the adjoint (first relation of Section 3.4) and forms dF/dp per
// block (second relation).  Every 8 steps the forward state is replaced by the exact checkpoint, after
// comparing the two (at the left end the recovered state is compared with the boundary value 1): a difference above
// kDriftTol of the lane's largest forward value disqualifies the pair - nothing of it reaches the gradients, and it
// is listed for the replay kernel, which solves it once more.  Outside the grid the adjoint is exactly zero (the
// seed dF/dk enters through the adjoint hand-over row under the last strip), and the products of zero with
// the finite values computed there stay zero.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "sk_dev.h"
#include "sk_kernels.h"
#include "sk_lane.h"

namespace sk {

__device__ __forceinline__ void chunk_barrier()
{
    // LDS traffic of this wave has completed; global traffic (checkpoints) may stay in flight
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Roles of the waves of a workgroup.  Waves w and w + 4 of a workgroup share a SIMD, so the stencil waves
// (which carry the serial chain) get the low indices and, for up to two strips, a SIMD of their own; the
// coefficient and gradient waves of two strips share the other two SIMDs.
// Role kRoleCoef computes the coefficients of the strip; kRoleAux is its second helper wave: in forward
// sweeps it takes over half of the coefficient work (then kRoleCoef does the other half), in the reverse sweep
// it maps dF/dp to the increment gradients.
enum { kRoleStencil = 0, kRoleCoef = 1, kRoleAux = 2, kRoleIdle = 3 };
__host__ __device__ inline int lock_waves(int ns) { return ns == 1 ? 3 : (ns == 2 ? 8 : 12); }
__device__ __forceinline__ void lock_role(int w, int ns, int& role, int& strip)
{
    role = kRoleIdle;
    strip = 0;
    if (w < ns) { role = kRoleStencil; strip = w; return; }
    const int c0 = ns <= 2 ? ns : 4;                    // first coefficient wave
    if (w >= c0 && w < c0 + ns) { role = kRoleCoef; strip = w - c0; return; }
    const int g0 = ns == 1 ? 2 : (ns == 2 ? 6 : 8);     // first auxiliary wave
    if (w >= g0 && w < g0 + ns) { role = kRoleAux; strip = w - g0; }
}

// LDS carve-up shared by both kernels
struct LockLds {
    SK_LDS real* y;
    SK_LDS real* gy;
    SK_LDS real* cring;   // this strip's coefficient ring
    SK_LDS real* gp;      // this strip's dF/dp ring
    SK_LDS real* krows;
    SK_LDS real* arows;
    SK_LDS real* dump;
    SK_LDS real* ck;      // this strip's checkpoint staging buffer (backward)
};

__device__ __forceinline__ LockLds carve_lock_lds(unsigned char* smem, const SweepArgs& a, int strip)
{
    LockLds l;
    l.y = (SK_LDS real*)(smem + a.lk_off_y);
    l.gy = (SK_LDS real*)(smem + a.lk_off_gy);
    l.cring = (SK_LDS real*)(smem + a.lk_off_cring + (size_t)strip * a.lk_cring_stride);
    l.gp = (SK_LDS real*)(smem + a.lk_off_gp + (size_t)strip * a.lk_gp_stride);
    l.krows = (SK_LDS real*)(smem + a.lk_off_krows);
    l.arows = (SK_LDS real*)(smem + a.lk_off_arows);
    l.dump = (SK_LDS real*)(smem + a.lk_off_dump);
    l.ck = (SK_LDS real*)(smem + a.lk_off_ck + (size_t)strip * a.lk_ck_stride);
    return l;
}

// y increments of the pair into LDS ([q][DSc], channels beyond d zero), from the increment workspace or, in
// fused mode, from the caller's points (first line of the paper's forward listing).
template <int DSc, bool ZERO_G>
__device__ __forceinline__ void stage_y(const SweepArgs& a, long yi, SK_LDS real* y, SK_LDS real* gy)
{
    const int n = a.q * DSc;
    if (a.fused) {
        const real* yp = a.yraw + yi * (long)a.L2 * a.d;
        for (int t = threadIdx.x; t < n; t += blockDim.x) {
            const int b = t / DSc, c = t - b * DSc;
            y[t] = c < a.d ? yp[(long)(b + 1) * a.d + c] - yp[(long)b * a.d + c] : 0.0;
            if (ZERO_G) gy[t] = 0.0;
        }
    } else {
        const real* dyg = a.dy + yi * a.ystride;
        for (int t = threadIdx.x; t < n; t += blockDim.x) {
            y[t] = dyg[t];
            if (ZERO_G) gy[t] = 0.0;
        }
    }
}

// ------------------------------------------------------------------------------------------------
// forward
// ------------------------------------------------------------------------------------------------
template <int BL, int D, int M, int LL>
__global__ __launch_bounds__(12 * kWave) void lock_fwd_kernel(SweepArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    using LK = Lock<BL, D, M, LL>;
    constexpr int C = LK::C, CH = LK::CH1;
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int ns = a.lk_ns;
    int role, strip;
    lock_role(w, ns, role, strip);
    const LockLds l = carve_lock_lds(smem, a, strip);
    const long pid = blockIdx.x;
    long xi, yi;
    pair_ids(a, pid, xi, yi);
    const real* dxp = a.fused ? a.xraw + xi * (long)a.L1 * a.d : a.dx + xi * a.xstride;
    const int rowlen = a.lk_rowlen;

    stage_y<LK::DSc, false>(a, yi, l.y, l.y);
    for (int t = threadIdx.x; t < (ns + 1) * rowlen; t += blockDim.x) l.krows[t] = 1.0;
    __syncthreads();

    const int nck = a.lk_NT / CH;
    const int lagc = kLockLag1 / CH;
    const int niter = nck + (ns - 1) * lagc;
    const SK_LDS real* rowprev = l.krows + strip * rowlen + LK::PADF;   // row above the strip (ones for strip 0)
    SK_LDS real* rowcur = l.krows + (strip + 1) * rowlen + LK::PADF;

    typename LK::Fwd f;
    typename LK::Coef cf;
    typename LK::Off off;   // lead-lag blocks: the stencil wave's own coefficients of the off-diagonal quadrants
    constexpr int kSplit = 1;   // two coefficient waves per strip
    if (role == kRoleCoef || role == kRoleAux) cf.setup(a, strip, lane, dxp, l.y);
    else f.init();
    off.setup(a, strip, lane);

    for (int g = -1; g < niter; ++g) {
        const int lc = g - strip * lagc;
        if (role == kRoleStencil) {
            if (lc >= 0 && lc < nck) f.chunk(lc * CH, lane, l.cring + (lc & 1) * LK::CR1, rowprev, rowcur, l.dump, off);
        } else if (role == kRoleCoef || (kSplit && role == kRoleAux)) {
            const int hc = lc + 1;
            if (hc >= 0 && hc < nck)
                cf.produce_fwd(hc * CH, l.cring + (hc & 1) * LK::CR1, kSplit ? (role == kRoleCoef ? 1 : 2) : 0);
        }
        chunk_barrier();
    }
    // k[m, n]: the last node of the last strip's bottom row
    if (threadIdx.x == 0) a.k_out[pid] = l.krows[ns * rowlen + LK::PADF + a.nb * C];
}

// ------------------------------------------------------------------------------------------------
// backward
// ------------------------------------------------------------------------------------------------
// PHASE 0: the whole backward call.  PHASE 1 / 2: its two halves as launches of their own (a forward call whose
// sweep is kept, and the backward call that follows it): what crosses from phase 1 to phase 2 is the checkpoints,
// which are in global memory anyway, and the hand-over rows, which phase 1 then copies out and phase 2 copies in.
template <int BL, int D, int M, int PHASE, int LL>
__global__ __launch_bounds__(8 * kWave) void lock_bwd_kernel(SweepArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    using LK = Lock<BL, D, M, LL>;
    constexpr int C = LK::C, RR = LK::RR, NVC = LK::NVC, CH1 = LK::CH1, CH2 = LK::CH2;
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int ns = a.lk_ns;
    int role, strip;
    lock_role(w, ns, role, strip);
    const bool stencil = role == kRoleStencil;
    const LockLds l = carve_lock_lds(smem, a, strip);
    const long pid = blockIdx.x;
    long xi, yi;
    pair_ids(a, pid, xi, yi);
    const real* dxp = a.fused ? a.xraw + xi * (long)a.L1 * a.d : a.dx + xi * a.xstride;
    real* gdx = a.fused ? nullptr : a.gdx + xi * a.xstride;
    real* gdy = a.fused ? nullptr : a.gdy + yi * a.ystride;
    const int rowlen = a.lk_rowlen;
    const int nckS = a.lk_NT / kLockS;   // checkpoints per strip: nckS + 1
    real* ckpt = a.ckpt + pid * a.ckpt_slot + (long)strip * (nckS + 1) * NVC * kWave + lane;

    stage_y<LK::DSc, true>(a, yi, l.y, l.gy);
    real* keep = PHASE == 0 ? nullptr : a.lk_keep + pid * (long)(ns + 1) * rowlen;
    if constexpr (PHASE == 2) {
        // the kept rows, 16 bytes per access and four accesses in flight per thread (rowlen is even, the rows' place
        // in the workspace 256-byte aligned)
        const int n2 = ((ns + 1) * rowlen) >> 1;
        const real2* kp = reinterpret_cast<const real2*>(keep);
        SK_LDS real2* kr = (SK_LDS real2*)l.krows;
        SK_LDS real2* ar = (SK_LDS real2*)l.arows;
        const int stride = blockDim.x;
        for (int t0 = threadIdx.x; t0 < n2; t0 += 4 * stride) {
            real2 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = t0 + u * stride < n2 ? kp[t0 + u * stride] : real2{0.0, 0.0};
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                if (t0 + u * stride < n2) { kr[t0 + u * stride] = v[u]; ar[t0 + u * stride] = real2{0.0, 0.0}; }
            }
        }
    } else {
        for (int t = threadIdx.x; t < (ns + 1) * rowlen; t += blockDim.x) { l.krows[t] = 1.0; l.arows[t] = 0.0; }
    }
    __syncthreads();
    // dF/dk[m, n] enters through the adjoint row under the last strip
    if (PHASE != 1 && threadIdx.x == 0) l.arows[ns * rowlen + LK::PADF + (a.nb - 1) * C + (C - 1)] = a.grad_k[pid];

    const SK_LDS real* rowprev = l.krows + strip * rowlen + LK::PADF;
    SK_LDS real* rowcur = l.krows + (strip + 1) * rowlen + LK::PADF;
    const SK_LDS real* arow_in = l.arows + (strip + 1) * rowlen + LK::PADF;   // written by the strip below
    SK_LDS real* arow_out = l.arows + strip * rowlen + LK::PADF;               // read by the strip above

    typename LK::Coef cf;
    typename LK::Off off;   // lead-lag blocks: the stencil wave's own coefficients of the off-diagonal quadrants
    constexpr int kSplit = 1;   // two coefficient waves per strip in the forward phase
    if (role == kRoleCoef || role == kRoleAux) cf.setup(a, strip, lane, dxp, l.y);
    off.setup(a, strip, lane);

    // ---- phase 1: forward with checkpoints ----
    if constexpr (PHASE != 2) {
        typename LK::Fwd f;
        f.init();
        const int nck = a.lk_NT / CH1;
        const int lagc = kLockLag1 / CH1;
        const int niter = nck + (ns - 1) * lagc;
        for (int g = -1; g < niter; ++g) {
            const int lc = g - strip * lagc;
            if (stencil) {
                if (lc >= 0 && lc < nck) {
                    f.store_ckpt(ckpt + (long)lc * NVC * kWave);   // kLockS == CH1: one checkpoint per chunk
                    f.chunk(lc * CH1, lane, l.cring + (lc & 1) * LK::CR1, rowprev, rowcur, l.dump, off);
                    if (lc == nck - 1) f.store_ckpt(ckpt + (long)nck * NVC * kWave);
                }
            } else if (role == kRoleCoef || (kSplit && role == kRoleAux)) {
                const int hc = lc + 1;
                if (hc >= 0 && hc < nck)
                    cf.produce_fwd(hc * CH1, l.cring + (hc & 1) * LK::CR1, kSplit ? (role == kRoleCoef ? 1 : 2) : 0);
            }
            chunk_barrier();
        }
    }
    if (threadIdx.x == 0 && a.k_out) a.k_out[pid] = l.krows[ns * rowlen + LK::PADF + a.nb * C];
    __syncthreads();   // also completes the checkpoint stores before they are read back
    if constexpr (PHASE == 1) {
        for (int t = threadIdx.x; t < (ns + 1) * rowlen; t += blockDim.x) keep[t] = l.krows[t];
        if (pid == 0 && threadIdx.x == 0) *a.keep_tag = a.keep_tag_val;
        return;
    }
    // both sweeps in one call: whatever sweep the workspace held is gone
    if (PHASE == 0 && a.keep_tag && pid == 0 && threadIdx.x == 0) *a.keep_tag = 0;
    // the reverse sweep alone: is the sweep in the workspace the one of this call's arguments?
    bool stale = false;
    if (PHASE == 2 && threadIdx.x == 0) stale = *a.keep_tag != a.keep_tag_val;

    // ---- phase 2: the mirror image ----
    real gacc[M][D];
#pragma unroll
    for (int m = 0; m < M; ++m)
#pragma unroll
        for (int c = 0; c < D; ++c) gacc[m][c] = 0.0;
    // Drift of the recovered forward values against the exact checkpoints, measured against the largest
    // forward value this lane has met (the gradients are sums of products of adjoints with forward values,
    // and are checked against their own largest entry).
    bool drift = false;
    {
        typename LK::Rev rv;
        rv.init();
        const int nck = a.lk_NT / CH2;
        const int lagc = kLockLag2 / CH2;
        const int niter = nck + (ns - 1) * lagc;
        const int rs = ns - 1 - strip;   // strips start bottom-up
        real kscale = 1.0;
        // Checkpoints reach the stencil wave through LDS: the coefficient wave of the strip loads checkpoint idx
        // from global memory three chunks before it is needed, writes it into half (idx & 1) of the strip's
        // staging buffer two chunks later, and the stencil wave reads it after the next barrier.  Stored per
        // lane: the lane's right edge (RR + 1 values), then the bottom edge of the lane above with its left
        // corner (C values), which that lane takes over this lane's top edge hand-over.
        constexpr int NVS = RR + 1 + C;
        SK_LDS real* ckl = l.ck + lane;
        real ckr[NVS];
        const int up1 = lane > 0 ? -1 : 0;
        auto load_ckpt = [&](int idx) {
            const real* cp = ckpt + (long)idx * NVC * kWave;
#pragma unroll
            for (int q = 0; q <= RR; ++q) ckr[q] = ld_scratch(cp + q * kWave);
            ckr[RR + 1] = ld_scratch(cp + (RR + 1 + C) * kWave + up1);                                // corner
#pragma unroll
            for (int q = 1; q < C; ++q) ckr[RR + 1 + q] = ld_scratch(cp + (RR + 1 + q - 1) * kWave + up1);
        };
        if (role == kRoleCoef) load_ckpt(nckS);
        auto rev_chunk = [&](auto restore_c, int fc, int rc) {
            constexpr bool RESTORE = decltype(restore_c)::value;
            if constexpr (RESTORE) {
                const int idx = (fc + 1) / 2;
                const SK_LDS real* cs = ckl + (idx & 1) * (NVS * kWave);
                real cv[NVS];
#pragma unroll
                for (int i = 0; i < NVS; ++i) cv[i] = cs[i * kWave];
#pragma unroll
                for (int i = 0; i <= RR; ++i) kscale = fmax(kscale, fabs(cv[i]));
                if (rc > 0) {
#pragma unroll
                    for (int i = 0; i <= RR; ++i)   // written so that a NaN counts as drift
                        if (!(fabs(rv.kR[i] - cv[i]) <= kDriftTol * kscale)) drift = true;
                }
#pragma unroll
                for (int i = 0; i <= RR; ++i) rv.kR[i] = cv[i];
#pragma unroll
                for (int i = 0; i < C; ++i) rv.ktop[i] = cv[RR + 1 + i];
            }
            rv.chunk(fc * CH2, lane, l.cring + (rc & 1) * LK::CR2, arow_in, rowcur, arow_out, l.dump,
                     l.gp + (rc & 1) * LK::GPH, off);
        };
        for (int g = -1; g <= niter; ++g) {
            const int rc = g - rs * lagc;
            if (stencil) {
                if (rc >= 0 && rc < nck) {
                    const int fc = nck - 1 - rc;
                    if (fc & 1) rev_chunk(std::true_type(), fc, rc);
                    else rev_chunk(std::false_type(), fc, rc);
                }
            } else if (role == kRoleCoef) {
                const int hc = rc + 1, gc = rc - 1;
                // the stencil wave restores checkpoint idx in reverse chunk nck - 2 idx: stage it one chunk before
                if (rc >= -1 && ((nck - rc - 1) & 1) == 0) {
                    const int idx = (nck - rc - 1) / 2;
                    if (idx >= 1) {
                        SK_LDS real* cs = ckl + (idx & 1) * (NVS * kWave);
#pragma unroll
                        for (int i = 0; i < NVS; ++i) cs[i * kWave] = ckr[i];
                        if (idx >= 2) load_ckpt(idx - 1);
                    }
                }
                if (hc >= 0 && hc < nck) cf.produce_rev((nck - 1 - hc) * CH2, l.cring + (hc & 1) * LK::CR2);
                if (a.want_gx && gc >= 0 && gc < nck)
                    cf.consume_gx((nck - 1 - gc) * CH2, l.gp + (gc & 1) * LK::GPH, gacc);
            } else if (role == kRoleAux) {
                const int gc = rc - 1;
                if (a.want_gy && gc >= 0 && gc < nck) cf.consume_gy((nck - 1 - gc) * CH2, l.gp + (gc & 1) * LK::GPH, l.gy);
            }
            chunk_barrier();
        }
        if (stencil) {   // the left end: every strip started from the boundary value 1 in every lane
#pragma unroll
            for (int i = 0; i <= RR; ++i)
                if (!(fabs(rv.kR[i] - 1.0) <= kDriftTol * kscale)) drift = true;
        }
    }
    // The rings are free now.  In the fused form their memory collects the gradients with respect to the x
    // increments, [r][DSc]; two ints of the dump row say how the pair went.
    SK_LDS real* gxl = (SK_LDS real*)(smem + a.lk_off_cring);
    SK_LDS int* bad = (SK_LDS int*)l.dump;   // [0]: the inverse recurrence drifted, [1]: not this call's forward sweep
    if (a.fused) {
        for (int t = threadIdx.x; t < a.r * LK::DSc; t += blockDim.x) gxl[t] = 0.0;
    }
    if (threadIdx.x == 0) { bad[0] = 0; bad[1] = stale ? 1 : 0; }
    __syncthreads();
    if (stencil) {
        if (drift) bad[0] = 1;
    } else if (a.fused && role == kRoleCoef && a.want_gx) {
#pragma unroll
        for (int m = 0; m < M; ++m) {
            const int I = (strip * kWave + lane) * M + m - a.lk_padb;
            if (I >= 0) {
                SK_LDS real* gq = gxl + (I >> a.rs1) * LK::DSc;
#pragma unroll
                for (int c = 0; c < D; ++c) lds_atomic_add(gq + c, gacc[m][c] * a.sc);
            }
        }
    }
    __syncthreads();
    const bool is_stale = bad[1] != 0;
    if (bad[0] != 0 && !is_stale) {
        // A drifted pair adds nothing to the gradients: it is listed for the replay kernel, which solves it once more
        // (and, in the fused form, writes the pair's gradients itself).
        if (threadIdx.x == 0) list_drifted(a, pid, pid);
        return;
    }
    if (!a.fused) {
        if (role == kRoleCoef && a.want_gx) {
#pragma unroll
            for (int m = 0; m < M; ++m) {
                const int I = (strip * kWave + lane) * M + m - a.lk_padb;
                if (I >= 0) {
                    real* gq = gdx + (long)(I >> a.rs1) * LK::DSc;
#pragma unroll
                    for (int c = 0; c < D; ++c) unsafeAtomicAdd(gq + c, gacc[m][c] * a.sc);
                }
            }
        }
        if (a.want_gy) {
            const int n = a.q * LK::DSc;
            for (int t = threadIdx.x; t < n; t += blockDim.x) {
                const real v = l.gy[t];
                if (v != 0.0) unsafeAtomicAdd(&gdy[t], v);
            }
        }
    } else {
        // The increments are differences of consecutive points, so the gradient of a point collects the two
        // increments it touches (the linear map of Section 3.4).  A reverse sweep that found another call's forward
        // sweep in the workspace returns NaN.
        const real nan = __builtin_nan("");
        const int d = a.d;
        if (a.gxraw) {
            real* go = a.gxraw + xi * (long)a.L1 * d;
            for (int t = threadIdx.x; t < a.L1 * d; t += blockDim.x) {
                const int pt = t / d, c = t - pt * d;
                const real hi = pt >= 1 ? gxl[(pt - 1) * LK::DSc + c] : 0.0;
                const real lo = pt < a.L1 - 1 ? gxl[pt * LK::DSc + c] : 0.0;
                go[t] = is_stale ? nan : hi - lo;
            }
        }
        if (a.gyraw) {
            real* go = a.gyraw + yi * (long)a.L2 * d;
            for (int t = threadIdx.x; t < a.L2 * d; t += blockDim.x) {
                const int pt = t / d, c = t - pt * d;
                const real hi = pt >= 1 ? l.gy[(pt - 1) * LK::DSc + c] : 0.0;
                const real lo = pt < a.L2 - 1 ? l.gy[pt * LK::DSc + c] : 0.0;
                go[t] = is_stale ? nan : hi - lo;
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// launchers
// ------------------------------------------------------------------------------------------------
template <int BL, int D, int M, int LL>
hipError_t launch_lock_fwd(const SweepArgs& a, int grid, size_t lds, hipStream_t st)
{
    if (hipError_t e = allow_full_lds(reinterpret_cast<const void*>(&lock_fwd_kernel<BL, D, M, LL>)); e != hipSuccess) return e;
    hipLaunchKernelGGL((lock_fwd_kernel<BL, D, M, LL>), dim3(grid), dim3(lock_waves(a.lk_ns) * kWave), lds, st, a);
    return hipGetLastError();
}

template <int BL, int D, int M, int PHASE, int LL>
hipError_t launch_lock_bwd_phase(const SweepArgs& a, int grid, size_t lds, hipStream_t st)
{
    if (hipError_t e = allow_full_lds(reinterpret_cast<const void*>(&lock_bwd_kernel<BL, D, M, PHASE, LL>)); e != hipSuccess) return e;
    hipLaunchKernelGGL((lock_bwd_kernel<BL, D, M, PHASE, LL>), dim3(grid), dim3(lock_waves(a.lk_ns) * kWave), lds, st, a);
    return hipGetLastError();
}

template <int BL, int D, int M, int LL>
hipError_t launch_lock_bwd(const SweepArgs& a, int grid, size_t lds, hipStream_t st)
{
    if (a.lk_phase == 0) return launch_lock_bwd_phase<BL, D, M, 0, LL>(a, grid, lds, st);
    // the halves exist for the calls that work on the caller's arrays, and need the rows' place in global memory
    if (!a.fused || !a.lk_keep || !a.keep_tag) return hipErrorInvalidValue;
    if (a.lk_phase == 1) return launch_lock_bwd_phase<BL, D, M, 1, LL>(a, grid, lds, st);
    if (a.lk_phase == 2) return launch_lock_bwd_phase<BL, D, M, 2, LL>(a, grid, lds, st);
    return hipErrorInvalidValue;
}

// Two block rows per lane are only built where the registers allow it (lock_max_rows in sk_plan.h).
template <int BL, int D, int LL>
hipError_t launch_lock_m(bool backward, const SweepArgs& a, int grid, size_t lds, hipStream_t st)
{
    if (a.lk_M > lock_max_rows(backward, BL, D)) return hipErrorInvalidValue;
    if (backward) {
        if constexpr (lock_max_rows(true, BL, D) >= 1) {
            if (a.lk_M == 1) return launch_lock_bwd<BL, D, 1, LL>(a, grid, lds, st);
        }
        if constexpr (lock_max_rows(true, BL, D) >= 2) return launch_lock_bwd<BL, D, 2, LL>(a, grid, lds, st);
    } else {
        if (a.lk_M == 1) return launch_lock_fwd<BL, D, 1, LL>(a, grid, lds, st);
        if constexpr (lock_max_rows(false, BL, D) >= 2) return launch_lock_fwd<BL, D, 2, LL>(a, grid, lds, st);
    }
    return hipErrorInvalidValue;
}

// lead-lag form of the sweep (SweepArgs::ll): inside the blocks (1) for blocks that hold every refined cell of a pair
// of increments, above them (2) otherwise
template <int BL, int D>
hipError_t launch_lock_ll(bool backward, const SweepArgs& a, int grid, size_t lds, hipStream_t st)
{
    if (a.ll == 0) return launch_lock_m<BL, D, 0>(backward, a, grid, lds, st);
    if constexpr (BL >= 1) {
        if (a.ll == 1 && a.rs1 == 0 && a.rs2 == 0) return launch_lock_m<BL, D, 1>(backward, a, grid, lds, st);
    }
    if (a.ll == 2 && a.rs1 >= 1 && a.rs2 >= 1) return launch_lock_m<BL, D, 2>(backward, a, grid, lds, st);
    return hipErrorInvalidValue;
}

template <int BL>
hipError_t launch_lock_bl(bool backward, int DT, const SweepArgs& a, int grid, size_t lds, hipStream_t st)
{
    switch (DT) {
#ifndef SK_ONLY_C2   /* development builds instantiate a single shape */
        case 2: return launch_lock_ll<BL, 2>(backward, a, grid, lds, st);
        case 3: return launch_lock_ll<BL, 3>(backward, a, grid, lds, st);
        case 4: return launch_lock_ll<BL, 4>(backward, a, grid, lds, st);
        case 6: return launch_lock_ll<BL, 6>(backward, a, grid, lds, st);
        case 8: return launch_lock_ll<BL, 8>(backward, a, grid, lds, st);
        case 16: return launch_lock_ll<BL, 16>(backward, a, grid, lds, st);
#endif
        case 5: return launch_lock_ll<BL, 5>(backward, a, grid, lds, st);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_sweep_lockstep(bool backward, int BL, int DT, const SweepArgs& a, int grid, size_t lds,
                                 hipStream_t st)
{
    if (a.lk_ns < 1 || a.lk_ns > (backward ? kLockMaxStripsBwd : kLockMaxStrips) || (a.lk_NT & 7) != 0 ||
        (backward && a.lk_phase != 1 && (!a.bad_list || !a.bad_count)))
        return hipErrorInvalidValue;
    switch (BL) {
#ifndef SK_ONLY_C2
        case 0: return launch_lock_bl<0>(backward, DT, a, grid, lds, st);
        case 2: return launch_lock_bl<2>(backward, DT, a, grid, lds, st);
#endif
        case 1: return launch_lock_bl<1>(backward, DT, a, grid, lds, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace sk

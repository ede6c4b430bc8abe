// Band sweeps (gfx950): a few pairs of long paths (many strips of 64 block rows per pair, far fewer pairs than
// compute units).  One workgroup per band of kBandStrips consecutive strips; the bands of a pair run on
// different compute units at the same time, as one pipeline: strip s + 1 follows strip s at a fixed lag of
// macro-steps, inside a workgroup (hand-over through a small ring in LDS, all waves advancing in chunks of
// macro-steps separated by barriers, as in the lock-step kernels) and across workgroups (hand-over through a
// row in global memory and a progress counter).  The cells of an anti-diagonal are independent (Section 3.3);
// here the anti-diagonal of blocks is cut into strips that are all in flight, instead of one strip of 32
// rows per pair at a time.
//
// Roles.  Waves 0 .. kBandStrips - 1 each carry one strip: the contraction of the lane's x increments with
// the column's y increments (Eq. (1), third line), the coefficients, the recurrence, and in the reverse sweep
// the adjoint recurrence and the linear map of Section 3.4.  The last wave moves data: y increments of the
// coming columns into a ring in LDS (the four strips of a band touch a window of about 300 columns), the row
// above the band from global memory into the first strip's hand-over ring, finished pieces of the strips'
// bottom rows out to global memory, and it is the only wave that ever waits for another workgroup.  Every
// such wait is bounded: when it runs out the call's error flag is raised, the wave goes on, and the
// finalisation returns NaN gradients; no wave can hang.
//
// Order.  Workgroup index = band * pairs + pair in the forward kernel: a band only waits for the band before
// it, which has a smaller index and was dispatched earlier.  The reverse sweep is a launch of its own with
// the bands in the opposite order, for the same reason.
//
// Visibility between workgroups: the rows and counters that cross workgroups are written and read with
// agent-scope atomic accesses (they bypass the per-compute-unit cache and are coherent at the device's L2 /
// memory side); the writer waits for its stores to complete before it advances the counter.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "sk_dev.h"
#include "sk_kernels.h"
#include "sk_lane.h"

namespace sk {

__device__ __forceinline__ void band_barrier()
{
    // LDS traffic of this wave has completed; global traffic may stay in flight
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

__device__ __forceinline__ void st_agent(real* p, real v)
{
    __hip_atomic_store(reinterpret_cast<unsigned long long*>(p), (unsigned long long)__double_as_longlong(v),
                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int ld_agent_int(const int* p)
{
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_agent_int(int* p, int v)
{
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Every vector memory operation this wave has issued has completed (stores acknowledged).  The rows that cross
// workgroups are written with agent-scope atomic stores and read with agent-scope atomic loads, which are
// coherent at the device's memory side by themselves (no cache has to be written back or invalidated); what
// is left to do is to keep the order: a counter is advanced only after the data it announces has arrived.
__device__ __forceinline__ void stores_done() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Polls *ctr until it is at least `want` (bounded).  Returns the last value read (below `want`: the wait ran out).
__device__ __forceinline__ int wait_progress(const int* ctr, int want, int limit)
{
    int v = ld_agent_int(ctr);
    for (int spin = 1; v < want && spin < limit; ++spin) {
        __builtin_amdgcn_s_sleep(4);
        v = ld_agent_int(ctr);
    }
    return v;
}

template <int BL, int D, int LL>
struct Band {
    using LK = Lock<BL, D, 1, LL>;
    static constexpr int C = LK::C, DSc = LK::DSc;
    static constexpr int RM = kBandRing - 1, YM = kBandYRing - 1;

    // y increments of the block column lane `lane` is at in macro-step T, from the ring
    template <bool EDGE>
    static __device__ __forceinline__ void fetch(const typename LK::Coef& cf, const SK_LDS real* yring, int T, int& J,
                                                 int& b, real (&y)[D])
    {
        J = T - cf.lane;
        b = (EDGE ? clamp_col(J, cf.nbm1) : J) >> cf.rs2;
        const SK_LDS real* yp = yring + __mul24(b & YM, DSc);
#pragma unroll
        for (int c = 0; c < D; ++c) y[c] = yp[c];
    }
};

// ------------------------------------------------------------------------------------------------
// forward (CKPT: phase 1 of the backward pass: checkpoints and every strip's bottom row go to global memory)
// ------------------------------------------------------------------------------------------------
template <int BL, int D, bool CKPT, int LL>
__global__ __launch_bounds__((kBandStrips + 1) * kWave, 1) void band_fwd_kernel(SweepArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    using BD = Band<BL, D, LL>;
    using LK = Lock<BL, D, 1, LL>;
    constexpr int C = LK::C, DSc = LK::DSc, CH = kLockCH1, NVC = LK::NVC, SPB = kBandStrips;
    constexpr int RM = BD::RM, YM = BD::YM;
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int npairs = (int)a.npairs;
    const int band = blockIdx.x / npairs;
    const long pid = blockIdx.x - band * npairs;
    long xi, yi;
    pair_ids(a, pid, xi, yi);
    SK_LDS real* yring = (SK_LDS real*)(smem + a.bd_off_y);
    SK_LDS real* rings = (SK_LDS real*)(smem + a.bd_off_rings);   // [SPB + 1][kBandRing][C]: ring s is read by strip s
    const int ns = a.lk_ns, nb = a.nb;
    // A strip's last lane visits block columns up to nbx - 1, a few beyond the grid (the macro-steps are rounded up to
    // whole chunks).  The values it computes there are of no interest by themselves, but the reverse sweep inverts
    // those macro-steps too and needs them under the last lane exactly as they were: the bottom rows cover them.
    const int nbx = a.lk_NT - (kWave - 1);
    const int s0 = band * SPB;
    const int nsw = ns - s0 < SPB ? ns - s0 : SPB;   // strips of this band
    const int nck = a.lk_NT / CH;
    const int lagc = kLockLag1 / CH;
    const int niter = nck + (SPB - 1) * lagc;
    real* rowsg = a.rows + pid * a.rows_slot;        // [ns][rowlen], by node column
    int* prog = a.bd_flags + pid * a.bd_nbands;      // per band: chunks of its last strip whose row is in global memory

    for (int t = threadIdx.x; t < (SPB + 1) * kBandRing * C; t += blockDim.x) rings[t] = 1.0;
    __syncthreads();

    if (w < SPB) {
        // ---------------- a strip ----------------
        const int sg = s0 + w;
        const bool active = w < nsw;
        const bool laststrip = sg == ns - 1;
        typename LK::Coef cf;
        typename LK::Fwd f;
        cf.setup(a, active ? sg : 0, lane, a.dx + xi * a.xstride, yring);
        f.init();
        real kfin = 0.0;   // k[m, n], in the last lane of the pair's last strip
        const SK_LDS real* rin = rings + w * (kBandRing * C);
        SK_LDS real* rout = rings + (w + 1) * (kBandRing * C);
        real* ckpt = CKPT ? a.ckpt + pid * a.ckpt_slot + (long)sg * (nck + 1) * NVC * kWave + lane : nullptr;

        auto chunk = [&](auto edge_c, int T0) {
            constexpr bool EDGE = decltype(edge_c)::value;
            // top edge of the strip's first lane for the whole chunk (the row above the strip)
            real edge[CH][C];
#pragma unroll
            for (int i = 0; i < CH; ++i)
#pragma unroll
                for (int cc = 0; cc < C; ++cc) edge[i][cc] = 1.0;
            if (lane == 0) {
#pragma unroll
                for (int i = 0; i < CH; ++i)
#pragma unroll
                    for (int cc = 0; cc < C; ++cc) edge[i][cc] = rin[((T0 + i) & RM) * C + cc];
            }
            int J[2], b[2];
            real y[2][D];
            BD::template fetch<EDGE>(cf, yring, T0, J[0], b[0], y[0]);
#pragma unroll
            for (int i = 0; i < CH; ++i) {
                if (i + 1 < CH) BD::template fetch<EDGE>(cf, yring, T0 + i + 1, J[(i + 1) & 1], b[(i + 1) & 1], y[(i + 1) & 1]);
                real Ac[1], Bc[1], A0[1], B0[1];
                LK::coef_fwd(cf.template inner<EDGE>(0, J[i & 1], y[i & 1]), Ac[0], Bc[0]);
                if constexpr (LL == 1) LK::coef_fwd(cf.template inner_off<EDGE>(0, J[i & 1]), A0[0], B0[0]);
                else { A0[0] = Ac[0]; B0[0] = Bc[0]; }
                real recv[C];
#pragma unroll
                for (int cc = 0; cc < C; ++cc) recv[cc] = wave_from_above_or(f.bot[cc], edge[i][cc]);
                f.step(recv, Ac, Bc, A0, B0);
                if (lane == kWave - 1) {
                    const int Jw = T0 + i - (kWave - 1);
                    if (!EDGE || Jw >= 0) {
#pragma unroll
                        for (int cc = 0; cc < C; ++cc) rout[(Jw & RM) * C + cc] = f.bot[cc];
                        if (EDGE && Jw == nb - 1) kfin = f.bot[C - 1];
                    }
                }
            }
        };

        for (int g = -kBandLead; g <= niter + 1; ++g) {
            const int lc = g - w * lagc;
            if (active && lc >= 0 && lc < nck) {
                if (CKPT) f.store_ckpt(ckpt + (long)lc * NVC * kWave);
                if (cf.interior(lc * CH, CH)) chunk(std::false_type(), lc * CH);
                else chunk(std::true_type(), lc * CH);
                if (CKPT && lc == nck - 1) f.store_ckpt(ckpt + (long)nck * NVC * kWave);
            }
            band_barrier();
        }
        // A wait that ran out in this band or in one above it (their counters were read after their flag was set)
        // leaves rows that were never written behind: the value is not to be trusted.
        if (laststrip && active && lane == kWave - 1 && a.k_out)
            a.k_out[pid] = ld_agent_int(a.err) != 0 ? __builtin_nan("") : kfin;
    } else {
        // ---------------- the data-moving wave ----------------
        const real* dyg = a.dy + yi * a.ystride;
        const real* rowprev = band > 0 ? rowsg + (long)(s0 - 1) * a.rowlen : nullptr;
        const int* progprev = band > 0 ? prog + band - 1 : nullptr;
        const bool publish = band < a.bd_nbands - 1;
        int ynext = 0;              // next coarse y column to stage
        int yh0 = 0, yhn = 0;       // columns [yh0, yh0 + yhn) are held in registers, on their way into the ring
        real yh[2] = {0.0, 0.0};
        real inh = 1.0;             // one value of the incoming row piece held in registers
        int seen = 0;               // progress of the band above, as last read
        int pub = 0;                // progress of this band to announce at the start of the next iteration
        bool dead = false;
        if (CKPT && lane < nsw) st_agent(rowsg + (long)(s0 + lane) * a.rowlen, 1.0);   // node column 0 of each row

        for (int g = -kBandLead; g <= niter + 1; ++g) {
            // (0) the row pieces written out in the last iteration have had a whole chunk to arrive: announce them
            if (pub > 0) {
                stores_done();
                if (lane == 0) st_agent_int(prog + band, pub);
                pub = 0;
            }
            // (1) y increments: what was loaded in the last iteration goes into the ring; columns for the first
            //     strip's chunk g + 2 are requested (block columns up to (g + 2) CH + CH - 1)
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int t = lane + u * kWave;
                if (t < yhn * DSc) yring[__mul24((yh0 + t / DSc) & YM, DSc) + t % DSc] = yh[u];
            }
            {
                const int cneed = g + 2;
                int upto = cneed >= 0 ? (((cneed + 1) * CH - 1) >> a.rs2) + 1 : 0;
                if (upto > a.q) upto = a.q;
                int n = upto - ynext;
                if (n > CH) n = CH;           // at most CH columns (2 values per lane) per iteration
                if (n < 0) n = 0;
                yh0 = ynext; yhn = n; ynext += n;
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const int t = lane + u * kWave;
                    if (t < n * DSc) yh[u] = dyg[(long)yh0 * DSc + t];
                }
            }
            // (2) the row above the band: the piece for the first strip's chunk g + 1 (loaded in the last
            //     iteration) goes into ring 0; the piece for chunk g + 2 is requested once the band above has it
            if (band > 0) {
                const int cw = g + 1;
                if (cw >= 0 && cw < nck && lane < CH * C) rings[((cw * CH + lane / C) & RM) * C + lane % C] = inh;
                const int cr = g + 2;
                if (cr >= 0 && cr < nck) {
                    // nodes of block columns [cr CH, cr CH + CH): written by the upper strip's chunks <= cr + 8
                    int need = cr + 9;
                    if (need > nck) need = nck;
                    if (seen < need && !dead) {
                        // ask for some chunks more than needed, so that the counter is read once in a while and
                        // not in every iteration (a read is a round trip to the memory side)
                        int want = need + kBandSlack;
                        if (want > nck) want = nck;
                        seen = wait_progress(progprev, want, a.bd_spin);
                        if (seen < need) {
                            dead = true;
                            if (lane == 0) atomicExch(a.err, 1);
                        }
                    }
                    const int col = cr * CH + lane / C;
                    inh = (lane < CH * C && col < nbx) ? ld_scratch(rowprev + (long)col * C + 1 + lane % C) : 1.0;
                }
            }
            // (3) bottom rows: the pieces the strips finished in the last iteration go out to global memory
#pragma unroll
            for (int u = 0; u < (SPB * CH * C + kWave - 1) / kWave; ++u) {
                const int t = lane + u * kWave;
                const int ws = t / (CH * C), off = t % (CH * C);
                const int lc = g - 1 - ws * lagc;
                const bool wanted = CKPT || (publish && ws == nsw - 1);
                if (ws < nsw && wanted && lc >= 0 && lc < nck) {
                    const int col = lc * CH - (kWave - 1) + off / C;
                    if (col >= 0)
                        st_agent(rowsg + (long)(s0 + ws) * a.rowlen + (long)col * C + 1 + off % C,
                                 rings[(ws + 1) * (kBandRing * C) + (col & RM) * C + off % C]);
                }
            }
            if (publish) {
                const int lc = g - 1 - (nsw - 1) * lagc;
                if (lc >= 0 && lc < nck) pub = lc + 1;
            }
            band_barrier();
        }
    }
}

// ------------------------------------------------------------------------------------------------
// reverse sweep (phase 2 of the backward pass; Section 3.4)
// ------------------------------------------------------------------------------------------------
// The mirror image of the forward kernel in time: the bands of a pair start at the bottom, the strips of a band
// likewise, each strip kLockLag2 macro-steps behind the one below it.  A strip recovers the forward values by
// inverting Eq. (1) between the checkpoints of phase 1 (see sk_lane.h), takes the forward values under its last
// lane from the strip's bottom row written in phase 1, and hands the adjoint contributions of its first lane's
// top edges to the strip above.  dF/dp of every block is mapped to the increments at once: the x side in the
// lane's registers, the y side in a ring of accumulators in LDS that the data-moving wave flushes to global
// memory once all strips of the band have passed a column.
template <int BL, int D, int LL>
__global__ __launch_bounds__((kBandStrips + 1) * kWave, 1) void band_rev_kernel(SweepArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    using BD = Band<BL, D, LL>;
    using LK = Lock<BL, D, 1, LL>;
    constexpr int C = LK::C, RR = LK::RR, DSc = LK::DSc, CH = kLockCH2, S = kLockS, NVC = LK::NVC, SPB = kBandStrips;
    constexpr int NVS = RR + 1 + C;
    constexpr int RM = BD::RM, YM = BD::YM;
    constexpr int RSZ = kBandRing * C;
    static_assert(S == 2 * CH, "a checkpoint every second chunk");
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int npairs = (int)a.npairs;
    const int nbands = a.bd_nbands;
    const int band = nbands - 1 - (int)(blockIdx.x / npairs);
    const long pid = blockIdx.x % npairs;
    long xi, yi;
    pair_ids(a, pid, xi, yi);
    SK_LDS real* yring = (SK_LDS real*)(smem + a.bd_off_y);
    SK_LDS real* gyring = (SK_LDS real*)(smem + a.bd_off_gy);
    SK_LDS real* rings = (SK_LDS real*)(smem + a.bd_off_rings);   // adjoint hand-over: ring s + 1 feeds strip s's last lane
    SK_LDS real* krings = rings + (SPB + 1) * RSZ;                // forward values under each strip's last lane
    SK_LDS real* ckst = krings + SPB * RSZ;                       // checkpoint staging: [SPB][2][NVS][64]
    const int ns = a.lk_ns, nb = a.nb;
    const int nbx = a.lk_NT - (kWave - 1);   // block columns a strip's last lane visits (some beyond the grid)
    const int s0 = band * SPB;
    const int nsw = ns - s0 < SPB ? ns - s0 : SPB;
    const int nck = a.lk_NT / CH;
    const int nckS = a.lk_NT / S;
    const int lagc = kLockLag2 / CH;
    const int niter = nck + (SPB - 1) * lagc;
    const real* rowsg = a.rows + pid * a.rows_slot;            // forward bottom rows of phase 1, [ns][rowlen]
    real* adjg = a.adj + pid * a.adj_slot;                     // [nbands][rowlen]: adjoint row above each band
    int* prog = a.bd_flags + (long)npairs * nbands + pid * nbands;

    for (int t = threadIdx.x; t < (SPB + 1) * RSZ; t += blockDim.x) rings[t] = 0.0;
    for (int t = threadIdx.x; t < SPB * RSZ; t += blockDim.x) krings[t] = 1.0;
    __syncthreads();
    // dF/dk[m, n] enters under the last lane of the pair's last strip, at the last column
    if (band == nbands - 1 && threadIdx.x == 0) rings[nsw * RSZ + ((nb - 1) & RM) * C + (C - 1)] = a.grad_k[pid];
    __syncthreads();

    if (w < SPB) {
        // ---------------- a strip ----------------
        const int sg = s0 + w;
        const bool active = w < nsw;
        const int rs = nsw - 1 - w;   // the band's last strip starts
        typename LK::Coef cf;
        typename LK::Rev rv;
        cf.setup(a, active ? sg : 0, lane, a.dx + xi * a.xstride, yring);
        rv.init();
        real gacc[D];
#pragma unroll
        for (int c = 0; c < D; ++c) gacc[c] = 0.0;
        const SK_LDS real* arin = rings + (w + 1) * RSZ;
        SK_LDS real* arout = rings + w * RSZ;
        const SK_LDS real* krow = krings + w * RSZ;
        const SK_LDS real* cks = ckst + w * (2 * NVS * kWave) + lane;
        const bool plain = a.rs2 == 0;   // 64 lanes at 64 different y rows: plain read-modify-write is safe
        bool drift = false;
        real kscale = 1.0;

        auto chunk = [&](auto edge_c, int T0) {
            constexpr bool EDGE = decltype(edge_c)::value;
            // feeds of the strip's last lane: adjoint contributions from the strip below (zero outside the grid) and
            // the forward values of the strip's bottom row exactly as phase 1 left them (ones left of the grid)
            real ea[CH][C], ek[CH][C];
#pragma unroll
            for (int i = 0; i < CH; ++i)
#pragma unroll
                for (int cc = 0; cc < C; ++cc) { ea[i][cc] = 0.0; ek[i][cc] = 1.0; }
            if (lane == kWave - 1) {
#pragma unroll
                for (int i = 0; i < CH; ++i) {
                    const int Jl = T0 + i - (kWave - 1);
                    if (!EDGE || (unsigned)Jl < (unsigned)nb) {
#pragma unroll
                        for (int cc = 0; cc < C; ++cc) ea[i][cc] = arin[(Jl & RM) * C + cc];
                    }
                    if (!EDGE || Jl >= 0) {
#pragma unroll
                        for (int cc = 0; cc < C; ++cc) ek[i][cc] = krow[(Jl & RM) * C + cc];
                    }
                }
            }
            int J[2], b[2];
            real y[2][D];
            BD::template fetch<EDGE>(cf, yring, T0 + CH - 1, J[(CH - 1) & 1], b[(CH - 1) & 1], y[(CH - 1) & 1]);
#pragma unroll
            for (int i = CH - 1; i >= 0; --i) {
                if (i >= 1) BD::template fetch<EDGE>(cf, yring, T0 + i - 1, J[(i - 1) & 1], b[(i - 1) & 1], y[(i - 1) & 1]);
                real Ac[1], Bc[1], iB[1], p6[1], A0[1], B0[1], iB0[1], accP[1];
                const real p = cf.template inner<EDGE>(0, J[i & 1], y[i & 1]);
                LK::coef_rev(p, Ac[0], Bc[0], iB[0]);
                p6[0] = p * (1.0 / 6.0);
                if constexpr (LL == 1) LK::coef_rev(cf.template inner_off<EDGE>(0, J[i & 1]), A0[0], B0[0], iB0[0]);
                else { A0[0] = Ac[0]; B0[0] = Bc[0]; iB0[0] = iB[0]; }
                real recv[C], recvk[C];
#pragma unroll
                for (int cc = 0; cc < C; ++cc) {
                    recv[cc] = wave_from_below_or(rv.up[cc], ea[i][cc]);
                    recvk[cc] = wave_from_below_or(rv.ktop[cc], ek[i][cc]);
                }
                rv.step(recv, recvk, Ac, Bc, iB, p6, A0, B0, iB0, accP);
                if (lane == 0) {
                    const int J0 = T0 + i;
                    if (!EDGE || J0 < nb) {
#pragma unroll
                        for (int cc = 0; cc < C; ++cc) arout[(J0 & RM) * C + cc] = rv.up[cc];
                    }
                }
                // the linear map of Section 3.4 (outside the grid dF/dp is not zero on the left: the adjoint has left
                // the grid there; rows above the grid have zero increments and are never flushed)
                // (lead-lag: blocks off the diagonal of that level have no increment)
                const real gp = ((!EDGE || (unsigned)J[i & 1] < (unsigned)cf.nbl[0]) && !cf.off_block(0, J[i & 1])) ? accP[0] : 0.0;
                if (a.want_gx) {
#pragma unroll
                    for (int c = 0; c < D; ++c) gacc[c] = fma(gp, y[i & 1][c], gacc[c]);
                }
                if (a.want_gy) {
                    SK_LDS real* gq = gyring + __mul24(b[i & 1] & YM, DSc);
                    real t[D];
#pragma unroll
                    for (int c = 0; c < D; ++c) t[c] = gp * cf.dxr[0][c];
                    if (plain) {
                        if (!EDGE || (unsigned)J[i & 1] < (unsigned)nb) {
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

        for (int g = -kBandLeadRev; g <= niter + 1; ++g) {
            const int rc = g - rs * lagc;
            if (active && rc >= 0 && rc < nck) {
                const int fc = nck - 1 - rc;
                if (fc & 1) {
                    // the exact state after this chunk's last macro-step, staged in LDS by the data-moving wave
                    const int idx = (fc + 1) / 2;
                    const SK_LDS real* cs = cks + (idx & 1) * (NVS * kWave);
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
                if (cf.interior(fc * CH, CH)) chunk(std::false_type(), fc * CH);
                else chunk(std::true_type(), fc * CH);
            }
            band_barrier();
        }
        if (active) {
            // the left end: every strip started from the boundary value 1 in every lane
#pragma unroll
            for (int i = 0; i <= RR; ++i)
                if (!(fabs(rv.kR[i] - 1.0) <= kDriftTol * kscale)) drift = true;
            // the sums of a pair are spread over workgroups and already on their way: every pair of the call is then
            // solved once more by the replay kernel
            if (drift) atomicCAS(a.err, 0, 2);   // (an error already raised stays)
            if (a.want_gx) {
                const int I = sg * kWave + lane - a.lk_padb;
                if (I >= 0) {
                    real* gq = a.gdx + xi * a.xstride + (long)(I >> a.rs1) * DSc;
#pragma unroll
                    for (int c = 0; c < D; ++c) unsafeAtomicAdd(gq + c, gacc[c] * a.sc);
                }
            }
        }
    } else {
        // ---------------- the data-moving wave ----------------
        const real* dyg = a.dy + yi * a.ystride;
        real* gdyg = a.gdy + yi * a.ystride;
        const real* adjprev = band < nbands - 1 ? adjg + (long)(band + 1) * a.rowlen : nullptr;   // written by the band below
        real* adjout = adjg + (long)band * a.rowlen;
        const int* progprev = band < nbands - 1 ? prog + band + 1 : nullptr;
        const bool publish = band > 0;
        int ylow = a.q;             // coarse y columns >= ylow are staged
        int yh0 = 0, yhn = 0;
        real yh = 0.0;
        int fhigh = a.q;            // accumulator columns >= fhigh are flushed
        real inh = 0.0;             // incoming adjoint values on their way into the ring
        real kh = 1.0;              // forward bottom-row values on their way into the rings
        real ckr[SPB][NVS];         // checkpoints on their way into the staging buffers
        int seen = 0, pub = 0;
        bool dead = false;
        const int up1 = lane > 0 ? -1 : 0;
        auto load_ckpt = [&](int ws, int idx) {
            const real* cp = a.ckpt + pid * a.ckpt_slot + ((long)(s0 + ws) * (nckS + 1) + idx) * NVC * kWave + lane;
#pragma unroll
            for (int q = 0; q <= RR; ++q) ckr[ws][q] = ld_scratch(cp + q * kWave);
            ckr[ws][RR + 1] = ld_scratch(cp + (RR + 1 + C) * kWave + up1);   // corner of the lane above
#pragma unroll
            for (int q = 1; q < C; ++q) ckr[ws][RR + 1 + q] = ld_scratch(cp + (RR + 1 + q - 1) * kWave + up1);
        };
#pragma unroll
        for (int ws = 0; ws < SPB; ++ws) {
#pragma unroll
            for (int q = 0; q < NVS; ++q) ckr[ws][q] = 1.0;
            if (ws < nsw) load_ckpt(ws, nckS);
        }
        // first macro-step column of chunk rc of the strip with reverse index rs (may be negative before it starts)
        auto chunk_T0 = [&](int rc) { return (nck - 1 - rc) * CH; };

        for (int g = -kBandLeadRev; g <= niter + 1; ++g) {
            // (0) announce the adjoint row pieces written out in the last iteration
            if (pub > 0) {
                stores_done();
                if (lane == 0) st_agent_int(prog + band, pub);
                pub = 0;
            }
            // the seed has been taken (the pair's last strip passes the last column in its first chunks): its ring
            // slot serves other columns from now on
            if (band == nbands - 1 && g == 8 && lane == 0) rings[nsw * RSZ + ((nb - 1) & RM) * C + (C - 1)] = 0.0;
            // (1) y increments of the coming columns (descending), their accumulators cleared
            if (lane < yhn * DSc) {
                const int slot = __mul24((yh0 + lane / DSc) & YM, DSc) + lane % DSc;
                yring[slot] = yh;
                gyring[slot] = 0.0;
            }
            {
                // the band's last strip is the first to reach a column: its chunk g + 2
                const int rcn = g + 2 < 0 ? 0 : (g + 2 < nck ? g + 2 : nck - 1);
                int lo = chunk_T0(rcn) - (kWave - 1);
                if (lo < 0) lo = 0;
                if (lo > nb - 1) lo = nb - 1;
                lo >>= a.rs2;
                int n = ylow - lo;
                if (n > CH) n = CH;
                if (n < 0) n = 0;
                yh0 = ylow - n; yhn = n; ylow -= n;
                if (lane < n * DSc) yh = dyg[(long)yh0 * DSc + lane];
            }
            // (2) accumulators of the columns every strip of the band has passed go out to global memory
            if (a.want_gy) {
                const int rct = g - (nsw - 1) * lagc;   // chunk of the band's first strip (the last to pass)
                int bnd;
                if (rct < 0) bnd = a.q;
                else if (rct >= nck) bnd = 0;
                else { bnd = ((chunk_T0(rct) + CH + CH) >> a.rs2) + 1; if (bnd > a.q) bnd = a.q; }
                int n = fhigh - bnd;
                if (n > 2 * CH) n = 2 * CH;
                if (n < 0) n = 0;
                const int f0 = fhigh - n;
                fhigh -= n;
                for (int t = lane; t < n * DSc; t += kWave) {
                    const int bcol = f0 + t / DSc, c = t % DSc;
                    const real v = gyring[__mul24(bcol & YM, DSc) + c];
                    if (c < D && v != 0.0) unsafeAtomicAdd(&gdyg[(long)bcol * DSc + c], v);
                }
            }
            // (3) adjoint row from the band below: the piece for the last strip's chunk g + 1 goes into its ring, the
            //     piece for chunk g + 2 is requested once the band below has written it
            if (band < nbands - 1) {
                const int cw = g + 1;
                if (cw >= 0 && cw < nck && lane < CH * C) {
                    const int col = chunk_T0(cw) - (kWave - 1) + lane / C;
                    if ((unsigned)col < (unsigned)nb) rings[nsw * RSZ + (col & RM) * C + lane % C] = inh;
                }
                const int cr = g + 2;
                if (cr >= 0 && cr < nck) {
                    int need = cr + lagc;   // the lower band's first strip has finished these columns after this many chunks
                    if (need > nck) need = nck;
                    if (seen < need && !dead) {
                        int want = need + kBandSlack;
                        if (want > nck) want = nck;
                        seen = wait_progress(progprev, want, a.bd_spin);
                        if (seen < need) {
                            dead = true;
                            if (lane == 0) atomicExch(a.err, 1);
                        }
                    }
                    const int col = chunk_T0(cr) - (kWave - 1) + lane / C;
                    inh = (lane < CH * C && (unsigned)col < (unsigned)nb) ? ld_scratch(adjprev + (long)col * C + lane % C) : 0.0;
                }
            }
            // (4) the adjoint row above the band: what the first strip finished in the last iteration goes out
            if (publish) {
                const int rc = g - 1 - (nsw - 1) * lagc;
                if (rc >= 0 && rc < nck) {
                    const int col = chunk_T0(rc) + lane / C;
                    if (lane < CH * C && col < nb) st_agent(adjout + (long)col * C + lane % C, rings[(col & RM) * C + lane % C]);
                    pub = rc + 1;
                }
            }
            // (5) forward values under each strip's last lane: pieces loaded in the last iteration into the rings,
            //     the pieces for each strip's chunk after next requested
            {
                const int ws = lane / (CH * C), off = lane % (CH * C);
                if (ws < nsw) {
                    const int rs = nsw - 1 - ws;
                    const int cw = g + 1 - rs * lagc;
                    if (cw >= 0 && cw < nck) {
                        const int col = chunk_T0(cw) - (kWave - 1) + off / C;
                        if (col >= 0) krings[ws * RSZ + (col & RM) * C + off % C] = kh;
                    }
                    const int cr = g + 2 - rs * lagc;
                    if (cr >= 0 && cr < nck) {
                        const int col = chunk_T0(cr) - (kWave - 1) + off / C;
                        kh = (unsigned)col < (unsigned)nbx ? rowsg[(long)(s0 + ws) * a.rowlen + (long)col * C + off % C] : 1.0;
                    }
                }
            }
            // (6) checkpoints: strip ws restores checkpoint idx at the start of its chunk rc with nck - 1 - rc odd,
            //     idx = (nck - rc) / 2; it is written into half (idx & 1) of the strip's staging buffer one iteration
            //     before, and was requested two chunks before that
#pragma unroll
            for (int ws = 0; ws < SPB; ++ws) {
                if (ws < nsw) {
                    const int rc = g - (nsw - 1 - ws) * lagc;
                    if (rc >= -1 && rc < nck && ((nck - rc - 1) & 1) == 0) {
                        const int idx = (nck - rc - 1) / 2;
                        if (idx >= 1) {
                            SK_LDS real* cs = ckst + ws * (2 * NVS * kWave) + (idx & 1) * (NVS * kWave) + lane;
#pragma unroll
                            for (int i = 0; i < NVS; ++i) cs[i * kWave] = ckr[ws][i];
                            if (idx >= 2) load_ckpt(ws, idx - 1);
                        }
                    }
                }
            }
            band_barrier();
        }
        // what is left in the accumulators
        if (a.want_gy) {
            for (int t = lane; t < fhigh * DSc; t += kWave) {
                const int bcol = t / DSc, c = t % DSc;
                const real v = gyring[__mul24(bcol & YM, DSc) + c];
                if (c < D && v != 0.0) unsafeAtomicAdd(&gdyg[(long)bcol * DSc + c], v);
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// launchers
// ------------------------------------------------------------------------------------------------
template <int BL, int D, int LL>
hipError_t launch_band_t(int phase, const SweepArgs& a, int grid, size_t lds, hipStream_t st)
{
    const dim3 block((kBandStrips + 1) * kWave);
    auto prep = [&](const void* fn) { return allow_full_lds(fn); };
    hipError_t e;
    if (phase == 0) {
        e = prep(reinterpret_cast<const void*>(&band_fwd_kernel<BL, D, false, LL>));
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((band_fwd_kernel<BL, D, false, LL>), dim3(grid), block, lds, st, a);
    } else {
        // backward: the forward sweep with checkpoints, then the reverse sweep with the bands in reverse order
        // (phase 2 / 3: one of the two only, for a forward sweep that is kept for the backward call)
        e = prep(reinterpret_cast<const void*>(&band_fwd_kernel<BL, D, true, LL>));
        if (e != hipSuccess) return e;
        e = prep(reinterpret_cast<const void*>(&band_rev_kernel<BL, D, LL>));
        if (e != hipSuccess) return e;
        if (phase != 3) {
            hipLaunchKernelGGL((band_fwd_kernel<BL, D, true, LL>), dim3(grid), block, lds, st, a);
            e = hipGetLastError();
            if (e != hipSuccess) return e;
        }
        if (phase != 2) hipLaunchKernelGGL((band_rev_kernel<BL, D, LL>), dim3(grid), block, lds, st, a);
    }
    return hipGetLastError();
}

// lead-lag form of the sweep (SweepArgs::ll): inside the blocks (1) for blocks that hold every refined cell of a pair
// of increments, above them (2) otherwise
template <int BL, int D>
hipError_t launch_band_ll(int phase, const SweepArgs& a, int grid, size_t lds, hipStream_t st)
{
    if (a.ll == 0) return launch_band_t<BL, D, 0>(phase, a, grid, lds, st);
    if constexpr (BL >= 1) {
        if (a.ll == 1 && a.rs1 == 0 && a.rs2 == 0) return launch_band_t<BL, D, 1>(phase, a, grid, lds, st);
    }
    if (a.ll == 2 && a.rs1 >= 1 && a.rs2 >= 1) return launch_band_t<BL, D, 2>(phase, a, grid, lds, st);
    return hipErrorInvalidValue;
}

template <int BL>
hipError_t launch_band_bl(int phase, int DT, const SweepArgs& a, int grid, size_t lds, hipStream_t st)
{
    switch (DT) {
        case 2: return launch_band_ll<BL, 2>(phase, a, grid, lds, st);
        case 3: return launch_band_ll<BL, 3>(phase, a, grid, lds, st);
        case 4: return launch_band_ll<BL, 4>(phase, a, grid, lds, st);
        case 5: return launch_band_ll<BL, 5>(phase, a, grid, lds, st);
        case 6: return launch_band_ll<BL, 6>(phase, a, grid, lds, st);
        case 8: return launch_band_ll<BL, 8>(phase, a, grid, lds, st);
        default: return hipErrorInvalidValue;
    }
}

// phase 0: forward sweep; phase 1: backward pass (forward sweep with checkpoints, then the reverse sweep);
// phase 2 / 3: the first / second launch of phase 1 alone
hipError_t launch_sweep_band(int phase, int BL, int DT, const SweepArgs& a, int grid, size_t lds, hipStream_t st)
{
    // what the kernels assume about the launch
    if (phase < 0 || phase > 3 || a.lk_M != 1 || a.lk_ns < 1 || a.bd_nbands != (a.lk_ns + kBandStrips - 1) / kBandStrips ||
        (long)grid != a.npairs * a.bd_nbands || (a.lk_NT % 8) != 0 || a.lk_NT < a.nb + kWave - 1 ||
        a.lk_padb != a.lk_ns * kWave - a.mb || a.bd_flags == nullptr || a.lk_NT >= a.nb + kWave - 1 + 8 ||
        a.rowlen < (a.lk_NT - (kWave - 1)) * (1 << BL) + 1 ||
        a.rows_slot < (long)a.lk_ns * a.rowlen ||
        (phase != 0 && (a.adj == nullptr || a.ckpt == nullptr || a.adj_slot < (long)a.bd_nbands * a.rowlen ||
                        a.ckpt_slot < (long)a.lk_ns * (a.lk_NT / kLockS + 1) * ((1 << BL) * 2 + 2) * kWave)))
        return hipErrorInvalidValue;
    switch (BL) {
        case 0: return launch_band_bl<0>(phase, DT, a, grid, lds, st);
        case 1: return launch_band_bl<1>(phase, DT, a, grid, lds, st);
        case 2: return launch_band_bl<2>(phase, DT, a, grid, lds, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace sk

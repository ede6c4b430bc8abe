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
// Release at device scope: everything this wave has stored is visible to the other workgroups (which may run
// on a compute die with an L2 of its own) before a counter advanced afterwards is.
__device__ __forceinline__ void publish_fence() { __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent"); }
// Acquire at device scope: loads issued afterwards see what another workgroup released before the counter
// value this wave has just read.
__device__ __forceinline__ void consume_fence() { __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent"); }

// Waits until *ctr >= need (bounded); returns false when the wait ran out.
__device__ __forceinline__ bool wait_progress(const int* ctr, int need)
{
    for (int spin = 0; spin < kBandSpin; ++spin) {
        if (ld_agent_int(ctr) >= need) return true;
        __builtin_amdgcn_s_sleep(4);
    }
    return false;
}

template <int BL, int D>
struct Band {
    using LK = Lock<BL, D, 1>;
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
template <int BL, int D, bool CKPT>
__global__ __launch_bounds__((kBandStrips + 1) * kWave, 1) void band_fwd_kernel(SweepArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    using BD = Band<BL, D>;
    using LK = Lock<BL, D, 1>;
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
                real Ac[1], Bc[1];
                const real p = cf.template inner<EDGE>(0, J[i & 1], y[i & 1]);
                const real q2 = p * p;
                Bc[0] = fma(q2, -1.0 / 12.0, 1.0);
                Ac[0] = fma(p, 0.5, fma(q2, 1.0 / 12.0, 1.0));
                real recv[C];
#pragma unroll
                for (int cc = 0; cc < C; ++cc) recv[cc] = wave_from_above_or(f.bot[cc], edge[i][cc]);
                f.step(recv, Ac, Bc);
                if (lane == kWave - 1) {
                    const int Jw = T0 + i - (kWave - 1);
                    if (!EDGE || (unsigned)Jw < (unsigned)nb) {
#pragma unroll
                        for (int cc = 0; cc < C; ++cc) rout[(Jw & RM) * C + cc] = f.bot[cc];
                        if (EDGE && laststrip && Jw == nb - 1 && a.k_out) a.k_out[pid] = f.bot[C - 1];
                    }
                }
            }
        };

        for (int g = -kBandLead; g <= niter; ++g) {
            const int lc = g - w * lagc;
            if (active && lc >= 0 && lc < nck) {
                if (CKPT) f.store_ckpt(ckpt + (long)lc * NVC * kWave);
                if (cf.interior(lc * CH, CH)) chunk(std::false_type(), lc * CH);
                else chunk(std::true_type(), lc * CH);
                if (CKPT && lc == nck - 1) f.store_ckpt(ckpt + (long)nck * NVC * kWave);
            }
            band_barrier();
        }
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
        bool dead = false;
        if (CKPT && lane < nsw) st_agent(rowsg + (long)(s0 + lane) * a.rowlen, 1.0);   // node column 0 of each row

        for (int g = -kBandLead; g <= niter; ++g) {
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
                    if (!dead && !wait_progress(progprev, need)) {
                        dead = true;
                        if (lane == 0) atomicExch(a.err, 1);
                    }
                    consume_fence();
                    const int col = cr * CH + lane / C;
                    inh = (lane < CH * C && col < nb) ? ld_scratch(rowprev + (long)col * C + 1 + lane % C) : 1.0;
                }
            }
            // (3) bottom rows: the pieces the strips finished in the last iteration go out to global memory
            {
                bool any = false;
#pragma unroll
                for (int u = 0; u < (SPB * CH * C + kWave - 1) / kWave; ++u) {
                    const int t = lane + u * kWave;
                    const int ws = t / (CH * C), off = t % (CH * C);
                    const int lc = g - 1 - ws * lagc;
                    const bool wanted = CKPT || (publish && ws == nsw - 1);
                    if (ws < nsw && wanted && lc >= 0 && lc < nck) {
                        const int col = lc * CH - (kWave - 1) + off / C;
                        if ((unsigned)col < (unsigned)nb)
                            st_agent(rowsg + (long)(s0 + ws) * a.rowlen + (long)col * C + 1 + off % C,
                                     rings[(ws + 1) * (kBandRing * C) + (col & RM) * C + off % C]);
                        any = true;
                    }
                }
                (void)any;
                if (publish) {
                    const int lc = g - 1 - (nsw - 1) * lagc;
                    if (lc >= 0 && lc < nck) {
                        publish_fence();
                        if (lane == 0) st_agent_int(prog + band, lc + 1);
                    }
                }
            }
            band_barrier();
        }
    }
}

// ------------------------------------------------------------------------------------------------
// launchers
// ------------------------------------------------------------------------------------------------
template <int BL, int D>
hipError_t launch_band_t(int phase, const SweepArgs& a, int grid, size_t lds, hipStream_t st)
{
    const dim3 block((kBandStrips + 1) * kWave);
    auto prep = [&](const void* fn) {
        return hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsPerCU);
    };
    hipError_t e;
    if (phase == 0) {
        e = prep(reinterpret_cast<const void*>(&band_fwd_kernel<BL, D, false>));
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((band_fwd_kernel<BL, D, false>), dim3(grid), block, lds, st, a);
    } else {
        return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

template <int BL>
hipError_t launch_band_bl(int phase, int DT, const SweepArgs& a, int grid, size_t lds, hipStream_t st)
{
    switch (DT) {
        case 2: return launch_band_t<BL, 2>(phase, a, grid, lds, st);
        case 3: return launch_band_t<BL, 3>(phase, a, grid, lds, st);
        case 4: return launch_band_t<BL, 4>(phase, a, grid, lds, st);
        case 5: return launch_band_t<BL, 5>(phase, a, grid, lds, st);
        case 6: return launch_band_t<BL, 6>(phase, a, grid, lds, st);
        case 8: return launch_band_t<BL, 8>(phase, a, grid, lds, st);
        default: return hipErrorInvalidValue;
    }
}

// phase 0: forward sweep; phase 1: forward sweep of the backward pass; phase 2: reverse sweep
hipError_t launch_sweep_band(int phase, int BL, int DT, const SweepArgs& a, int grid, size_t lds, hipStream_t st)
{
    // what the kernels assume about the launch
    if (a.lk_M != 1 || a.lk_ns < 1 || a.bd_nbands != (a.lk_ns + kBandStrips - 1) / kBandStrips ||
        (long)grid != a.npairs * a.bd_nbands || (a.lk_NT % 8) != 0 || a.lk_NT < a.nb + kWave - 1 ||
        a.lk_padb != a.lk_ns * kWave - a.mb || a.bd_flags == nullptr || a.rowlen < a.nb * (1 << BL) + 1 ||
        a.rows_slot < (long)a.lk_ns * a.rowlen)
        return hipErrorInvalidValue;
    switch (BL) {
        case 0: return launch_band_bl<0>(phase, DT, a, grid, lds, st);
        case 1: return launch_band_bl<1>(phase, DT, a, grid, lds, st);
        case 2: return launch_band_bl<2>(phase, DT, a, grid, lds, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace sk

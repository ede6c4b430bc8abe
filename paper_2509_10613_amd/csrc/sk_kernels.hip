// HIP kernels (gfx950) for batched signature kernels: increments, forward PDE sweep, reverse (adjoint)
// sweep, and the map back to path gradients.  Paper Section 3 (Eq. (1), the two adjoint relations of
// Section 3.4); the mapping of the sweep onto wavefronts is this library's own.
//
// Sweep layout.  One wavefront (64 lanes) owns one path pair.  The refined grid is cut into square blocks
// of 2^BL x 2^BL refined cells that share one increment inner product p (the dyadic refinement is an
// index shift, Section 3.2 item (3)).  Lane l of a strip owns block row I = 64 s + l and, at macro-step T,
// processes block column J = T - l, so the 64 lanes sit on one anti-diagonal of blocks (Section 3.3: cells
// of an anti-diagonal are independent).  A lane needs the bottom edge of the block above it, which the
// lane above produced one macro-step earlier: one DPP wave shift per edge value and step.  Strips of 64
// block rows are chained through a boundary row in global memory (the idea of Section 3.3's blocks of 32
// rows, at wave64 width).  The increment inner product is formed in registers from the lane's own x
// increments and the y increments of column J; the Gram matrix of increments is never materialised.
//
// Backward.  The adjoint sweep needs the forward values at every node while it runs the other way
// (Section 3.4).  Forward values are not stored: the forward pass writes the wavefront state every S
// macro-steps (a checkpoint), and the reverse pass replays one segment of S steps at a time into an LDS
// ring (block input edges only), then walks that segment backwards, re-deriving the block interior.
#include <hip/hip_runtime.h>

#include "sk_kernels.h"

namespace sk {

// ------------------------------------------------------------------------------------------------
// lane exchange helpers (must be called with all 64 lanes active)
// ------------------------------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ T wave_from_above(T v)   // lane i receives lane i-1; lane 0 keeps its own
{
    constexpr int NW = sizeof(T) / 4;
    int w[NW];
    __builtin_memcpy(w, &v, sizeof(T));
#pragma unroll
    for (int i = 0; i < NW; ++i) w[i] = __builtin_amdgcn_update_dpp(w[i], w[i], 0x138, 0xf, 0xf, false);
    __builtin_memcpy(&v, w, sizeof(T));
    return v;
}

template <typename T>
__device__ __forceinline__ T wave_from_below(T v)   // lane i receives lane i+1; lane 63 keeps its own
{
    constexpr int NW = sizeof(T) / 4;
    int w[NW];
    __builtin_memcpy(w, &v, sizeof(T));
#pragma unroll
    for (int i = 0; i < NW; ++i) w[i] = __builtin_amdgcn_update_dpp(w[i], w[i], 0x130, 0xf, 0xf, false);
    __builtin_memcpy(&v, w, sizeof(T));
    return v;
}

template <typename T>
__device__ __forceinline__ T read_lane(T v, int lane)   // wave-uniform lane index
{
    constexpr int NW = sizeof(T) / 4;
    int w[NW];
    __builtin_memcpy(w, &v, sizeof(T));
#pragma unroll
    for (int i = 0; i < NW; ++i) w[i] = __builtin_amdgcn_readlane(w[i], lane);
    __builtin_memcpy(&v, w, sizeof(T));
    return v;
}

// Device-scope load that bypasses the per-CU vector cache: used for data this wave wrote to global
// scratch earlier in the same kernel.
__device__ __forceinline__ double ld_scratch(const double* p)
{
    unsigned long long u = __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p), __ATOMIC_RELAXED,
                                             __HIP_MEMORY_SCOPE_AGENT);
    return __longlong_as_double((long long)u);
}
__device__ __forceinline__ float ld_scratch(const float* p)
{
    unsigned int u = __hip_atomic_load(reinterpret_cast<const unsigned int*>(p), __ATOMIC_RELAXED,
                                       __HIP_MEMORY_SCOPE_AGENT);
    return __uint_as_float(u);
}

__device__ __forceinline__ void scratch_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
}

// Pointers into LDS keep their address space in the type, so that every access is a ds_* instruction.
#define SK_LDS __attribute__((address_space(3)))

template <typename T>
__device__ __forceinline__ void lds_atomic_add(SK_LDS T* p, T v)
{
    (void)__hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

template <typename T> __device__ __forceinline__ T fmaT(T a, T b, T c);
template <> __device__ __forceinline__ double fmaT<double>(double a, double b, double c) { return fma(a, b, c); }
template <> __device__ __forceinline__ float fmaT<float>(float a, float b, float c) { return fmaf(a, b, c); }

// ------------------------------------------------------------------------------------------------
// small kernels
// ------------------------------------------------------------------------------------------------
template <typename TA, typename TB>
__global__ void convert_kernel(const TA* __restrict__ in, TB* __restrict__ out, long n)
{
    long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    long st = (long)gridDim.x * blockDim.x;
    for (; i < n; i += st) out[i] = (TB)in[i];
}

template <typename T>
__global__ void fill_kernel(T* p, long n, T v)
{
    long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    long st = (long)gridDim.x * blockDim.x;
    for (; i < n; i += st) p[i] = v;
}

// Increments, transposed and padded: out[path][c][a] = x[path][a+1][c] - x[path][a][c] for a < L-1, c < d;
// zero elsewhere (first line of the paper's forward listing).  The difference is taken in double.
template <typename TI>
__global__ void increments_kernel(const TI* __restrict__ x, double* __restrict__ out, long npaths, int L, int d,
                                  int DP, int rpad)
{
    long total = npaths * (long)DP * rpad;
    long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    long st = (long)gridDim.x * blockDim.x;
    for (; i < total; i += st) {
        int a = (int)(i % rpad);
        long t = i / rpad;
        int c = (int)(t % DP);
        long pth = t / DP;
        double v = 0.0;
        if (a < L - 1 && c < d) {
            const TI* xp = x + (pth * L + a) * (long)d + c;
            v = (double)xp[d] - (double)xp[0];
        }
        out[i] = v;
    }
}

// grad[path][i][c] = g[path][c][i-1] - g[path][c][i] (out-of-range terms zero): the increments are
// differences of consecutive points, so the gradient of a point collects the two increments it touches.
template <typename TO>
__global__ void finalize_grad_kernel(const double* __restrict__ g, TO* __restrict__ grad, long npaths, int L, int d,
                                     int DP, int rpad)
{
    long total = npaths * (long)L * d;
    long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    long st = (long)gridDim.x * blockDim.x;
    for (; i < total; i += st) {
        int c = (int)(i % d);
        long t = i / d;
        int pt = (int)(t % L);
        long pth = t / L;
        const double* gp = g + (pth * DP + c) * (long)rpad;
        double hi = pt >= 1 ? gp[pt - 1] : 0.0;
        double lo = pt < L - 1 ? gp[pt] : 0.0;
        grad[i] = (TO)(hi - lo);
    }
}

// ------------------------------------------------------------------------------------------------
// sweep building blocks
// ------------------------------------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ T wave_from_above_or(T v, T edge)   // lane i receives v of lane i-1; lane 0 gets edge
{
    constexpr int NW = sizeof(T) / 4;
    int w[NW], o[NW];
    __builtin_memcpy(w, &v, sizeof(T));
    __builtin_memcpy(o, &edge, sizeof(T));
#pragma unroll
    for (int i = 0; i < NW; ++i) w[i] = __builtin_amdgcn_update_dpp(o[i], w[i], 0x138, 0xf, 0xf, false);
    __builtin_memcpy(&v, w, sizeof(T));
    return v;
}

template <typename T>
__device__ __forceinline__ T wave_from_below_or(T v, T edge)   // lane i receives v of lane i+1; lane 63 gets edge
{
    constexpr int NW = sizeof(T) / 4;
    int w[NW], o[NW];
    __builtin_memcpy(w, &v, sizeof(T));
    __builtin_memcpy(o, &edge, sizeof(T));
#pragma unroll
    for (int i = 0; i < NW; ++i) w[i] = __builtin_amdgcn_update_dpp(o[i], w[i], 0x130, 0xf, 0xf, false);
    __builtin_memcpy(&v, w, sizeof(T));
    return v;
}

template <typename T, int BL, int D>
struct Sweep {
    static constexpr int R = 1 << BL;
    static constexpr int C = 1 << BL;
    static constexpr int DN = D > 0 ? D : 1;
    static constexpr int NVR = R + C + 1;   // ring: top edge (C+1) + left edge below the corner (R)
    static constexpr int NVC = R + 1 + C;   // checkpoint: left edge (R+1) + own bottom edge (C)

    const SweepArgs<T>& a;
    const int lane;
    // per pair
    const T* dxrow = nullptr;   // transposed x increments of the pair: [c][rpad]
    const T* dyg = nullptr;     // transposed y increments in global memory: [c][qpad]
    const SK_LDS T* dyl = nullptr;   // the same staged in LDS (when a.y_lds)
    // per strip
    int s = 0, lb = 0, arow = 0;
    int nbl = 0;                // a.nb for lanes that own a block row, 0 otherwise
    T dxr[DN];
    const T* rowprev = nullptr;
    T* rowcur = nullptr;
    // forward lane state
    T left[R + 1];
    T bot[C];
    // top edge feed of lane 0: lane q of topc holds the boundary-row values of block column
    // (column of lane 0 at the current step) + q; the register rotates by one lane per step and is
    // refilled every 64 steps from topn, which is loaded one chunk ahead.
    T topc[C], topn[C];
    int chunk_end = 0;
    // y increments of the block this lane processes at the coming step (loaded one step ahead)
    T ycur[DN];

    __device__ __forceinline__ Sweep(const SweepArgs<T>& a_, int lane_) : a(a_), lane(lane_) {}

    __device__ __forceinline__ void begin_strip(int s_, T* rows)
    {
        s = s_;
        const int I = s * kWave + lane;
        nbl = I < a.mb ? a.nb : 0;
        int rem = a.mb - s * kWave - 1;
        lb = rem < kWave - 1 ? rem : kWave - 1;
        int ar = I >> a.rs1;
        arow = ar < a.r ? ar : a.r - 1;
        if constexpr (D > 0) {
#pragma unroll
            for (int c = 0; c < D; ++c) dxr[c] = a.sc * dxrow[(long)c * a.rpad + arow];
        }
        rowprev = s > 0 ? rows + (long)(s - 1) * a.rowlen : nullptr;
        rowcur = rows + (long)s * a.rowlen;
#pragma unroll
        for (int i = 0; i <= R; ++i) left[i] = T(1);
#pragma unroll
        for (int i = 0; i < C; ++i) bot[i] = T(1);
    }

    __device__ __forceinline__ bool rowvalid() const { return nbl != 0; }

    // y increments of block column J (clamped into range so that every lane may load)
    __device__ __forceinline__ void fetch_y(int J, T (&yv)[DN]) const
    {
        if constexpr (D > 0) {
            int Jc = J < 0 ? 0 : J;
            Jc = Jc < a.nb ? Jc : a.nb - 1;
            const int b = Jc >> a.rs2;
            if (a.y_lds) {
#pragma unroll
                for (int c = 0; c < D; ++c) yv[c] = dyl[c * a.qpad + b];
            } else {
#pragma unroll
                for (int c = 0; c < D; ++c) yv[c] = dyg[(long)c * a.qpad + b];
            }
        } else {
            yv[0] = T(0);
        }
    }

    __device__ __forceinline__ T load_y(int c, int b) const
    {
        return a.y_lds ? dyl[c * a.qpad + b] : dyg[(long)c * a.qpad + b];
    }

    // p = 2^-(lam1+lam2) <dx[a], dy[b]> (+ the time channel's constant product), Eq. (1) third line.
    __device__ __forceinline__ T inner(int b, const T (&yv)[DN]) const
    {
        T p = a.tc;
        if constexpr (D > 0) {
#pragma unroll
            for (int c = 0; c < D; ++c) p = fmaT(dxr[c], yv[c], p);
        } else {
            for (int c = 0; c < a.d; ++c) p = fmaT(a.sc * dxrow[(long)c * a.rpad + arow], load_y(c, b), p);
        }
        return p;
    }

    // Eq. (1) on the R x C cells of one block; e[0][*] and e[*][0] are given.
    static __device__ __forceinline__ void block_forward(T (&e)[R + 1][C + 1], T p)
    {
        const T q2 = p * p;
        const T Bc = fmaT(q2, T(-1.0 / 12.0), T(1));
        const T Ac = fmaT(p, T(0.5), fmaT(q2, T(1.0 / 12.0), T(1)));
#pragma unroll
        for (int rr = 0; rr < R; ++rr)
#pragma unroll
            for (int cc = 0; cc < C; ++cc)
                e[rr + 1][cc + 1] = fmaT(e[rr + 1][cc] + e[rr][cc + 1], Ac, -(e[rr][cc] * Bc));
    }

    __device__ __forceinline__ void load_top(int Jbase, T (&dst)[C]) const
    {
        const int Jq = Jbase + lane;
#pragma unroll
        for (int cc = 0; cc < C; ++cc)
            dst[cc] = (rowprev != nullptr && Jq < a.nb) ? ld_scratch(rowprev + (long)Jq * C + 1 + cc) : T(1);
    }

    // Call before the first forward_step of a run of consecutive steps starting at T0.
    __device__ __forceinline__ void prime(int T0)
    {
        load_top(T0, topc);
        load_top(T0 + kWave, topn);
        chunk_end = T0 + kWave;
        fetch_y(T0 - lane, ycur);
    }

    // One forward macro-step.  Returns whether this lane processed a block; e, p, yv describe it.
    template <bool WRITE_ROW>
    __device__ __forceinline__ bool forward_step(int Tstep, T (&e)[R + 1][C + 1], T& p, T (&yv)[DN])
    {
        if (Tstep == chunk_end) {
#pragma unroll
            for (int cc = 0; cc < C; ++cc) topc[cc] = topn[cc];
            load_top(Tstep + kWave, topn);
            chunk_end = Tstep + kWave;
        }
        T recv[C];
#pragma unroll
        for (int cc = 0; cc < C; ++cc) {
            recv[cc] = wave_from_above_or(bot[cc], topc[cc]);
            topc[cc] = wave_from_below(topc[cc]);
        }
        const int J = Tstep - lane;
#pragma unroll
        for (int c = 0; c < DN; ++c) yv[c] = ycur[c];
        fetch_y(J + 1, ycur);   // for the next step; consumed one iteration later
        const bool active = (unsigned)J < (unsigned)nbl;
        if (active) {
            e[0][0] = left[0];
#pragma unroll
            for (int cc = 0; cc < C; ++cc) e[0][cc + 1] = recv[cc];
#pragma unroll
            for (int rr = 1; rr <= R; ++rr) e[rr][0] = left[rr];
            p = inner(J >> a.rs2, yv);
            block_forward(e, p);
#pragma unroll
            for (int rr = 0; rr <= R; ++rr) left[rr] = e[rr][C];
#pragma unroll
            for (int cc = 0; cc < C; ++cc) bot[cc] = e[R][cc + 1];
            if (WRITE_ROW && lane == lb) {
#pragma unroll
                for (int cc = 0; cc < C; ++cc) rowcur[(long)J * C + 1 + cc] = bot[cc];
            }
        }
        return active;
    }

    __device__ __forceinline__ int strip_steps() const { return a.nb + lb; }
};

// ------------------------------------------------------------------------------------------------
// forward kernel: one wave per pair, kWavesPerWG independent waves per workgroup
// ------------------------------------------------------------------------------------------------
template <typename T, int BL, int D>
__global__ __launch_bounds__(kWavesPerWG* kWave) void sweep_fwd_kernel(SweepArgs<T> a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    using SW = Sweep<T, BL, D>;
    constexpr int R = SW::R, C = SW::C;
    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6;
    const long slot = (long)blockIdx.x * kWavesPerWG + w;
    const long nslots = (long)gridDim.x * kWavesPerWG;
    SK_LDS T* ylds = (SK_LDS T*)(smem + (size_t)w * a.lds_wave);
    T* rows = a.rows + slot * a.rows_slot;
    SW sw(a, lane);

    for (long pid = slot; pid < a.npairs; pid += nslots) {
        const long xi = a.gramM ? pid / a.gramM : pid;
        const long yi = a.gramM ? pid % a.gramM : pid;
        sw.dxrow = a.dxT + xi * a.xstride;
        sw.dyg = a.dyT + yi * a.ystride;
        sw.dyl = ylds;
        if (a.y_lds) {
            const int n = a.DP * a.qpad;
            for (int t = lane; t < n; t += kWave) ylds[t] = sw.dyg[t];
        }
        for (int s = 0; s < a.ns; ++s) {
            sw.begin_strip(s, rows);
            const int NT = sw.strip_steps();
            const bool last = s == a.ns - 1;
            sw.prime(0);
            if (last) {
                for (int Tstep = 0; Tstep < NT; ++Tstep) {
                    T e[R + 1][C + 1];
                    T p;
                    T yv[SW::DN];
                    sw.template forward_step<false>(Tstep, e, p, yv);
                }
                if (lane == sw.lb) a.k_out[pid] = sw.bot[C - 1];
            } else {
                for (int Tstep = 0; Tstep < NT; ++Tstep) {
                    T e[R + 1][C + 1];
                    T p;
                    T yv[SW::DN];
                    sw.template forward_step<true>(Tstep, e, p, yv);
                }
                scratch_fence();
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// backward kernel: forward with checkpoints, then reverse sweep with segment replay
// ------------------------------------------------------------------------------------------------
template <typename T, int BL, int D>
__global__ __launch_bounds__(kWavesPerWG* kWave) void sweep_bwd_kernel(SweepArgs<T> a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    using SW = Sweep<T, BL, D>;
    constexpr int R = SW::R, C = SW::C, NVR = SW::NVR, NVC = SW::NVC, DN = SW::DN;
    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6;
    const long slot = (long)blockIdx.x * kWavesPerWG + w;
    const long nslots = (long)gridDim.x * kWavesPerWG;
    unsigned char* mylds = smem + (size_t)w * a.lds_wave;
    SK_LDS T* ylds = (SK_LDS T*)mylds;
    SK_LDS T* glds = ylds + (size_t)a.DP * a.qpad;                // gradient accumulators for dy
    SK_LDS T* ring = (SK_LDS T*)(mylds + a.ring_off);
    T* rows = a.rows + slot * a.rows_slot;
    T* adj = a.adj + slot * a.adj_slot;
    T* ckpt = a.ckpt + slot * a.ckpt_slot;
    const int S = a.S;
    SW sw(a, lane);

    for (long pid = slot; pid < a.npairs; pid += nslots) {
        const long xi = a.gramM ? pid / a.gramM : pid;
        const long yi = a.gramM ? pid % a.gramM : pid;
        sw.dxrow = a.dxT + xi * a.xstride;
        sw.dyg = a.dyT + yi * a.ystride;
        sw.dyl = ylds;
        T* gdx = a.gdxT + xi * a.xstride;
        T* gdy = a.gdyT + yi * a.ystride;
        if (a.y_lds) {
            const int n = a.DP * a.qpad;
            for (int t = lane; t < n; t += kWave) { ylds[t] = sw.dyg[t]; glds[t] = T(0); }
        }
        const T gk = a.grad_k[pid];

        // ---- phase 1: forward, boundary rows of every strip and a checkpoint every S macro-steps ----
        for (int s = 0; s < a.ns; ++s) {
            sw.begin_strip(s, rows);
            const int NT = sw.strip_steps();
            sw.prime(0);
            for (int T0 = 0; T0 < NT; T0 += S) {
                T* cp = ckpt + ((long)(s * a.nseg + T0 / S) * NVC) * kWave + lane;
#pragma unroll
                for (int i = 0; i <= R; ++i) cp[i * kWave] = sw.left[i];
#pragma unroll
                for (int i = 0; i < C; ++i) cp[(R + 1 + i) * kWave] = sw.bot[i];
                const int T1 = T0 + S < NT ? T0 + S : NT;
                for (int Tstep = T0; Tstep < T1; ++Tstep) {
                    T e[R + 1][C + 1];
                    T p;
                    T yv[DN];
                    sw.template forward_step<true>(Tstep, e, p, yv);
                }
            }
            if (s == a.ns - 1 && lane == sw.lb && a.k_out) a.k_out[pid] = sw.bot[C - 1];
            scratch_fence();
        }

        // ---- phase 2: strips bottom-up, segments right-to-left ----
        for (int s = a.ns - 1; s >= 0; --s) {
            sw.begin_strip(s, rows);
            const int NT = sw.strip_steps();
            const int lb = sw.lb;
            const bool has_below = s < a.ns - 1;   // then lb == 63
            const T* adjr = adj + (long)((s + 1) & 1) * a.rowlen;   // written by the strip below
            T* adjw = adj + (long)(s & 1) * a.rowlen;
            // adjoint lane state
            T accL[R + 1];
            T up[C];
            T corner = T(0);
            // bottom edge feed of lane 63 (adjoint messages of the strip below): lane q of adjc holds
            // the entry of block column (column of lane 63 at the current step) - (63 - q); it rotates
            // by one lane per step and is refilled every 64 steps from adjn, loaded one chunk ahead.
            T adjc[C], adjn[C];
            int adj_end = 0;
            T gacc[DN];
#pragma unroll
            for (int i = 0; i <= R; ++i) accL[i] = T(0);
#pragma unroll
            for (int i = 0; i < C; ++i) { up[i] = T(0); adjc[i] = T(0); adjn[i] = T(0); }
#pragma unroll
            for (int i = 0; i < DN; ++i) gacc[i] = T(0);
            auto load_adj = [&](int Jb, T (&dst)[C]) {
                const int Jq = Jb - (kWave - 1 - lane);
#pragma unroll
                for (int cc = 0; cc < C; ++cc)
                    dst[cc] = (has_below && Jq >= 0 && Jq < a.nb) ? ld_scratch(adjr + (long)Jq * C + 1 + cc) : T(0);
            };
            {
                const int Jb0 = NT - 1 - lb;   // block column of lane lb at the first reverse step
                load_adj(Jb0, adjc);
                load_adj(Jb0 - kWave, adjn);
                adj_end = NT - 1 - kWave;
            }

            const int nsegs = (NT + S - 1) / S;
            for (int g = nsegs - 1; g >= 0; --g) {
                const int T0 = g * S;
                const int T1 = T0 + S < NT ? T0 + S : NT;
                // restore the forward lane state at T0 and replay the segment into the ring
                {
                    const T* cp = ckpt + ((long)(s * a.nseg + g) * NVC) * kWave + lane;
#pragma unroll
                    for (int i = 0; i <= R; ++i) sw.left[i] = ld_scratch(cp + i * kWave);
#pragma unroll
                    for (int i = 0; i < C; ++i) sw.bot[i] = ld_scratch(cp + (R + 1 + i) * kWave);
                    sw.prime(T0);
                }
                for (int Tstep = T0; Tstep < T1; ++Tstep) {
                    T e[R + 1][C + 1];
                    T p;
                    T yv[DN];
                    // keep the block input edges (forward_step leaves e[0][*] and e[*][0] untouched)
                    const bool act = sw.template forward_step<false>(Tstep, e, p, yv);
                    if (act) {
                        SK_LDS T* rp = ring + ((Tstep - T0) * NVR) * kWave + lane;
#pragma unroll
                        for (int cc = 0; cc <= C; ++cc) rp[cc * kWave] = e[0][cc];
#pragma unroll
                        for (int rr = 1; rr <= R; ++rr) rp[(C + rr) * kWave] = e[rr][0];
                    }
                }
                // walk the segment backwards; ring entries and y increments are fetched one step ahead
                T ein[NVR], ynx[DN];
                {
                    const SK_LDS T* rp = ring + ((T1 - 1 - T0) * NVR) * kWave + lane;
#pragma unroll
                    for (int v = 0; v < NVR; ++v) ein[v] = rp[v * kWave];
                    sw.fetch_y(T1 - 1 - lane, ynx);
                }
                for (int Tstep = T1 - 1; Tstep >= T0; --Tstep) {
                    if (Tstep == adj_end) {
#pragma unroll
                        for (int cc = 0; cc < C; ++cc) adjc[cc] = adjn[cc];
                        load_adj(Tstep - lb - kWave, adjn);
                        adj_end = Tstep - kWave;
                    }
                    T recv[C];
#pragma unroll
                    for (int cc = 0; cc < C; ++cc) {
                        recv[cc] = wave_from_below_or(up[cc], adjc[cc]);
                        adjc[cc] = wave_from_above(adjc[cc]);
                    }
                    const int J = Tstep - lane;
                    T e[R + 1][C + 1];
                    T yv[DN];
#pragma unroll
                    for (int cc = 0; cc <= C; ++cc) e[0][cc] = ein[cc];
#pragma unroll
                    for (int rr = 1; rr <= R; ++rr) e[rr][0] = ein[C + rr];
#pragma unroll
                    for (int c = 0; c < DN; ++c) yv[c] = ynx[c];
                    if (Tstep > T0) {
                        const SK_LDS T* rp = ring + ((Tstep - 1 - T0) * NVR) * kWave + lane;
#pragma unroll
                        for (int v = 0; v < NVR; ++v) ein[v] = rp[v * kWave];
                        sw.fetch_y(J - 1, ynx);
                    }
                    const bool active = (unsigned)J < (unsigned)sw.nbl;
                    if (active) {
                        // forward values of the block: edges from the ring, interior by Eq. (1)
                        const int b = J >> a.rs2;
                        const T p = sw.inner(b, yv);
                        SW::block_forward(e, p);
                        const T q2 = p * p;
                        const T Bc = fmaT(q2, T(-1.0 / 12.0), T(1));
                        const T Ac = fmaT(p, T(0.5), fmaT(q2, T(1.0 / 12.0), T(1)));
                        const T dA = fmaT(p, T(1.0 / 6.0), T(0.5));   // A'(p)
                        const T dB = p * T(1.0 / 6.0);                // -B'(p)
                        // adjoints of the block's nodes (first relation of Section 3.4, scatter form)
                        T gn[R + 1][C + 1];
#pragma unroll
                        for (int rr = 0; rr <= R; ++rr)
#pragma unroll
                            for (int cc = 0; cc <= C; ++cc) gn[rr][cc] = T(0);
#pragma unroll
                        for (int rr = 1; rr <= R; ++rr) gn[rr][C] = accL[rr];
#pragma unroll
                        for (int cc = 0; cc < C; ++cc) gn[R][cc + 1] += recv[cc];
                        gn[0][C] = corner;
                        if (s == a.ns - 1 && lane == lb && J == a.nb - 1) gn[R][C] = gk;
                        T accP = T(0);
#pragma unroll
                        for (int rr = R - 1; rr >= 0; --rr)
#pragma unroll
                            for (int cc = C - 1; cc >= 0; --cc) {
                                const T go = gn[rr + 1][cc + 1];
                                gn[rr + 1][cc] = fmaT(go, Ac, gn[rr + 1][cc]);
                                gn[rr][cc + 1] = fmaT(go, Ac, gn[rr][cc + 1]);
                                gn[rr][cc] = fmaT(-go, Bc, gn[rr][cc]);
                                // second relation of Section 3.4: dF/dp of this cell
                                const T loc = fmaT(e[rr + 1][cc] + e[rr][cc + 1], dA, e[rr][cc] * dB);
                                accP = fmaT(go, loc, accP);
                            }
#pragma unroll
                        for (int cc = 0; cc < C; ++cc) up[cc] = gn[0][cc + 1];
                        corner = gn[0][0];
#pragma unroll
                        for (int rr = 1; rr <= R; ++rr) accL[rr] = gn[rr][0];
                        if (lane == 0 && s > 0) {
#pragma unroll
                            for (int cc = 0; cc < C; ++cc) adjw[(long)J * C + 1 + cc] = up[cc];
                        }
                        // map to the increments (the linear transformation of Section 3.4)
                        if constexpr (D > 0) {
#pragma unroll
                            for (int c = 0; c < D; ++c) gacc[c] = fmaT(accP, yv[c], gacc[c]);
                            if (a.want_gy) {
                                if (a.y_lds) {
#pragma unroll
                                    for (int c = 0; c < D; ++c) lds_atomic_add(&glds[c * a.qpad + b], accP * sw.dxr[c]);
                                } else {
#pragma unroll
                                    for (int c = 0; c < D; ++c)
                                        unsafeAtomicAdd(&gdy[(long)c * a.qpad + b], accP * sw.dxr[c]);
                                }
                            }
                        } else {
                            const T ap = accP * a.sc;
                            for (int c = 0; c < a.d; ++c) {
                                if (a.want_gx)
                                    unsafeAtomicAdd(&gdx[(long)c * a.rpad + sw.arow], ap * sw.load_y(c, b));
                                if (a.want_gy) {
                                    const T val = ap * sw.dxrow[(long)c * a.rpad + sw.arow];
                                    if (a.y_lds) lds_atomic_add(&glds[c * a.qpad + b], val);
                                    else unsafeAtomicAdd(&gdy[(long)c * a.qpad + b], val);
                                }
                            }
                        }
                    }
                }
            }
            if constexpr (D > 0) {
                if (a.want_gx && sw.rowvalid()) {
#pragma unroll
                    for (int c = 0; c < D; ++c) unsafeAtomicAdd(&gdx[(long)c * a.rpad + sw.arow], gacc[c] * a.sc);
                }
            }
            scratch_fence();
        }
        if (a.y_lds && a.want_gy) {
            const int n = a.DP * a.qpad;
            for (int t = lane; t < n; t += kWave) {
                const T v = glds[t];
                if (v != T(0)) unsafeAtomicAdd(&gdy[t], v);
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// launchers
// ------------------------------------------------------------------------------------------------
template <typename T>
hipError_t launch_fill(T* p, long n, T v, hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    long blocks = (n + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(fill_kernel<T>, dim3((unsigned)blocks), dim3(256), 0, st, p, n, v);
    return hipGetLastError();
}

template <typename TA, typename TB>
hipError_t launch_convert(const TA* in, TB* out, long n, hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    long blocks = (n + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL((convert_kernel<TA, TB>), dim3((unsigned)blocks), dim3(256), 0, st, in, out, n);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_increments(const T* x, double* out, long npaths, int L, int d, int DP, int rpad, hipStream_t st)
{
    long total = npaths * (long)DP * rpad;
    if (total <= 0) return hipSuccess;
    long blocks = (total + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(increments_kernel<T>, dim3((unsigned)blocks), dim3(256), 0, st, x, out, npaths, L, d, DP,
                       rpad);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_finalize(const double* g, T* grad, long npaths, int L, int d, int DP, int rpad, hipStream_t st)
{
    long total = npaths * (long)L * d;
    if (total <= 0) return hipSuccess;
    long blocks = (total + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(finalize_grad_kernel<T>, dim3((unsigned)blocks), dim3(256), 0, st, g, grad, npaths, L, d, DP,
                       rpad);
    return hipGetLastError();
}

template <typename T, int BL, int D>
hipError_t launch_sweep_one(bool backward, const SweepArgs<T>& a, int grid, size_t lds, hipStream_t st)
{
    hipError_t e;
    if (backward) {
        static bool attr_done = false;
        if (!attr_done) {
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&sweep_bwd_kernel<T, BL, D>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsPerCU);
            if (e != hipSuccess) return e;
            attr_done = true;
        }
        hipLaunchKernelGGL((sweep_bwd_kernel<T, BL, D>), dim3(grid), dim3(kWavesPerWG * kWave), lds, st, a);
    } else {
        static bool attr_done = false;
        if (!attr_done) {
            e = hipFuncSetAttribute(reinterpret_cast<const void*>(&sweep_fwd_kernel<T, BL, D>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsPerCU);
            if (e != hipSuccess) return e;
            attr_done = true;
        }
        hipLaunchKernelGGL((sweep_fwd_kernel<T, BL, D>), dim3(grid), dim3(kWavesPerWG * kWave), lds, st, a);
    }
    return hipGetLastError();
}

template <typename T, int BL>
hipError_t launch_sweep_bl(bool backward, int DT, const SweepArgs<T>& a, int grid, size_t lds, hipStream_t st)
{
    switch (DT) {
        case 0: return launch_sweep_one<T, BL, 0>(backward, a, grid, lds, st);
        case 2: return launch_sweep_one<T, BL, 2>(backward, a, grid, lds, st);
        case 3: return launch_sweep_one<T, BL, 3>(backward, a, grid, lds, st);
        case 4: return launch_sweep_one<T, BL, 4>(backward, a, grid, lds, st);
        case 5: return launch_sweep_one<T, BL, 5>(backward, a, grid, lds, st);
        case 6: return launch_sweep_one<T, BL, 6>(backward, a, grid, lds, st);
        case 8: return launch_sweep_one<T, BL, 8>(backward, a, grid, lds, st);
        case 16: return launch_sweep_one<T, BL, 16>(backward, a, grid, lds, st);
        default: return hipErrorInvalidValue;
    }
}

template <typename T>
hipError_t launch_sweep(bool backward, int BL, int DT, const SweepArgs<T>& a, int grid, size_t lds, hipStream_t st)
{
    switch (BL) {
        case 0: return launch_sweep_bl<T, 0>(backward, DT, a, grid, lds, st);
        case 1: return launch_sweep_bl<T, 1>(backward, DT, a, grid, lds, st);
        case 2: return launch_sweep_bl<T, 2>(backward, DT, a, grid, lds, st);
        default: return hipErrorInvalidValue;
    }
}

template hipError_t launch_fill<float>(float*, long, float, hipStream_t);
template hipError_t launch_fill<double>(double*, long, double, hipStream_t);
template hipError_t launch_convert<float, double>(const float*, double*, long, hipStream_t);
template hipError_t launch_convert<double, float>(const double*, float*, long, hipStream_t);
template hipError_t launch_increments<float>(const float*, double*, long, int, int, int, int, hipStream_t);
template hipError_t launch_increments<double>(const double*, double*, long, int, int, int, int, hipStream_t);
template hipError_t launch_finalize<float>(const double*, float*, long, int, int, int, int, hipStream_t);
template hipError_t launch_finalize<double>(const double*, double*, long, int, int, int, int, hipStream_t);
template hipError_t launch_sweep<double>(bool, int, int, const SweepArgs<double>&, int, size_t, hipStream_t);

}  // namespace sk

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
//
// All sweeps run in double precision (see sk_api.hip for why float callers are converted at the edges).
#include <hip/hip_runtime.h>

#include <type_traits>

#include "sk_dev.h"
#include "sk_kernels.h"

namespace sk {

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

__global__ void keep_tag_kernel(unsigned long long* tag, unsigned long long val, int check, int* err)
{
    if (!check) *tag = val;
    else if (*tag != val) *err = 3;
    else if (*err == 3) *err = 0;   // an earlier call with other arguments was turned away; this one is not
}

template <typename T>
__global__ void fill_kernel(T* p, long n, T v)
{
    long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    long st = (long)gridDim.x * blockDim.x;
    for (; i < n; i += st) p[i] = v;
}

// Squared maximum mean discrepancy from the three Gram matrices (one workgroup, fixed summation order):
//   out = mean(Kxx) - 2 mean(Kxy) + mean(Kyy).
template <typename T>
__global__ __launch_bounds__(1024) void mmd2_reduce_kernel(const T* __restrict__ Kxx, const T* __restrict__ Kxy,
                                                           const T* __restrict__ Kyy, long nxx, long nxy, long nyy,
                                                           T* out)
{
    __shared__ real part[1024];
    real acc = 0.0;
    const real wxx = 1.0 / (real)nxx, wxy = -2.0 / (real)nxy, wyy = 1.0 / (real)nyy;
    for (long i = threadIdx.x; i < nxx; i += blockDim.x) acc += wxx * (real)Kxx[i];
    for (long i = threadIdx.x; i < nxy; i += blockDim.x) acc += wxy * (real)Kxy[i];
    for (long i = threadIdx.x; i < nyy; i += blockDim.x) acc += wyy * (real)Kyy[i];
    part[threadIdx.x] = acc;
    __syncthreads();
    for (int s = blockDim.x / 2; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) part[threadIdx.x] += part[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) *out = (T)part[0];
}

// dst[i] += src[i]
template <typename T>
__global__ void add_inplace_kernel(T* dst, const T* __restrict__ src, long n)
{
    long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const long st = (long)gridDim.x * blockDim.x;
    for (; i < n; i += st) dst[i] = (T)((real)dst[i] + (real)src[i]);
}

// Between the reverse sweep and the replay kernel that solves drifted pairs once more: if the reverse sweep could
// not tell which pairs drifted (*err == 2), every pair is solved again, and what the sweep has summed is dropped.
__global__ void second_chance_reset_kernel(real* g1, long n1, real* g2, long n2, const int* err)
{
    if (*err != 2) return;
    const long st = (long)gridDim.x * blockDim.x;
    for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < n1 + n2; i += st) {
        if (i < n1) g1[i] = 0.0;
        else g2[i - n1] = 0.0;
    }
}

// One set of paths for the preparation / finalisation kernels.
template <typename T>
struct PathSet {
    const T* x;      // [npaths][L][d] caller's points
    T* grad;         // [npaths][L][d] caller's gradient output (finalisation)
    real* inc;       // [npaths][rows][DS] increments (preparation)
    real* ginc;      // [npaths][rows][DS] gradient accumulators (zeroed by preparation, read by finalisation)
    long npaths;
    int L, rows;
};

// Preparation, one launch per call: increments of both path sets, padded with zeros
// (inc[path][a][c] = x[path][a+1][c] - x[path][a][c] for a < L-1, c < d: first line of the paper's
// forward listing), the gradient accumulators cleared, and the error flag cleared.
// (Lead-lag paths, Section 4, need nothing here: the sweeps work on the increments of the original paths.)
template <typename TI>
__global__ void prepare_kernel(PathSet<TI> px, PathSet<TI> py, int d, int DS, int* err, int nclear)
{
    const long nx = px.inc ? px.npaths * (long)px.rows * DS : 0;
    const long ny = py.inc ? py.npaths * (long)py.rows * DS : 0;
    long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const long st = (long)gridDim.x * blockDim.x;
    if (err) {   // the error flag and the nclear - 1 ints behind it (progress counters)
        for (long t = i; t < nclear; t += st) err[t] = 0;
    }
    for (; i < nx + ny; i += st) {
        const bool second = i >= nx;
        const PathSet<TI>& p = second ? py : px;
        const long j = second ? i - nx : i;
        const int c = (int)(j % DS);
        const long t = j / DS;
        const int a = (int)(t % p.rows);
        const long pth = t / p.rows;
        real v = 0.0;
        if (a < p.L - 1 && c < d) {
            const TI* xp = p.x + (pth * p.L + a) * (long)d + c;
            v = (real)xp[d] - (real)xp[0];
        }
        p.inc[j] = v;
        if (p.ginc) p.ginc[j] = 0.0;
    }
}

// Finalisation, one launch per backward call: grad[path][i][c] = g[path][i-1][c] - g[path][i][c]
// (out-of-range terms zero).  The increments are differences of consecutive points, so the gradient of
// a point collects the two increments it touches.
template <typename TO>
__global__ void finalize_kernel(PathSet<TO> px, PathSet<TO> py, int d, int DS, const int* err)
{
    // a bounded wait ran out (1) or the workspace held another call's forward sweep (3); 2 means that every pair was
    // solved once more by the replay kernel, whose results the accumulators then hold
    const bool bad = err != nullptr && *err != 0 && *err != 2;
    const long nx = px.grad ? px.npaths * (long)px.L * d : 0;
    const long ny = py.grad ? py.npaths * (long)py.L * d : 0;
    long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const long st = (long)gridDim.x * blockDim.x;
    for (; i < nx + ny; i += st) {
        const bool second = i >= nx;
        const PathSet<TO>& p = second ? py : px;
        const long j = second ? i - nx : i;
        const int c = (int)(j % d);
        const long t = j / d;
        const int pt = (int)(t % p.L);
        const long pth = t / p.L;
        const real* gp = p.ginc + (pth * p.rows) * (long)DS + c;
        const real hi = pt >= 1 ? gp[(long)(pt - 1) * DS] : 0.0;
        const real lo = pt < p.L - 1 ? gp[(long)pt * DS] : 0.0;
        p.grad[j] = bad ? (TO)__builtin_nan("") : (TO)(hi - lo);
    }
}

// ------------------------------------------------------------------------------------------------
// sweep building blocks
// ------------------------------------------------------------------------------------------------
template <int BL, int D, bool YLDS>
struct Sweep {
    static constexpr int R = 1 << BL;
    static constexpr int C = 1 << BL;
    static constexpr int DN = D > 0 ? D : 1;
    // Row stride (in doubles) of the increment arrays: odd, so that the 64 lanes of a wave, reading rows
    // one apart, spread over all LDS banks.
    static constexpr int DSc = D | 1;
    static constexpr int NVR = R + C + 1;   // ring: top edge (C+1) + left edge below the corner (R)
    static constexpr int NVC = R + C + 2;   // checkpoint: right edge (R+1), bottom edge (C), bottom-left corner

    const SweepArgs& a;
    const int lane;
    // per pair
    const real* dxp = nullptr;          // x increments of the pair: [rpad][DS]
    const real* dyg = nullptr;          // y increments in global memory: [qpad][DS]
    const SK_LDS real* dyl = nullptr;   // the same staged in LDS (YLDS)
    // per strip
    int s = 0, lb = 0, arow = 0;
    int nbl = 0;                        // a.nb for lanes that own a block row, 0 otherwise
    int nbm1 = 0;                       // a.nb - 1
    int rowpar = 0;                     // a.ll == 2: parity of the lead-lag step the lane's block row belongs to
    int lbw = -1;                       // lane that writes the strip's bottom row to global (-1: nobody)
    int lbany = -1;                     // lb if the bottom row goes anywhere (global row or outbox)
    real dxr[DN];
    const real* rowprev = nullptr;
    real* rowcur = nullptr;
    // forward lane state
    real left[R + 1];
    real bot[C];
    real blc = 1.0;                     // bottom-left corner e[R][0] of the last processed block
    // Top edge feed of lane 0: lane q of topc holds the boundary-row values of block column
    // (column of lane 0 at the current step) + q; the register shifts down by one lane per step.
    real topc[C];

    __device__ __forceinline__ Sweep(const SweepArgs& a_, int lane_) : a(a_), lane(lane_) {}

    __device__ __forceinline__ void begin_strip(int s_, real* rows, bool write_row)
    {
        s = s_;
        const int I = s * kWave + lane;
        nbl = I < a.mb ? a.nb : 0;
        nbm1 = a.nb - 1;
        int rem = a.mb - s * kWave - 1;
        lb = rem < kWave - 1 ? rem : kWave - 1;
        lbw = write_row ? lb : -1;
        lbany = lbw;
        lbo = -1;
        int ar = I >> a.rs1;
        arow = ar < a.r ? ar : a.r - 1;
        rowpar = a.ll == 2 ? (I >> (a.rs1 - 1)) & 1 : 0;
        if constexpr (D > 0) {
            const real* xp = dxp + (long)arow * DSc;
#pragma unroll
            for (int c = 0; c < D; ++c) dxr[c] = a.sc * xp[c];
        }
        rowprev = s > 0 ? rows + (long)(s - 1) * a.rowlen : nullptr;
        rowcur = rows + (long)s * a.rowlen;
#pragma unroll
        for (int i = 0; i <= R; ++i) left[i] = 1.0;
#pragma unroll
        for (int i = 0; i < C; ++i) bot[i] = 1.0;
    }

    __device__ __forceinline__ bool rowvalid() const { return nbl != 0; }

    // y increments of block column J (clamped into range so that every lane may load)
    __device__ __forceinline__ void fetch_y(int J, real (&yv)[DN]) const
    {
        if constexpr (D > 0) {
            const int Jc = min(max(J, 0), nbm1);
            const int b = Jc >> a.rs2;
            if constexpr (YLDS) {
                const SK_LDS real* yp = dyl + __mul24(b, DSc);
#pragma unroll
                for (int c = 0; c < D; ++c) yv[c] = yp[c];
            } else {
                const real* yp = dyg + (long)b * DSc;
#pragma unroll
                for (int c = 0; c < D; ++c) yv[c] = yp[c];
            }
        } else {
            yv[0] = 0.0;
        }
    }

    // p = 2^-(lam1+lam2) <dx[a], dy[b]> (+ the time channel's constant product), Eq. (1) third line.
    __device__ __forceinline__ real inner(int b, const real (&yv)[DN]) const
    {
        real p = a.tc;
        if constexpr (D > 0) {
#pragma unroll
            for (int c = 0; c < D; ++c) p = fma(dxr[c], yv[c], p);
        } else {
            const real* xp = dxp + (long)arow * a.DS;
            const real* yp = dyg + (long)b * a.DS;
            for (int c = 0; c < a.d; ++c) p = fma(a.sc * xp[c], yp[c], p);
        }
        return p;
    }

    // Lead-lag paths (Section 4; SweepArgs::ll) are swept on the grid of the original increments with one more level
    // of refinement: the diagonal quadrants of that level carry p, the other two the time constant alone.
    // a.ll == 2: the level lies above the blocks; whether block column J of this lane's row is off the diagonal
    __device__ __forceinline__ bool ll_off_block(int J) const
    {
        return a.ll == 2 && (((J >> (a.rs2 - 1)) ^ rowpar) & 1) != 0;
    }
    // p of the lane's block in column J
    __device__ __forceinline__ real p_block(int J, const real (&yv)[DN]) const
    {
        const real p = inner(J >> a.rs2, yv);
        return ll_off_block(J) ? a.tc : p;
    }
    // a.ll == 1: the level lies inside the block; whether cell (rr, cc) is off the diagonal quadrants
    static __device__ __forceinline__ constexpr bool cell_off(int rr, int cc)
    {
        return BL >= 1 && (((rr >> (BL > 0 ? BL - 1 : 0)) ^ (cc >> (BL > 0 ? BL - 1 : 0))) & 1) != 0;
    }
    static __device__ __forceinline__ void block_forward_ll(real (&e)[R + 1][C + 1], real p, real p0)
    {
        const real q2 = p * p, q0 = p0 * p0;
        const real Bc = fma(q2, -1.0 / 12.0, 1.0), B0 = fma(q0, -1.0 / 12.0, 1.0);
        const real Ac = fma(p, 0.5, fma(q2, 1.0 / 12.0, 1.0)), A0 = fma(p0, 0.5, fma(q0, 1.0 / 12.0, 1.0));
#pragma unroll
        for (int rr = 0; rr < R; ++rr)
#pragma unroll
            for (int cc = 0; cc < C; ++cc)
                e[rr + 1][cc + 1] = fma(e[rr + 1][cc] + e[rr][cc + 1], cell_off(rr, cc) ? A0 : Ac,
                                        -(e[rr][cc] * (cell_off(rr, cc) ? B0 : Bc)));
    }
    __device__ __forceinline__ void block_forward_any(real (&e)[R + 1][C + 1], real p) const
    {
        if (a.ll == 1) block_forward_ll(e, p, a.tc);
        else block_forward(e, p);
    }

    // Eq. (1) on the R x C cells of one block; e[0][*] and e[*][0] are given.
    static __device__ __forceinline__ void block_forward(real (&e)[R + 1][C + 1], real p)
    {
        const real q2 = p * p;
        const real Bc = fma(q2, -1.0 / 12.0, 1.0);
        const real Ac = fma(p, 0.5, fma(q2, 1.0 / 12.0, 1.0));
#pragma unroll
        for (int rr = 0; rr < R; ++rr)
#pragma unroll
            for (int cc = 0; cc < C; ++cc)
                e[rr + 1][cc + 1] = fma(e[rr + 1][cc] + e[rr][cc + 1], Ac, -(e[rr][cc] * Bc));
    }

    // Boundary-row values of block columns Jbase + lane (ones for the first strip and past the end).
    __device__ __forceinline__ void load_top(int Jbase, real (&dst)[C]) const
    {
        const int Jq = Jbase + lane;
        const bool ok = rowprev != nullptr && Jq >= 0 && Jq < a.nb;
#pragma unroll
        for (int cc = 0; cc < C; ++cc) dst[cc] = ok ? ld_scratch(rowprev + (long)Jq * C + 1 + cc) : 1.0;
    }

    // One forward macro-step: consumes ycur (the y increments of this lane's block at this step) and
    // fetches those of the next step into ynext.  Returns whether this lane processed a block.
    // EDGE = false: the top edge of lane 0 comes from the shifting register topc.
    // EDGE = true : it is given in edge[] (same value in every lane), and the bottom edge of lane lbo is
    //               also written to the outbox ring obox (cooperative mode).
    template <bool EDGE>
    __device__ __forceinline__ bool forward_step(int Tstep, const real (&ycur)[DN], real (&ynext)[DN],
                                                 real (&e)[R + 1][C + 1], const real (&edge)[C])
    {
        real recv[C];
#pragma unroll
        for (int cc = 0; cc < C; ++cc) {
            if constexpr (EDGE) {
                recv[cc] = wave_from_above_or(bot[cc], edge[cc]);
            } else {
                const real tnext = wave_shift_down(topc[cc]);
                recv[cc] = wave_from_above_or(bot[cc], topc[cc]);
                topc[cc] = tnext;
            }
        }
        const int J = Tstep - lane;
        fetch_y(J + 1, ynext);
        const bool active = (unsigned)J < (unsigned)nbl;
        if (active) {
            e[0][0] = left[0];
#pragma unroll
            for (int cc = 0; cc < C; ++cc) e[0][cc + 1] = recv[cc];
#pragma unroll
            for (int rr = 1; rr <= R; ++rr) e[rr][0] = left[rr];
            const real p = p_block(J, ycur);
            block_forward_any(e, p);
            blc = e[R][0];
#pragma unroll
            for (int rr = 0; rr <= R; ++rr) left[rr] = e[rr][C];
#pragma unroll
            for (int cc = 0; cc < C; ++cc) bot[cc] = e[R][cc + 1];
            if (lane == lbany) {   // the strip's last lane hands its bottom edge on
                if (lbw >= 0) {
                    real* wp = rowcur + (J * C + 1);
#pragma unroll
                    for (int cc = 0; cc < C; ++cc) wp[cc] = bot[cc];
                }
                if constexpr (EDGE) {
                    if (lbo >= 0) {
                        SK_LDS real* op = obox + (J & rbmask) * C;
#pragma unroll
                        for (int cc = 0; cc < C; ++cc) op[cc] = bot[cc];
                    }
                }
            }
        }
        return active;
    }

    __device__ __forceinline__ int strip_steps() const { return a.nb + lb; }

    // Lane state after the last processed block: its right edge, bottom edge and bottom-left corner.
    __device__ __forceinline__ void store_ckpt(real* cp) const
    {
#pragma unroll
        for (int i = 0; i <= R; ++i) cp[i * kWave] = left[i];
#pragma unroll
        for (int i = 0; i < C; ++i) cp[(R + 1 + i) * kWave] = bot[i];
        cp[(R + 1 + C) * kWave] = blc;
    }

    // Inverse of Eq. (1) on one block: the right edge e[*][C] and the bottom edge e[R][*] are given, every
    // other node follows from k[i,j] = ((k[i+1,j] + k[i,j+1]) A - k[i+1,j+1]) / B.
    static __device__ __forceinline__ void block_uncompute(real (&e)[R + 1][C + 1], real Ac, real invB)
    {
#pragma unroll
        for (int rr = R - 1; rr >= 0; --rr)
#pragma unroll
            for (int cc = C - 1; cc >= 0; --cc)
                e[rr][cc] = fma(e[rr + 1][cc] + e[rr][cc + 1], Ac, -e[rr + 1][cc + 1]) * invB;
    }

    // Adjoints of one block whose forward values e are all known (first relation of Section 3.4 in scatter
    // form) and its dF/dp (second relation).
    __device__ __forceinline__ real adjoint_block(const real (&e)[R + 1][C + 1], real p, real Ac, real Bc,
                                                  const real (&recv)[C], real (&accL)[R + 1], real& corner,
                                                  real (&up)[C]) const
    {
        const real dA = fma(p, 1.0 / 6.0, 0.5);   // A'(p)
        const real dB = p * (1.0 / 6.0);          // -B'(p)
        real gn[R + 1][C + 1];
#pragma unroll
        for (int rr = 0; rr <= R; ++rr)
#pragma unroll
            for (int cc = 0; cc <= C; ++cc) gn[rr][cc] = 0.0;
#pragma unroll
        for (int rr = 1; rr <= R; ++rr) gn[rr][C] = accL[rr];
#pragma unroll
        for (int cc = 0; cc < C; ++cc) gn[R][cc + 1] += recv[cc];
        gn[0][C] = corner;
        real accP = 0.0;
#pragma unroll
        for (int rr = R - 1; rr >= 0; --rr)
#pragma unroll
            for (int cc = C - 1; cc >= 0; --cc) {
                const real go = gn[rr + 1][cc + 1];
                gn[rr + 1][cc] = fma(go, Ac, gn[rr + 1][cc]);
                gn[rr][cc + 1] = fma(go, Ac, gn[rr][cc + 1]);
                gn[rr][cc] = fma(-go, Bc, gn[rr][cc]);
                const real loc = fma(e[rr + 1][cc] + e[rr][cc + 1], dA, e[rr][cc] * dB);
                accP = fma(go, loc, accP);
            }
#pragma unroll
        for (int cc = 0; cc < C; ++cc) up[cc] = gn[0][cc + 1];
        corner = gn[0][0];
#pragma unroll
        for (int rr = 1; rr <= R; ++rr) accL[rr] = gn[rr][0];
        return accP;
    }

    // One reverse step of the un-compute kernels on one block: e holds the right edge e[*][C] and the bottom edge
    // e[R][*] on entry and every node on exit; returns the block's dF/dp.
    __device__ __forceinline__ real uncompute_adjoint(real (&e)[R + 1][C + 1], real p, const real (&recv)[C],
                                                      real (&accL)[R + 1], real& corner, real (&up)[C]) const
    {
        if (a.ll == 1) return uncompute_adjoint_t<true>(e, p, a.tc, recv, accL, corner, up);
        return uncompute_adjoint_t<false>(e, p, p, recv, accL, corner, up);
    }
    // CHK: lead-lag level inside the block (see block_forward_ll and reverse_block_t)
    template <bool CHK>
    __device__ __forceinline__ real uncompute_adjoint_t(real (&e)[R + 1][C + 1], real p, real p0, const real (&recv)[C],
                                                        real (&accL)[R + 1], real& corner, real (&up)[C]) const
    {
        const real q2 = p * p;
        const real Bc = fma(q2, -1.0 / 12.0, 1.0);
        const real Ac = fma(p, 0.5, fma(q2, 1.0 / 12.0, 1.0));
        real invB = __builtin_amdgcn_rcp(Bc);
        invB = fma(fma(-Bc, invB, 1.0), invB, invB);
        if constexpr (!CHK) {
            block_uncompute(e, Ac, invB);
            return adjoint_block(e, p, Ac, Bc, recv, accL, corner, up);
        } else {
            const real q0 = p0 * p0;
            const real B0 = fma(q0, -1.0 / 12.0, 1.0);
            const real A0 = fma(p0, 0.5, fma(q0, 1.0 / 12.0, 1.0));
            real invB0 = __builtin_amdgcn_rcp(B0);
            invB0 = fma(fma(-B0, invB0, 1.0), invB0, invB0);
            const real dA = fma(p, 1.0 / 6.0, 0.5);   // A'(p)
            const real dB = p * (1.0 / 6.0);          // -B'(p)
            real gn[R + 1][C + 1];
#pragma unroll
            for (int rr = 0; rr <= R; ++rr)
#pragma unroll
                for (int cc = 0; cc <= C; ++cc) gn[rr][cc] = 0.0;
#pragma unroll
            for (int rr = 1; rr <= R; ++rr) gn[rr][C] = accL[rr];
#pragma unroll
            for (int cc = 0; cc < C; ++cc) gn[R][cc + 1] += recv[cc];
            gn[0][C] = corner;
            real accP = 0.0;
#pragma unroll
            for (int rr = R - 1; rr >= 0; --rr)
#pragma unroll
                for (int cc = C - 1; cc >= 0; --cc) {
                    const bool off = cell_off(rr, cc);
                    const real Aq = off ? A0 : Ac, Bq = off ? B0 : Bc, iBq = off ? invB0 : invB;
                    e[rr][cc] = fma(e[rr + 1][cc] + e[rr][cc + 1], Aq, -e[rr + 1][cc + 1]) * iBq;
                    const real go = gn[rr + 1][cc + 1];
                    gn[rr + 1][cc] = fma(go, Aq, gn[rr + 1][cc]);
                    gn[rr][cc + 1] = fma(go, Aq, gn[rr][cc + 1]);
                    gn[rr][cc] = fma(-go, Bq, gn[rr][cc]);
                    if (off) continue;
                    const real loc = fma(e[rr + 1][cc] + e[rr][cc + 1], dA, e[rr][cc] * dB);
                    accP = fma(go, loc, accP);
                }
#pragma unroll
            for (int cc = 0; cc < C; ++cc) up[cc] = gn[0][cc + 1];
            corner = gn[0][0];
#pragma unroll
            for (int rr = 1; rr <= R; ++rr) accL[rr] = gn[rr][0];
            return accP;
        }
    }

    // Steps [T0, T1) of the forward sweep of the current strip, T1 - T0 <= 64 and topc loaded for T0.
    // f(Tstep, active, e) is called after every step.
    template <class F>
    __device__ __forceinline__ void forward_run(int T0, int T1, F&& f)
    {
        real ya[DN], yb[DN];
        real none[C];
#pragma unroll
        for (int cc = 0; cc < C; ++cc) none[cc] = 0.0;
        fetch_y(T0 - lane, ya);
        int Tstep = T0;
        for (; Tstep + 2 <= T1; Tstep += 2) {
            {
                real e[R + 1][C + 1];
                const bool act = forward_step<false>(Tstep, ya, yb, e, none);
                f(Tstep, act, e);
            }
            {
                real e[R + 1][C + 1];
                const bool act = forward_step<false>(Tstep + 1, yb, ya, e, none);
                f(Tstep + 1, act, e);
            }
        }
        if (Tstep < T1) {
            real e[R + 1][C + 1];
            const bool act = forward_step<false>(Tstep, ya, yb, e, none);
            f(Tstep, act, e);
        }
    }

    // ---- cooperative mode: the strips of one pair run on different waves of one workgroup and hand
    // their boundary rows over through small rings in LDS ----
    SK_LDS real* obox = nullptr;         // this wave's outbox ring: (rbmask + 1) columns x C values
    const SK_LDS real* ibox = nullptr;   // outbox of the wave that runs the upstream strip (or all ones)
    int rbmask = 0;
    int lbo = -1;                        // lane that writes the outbox (-1: nobody)

    __device__ __forceinline__ void read_edge(int col, real (&dst)[C]) const
    {
        int cidx = col < a.nb ? col : a.nb - 1;
        const SK_LDS real* ip = ibox + (cidx & rbmask) * C;
#pragma unroll
        for (int cc = 0; cc < C; ++cc) dst[cc] = ip[cc];
    }

    // Steps [T0, T1) with the top edge of lane 0 read from ibox one step ahead; edge holds the values
    // for step T0 on entry and those for step T1 on exit.
    template <class F>
    __device__ __forceinline__ void forward_run_coop(int T0, int T1, real (&edge)[C], F&& f)
    {
        real ya[DN], yb[DN], eb[C];
        fetch_y(T0 - lane, ya);
        int Tstep = T0;
        for (; Tstep + 2 <= T1; Tstep += 2) {
            {
                real e[R + 1][C + 1];
                read_edge(Tstep + 1, eb);
                const bool act = forward_step<true>(Tstep, ya, yb, e, edge);
                f(Tstep, act, e);
            }
            {
                real e[R + 1][C + 1];
                read_edge(Tstep + 2, edge);
                const bool act = forward_step<true>(Tstep + 1, yb, ya, e, eb);
                f(Tstep + 1, act, e);
            }
        }
        if (Tstep < T1) {
            real e[R + 1][C + 1];
            read_edge(Tstep + 1, eb);
            const bool act = forward_step<true>(Tstep, ya, yb, e, edge);
            f(Tstep, act, e);
#pragma unroll
            for (int cc = 0; cc < C; ++cc) edge[cc] = eb[cc];
        }
    }

    // Adjoints of one block (first relation of Section 3.4 in scatter form) and its dF/dp (second
    // relation).  ein: block input edges of the forward values; recv: adjoint messages from the block
    // row below; accL / corner / up: adjoint state carried to the left neighbour block and upwards.
    __device__ __forceinline__ real reverse_block(const real (&ein)[NVR], real p, const real (&recv)[C], bool seed,
                                                  real gk, real (&accL)[R + 1], real& corner, real (&up)[C]) const
    {
        if (a.ll == 1) return reverse_block_t<true>(ein, p, a.tc, recv, seed, gk, accL, corner, up);
        return reverse_block_t<false>(ein, p, p, recv, seed, gk, accL, corner, up);
    }
    // CHK: lead-lag level inside the block; the cells off its diagonal quadrants have the constant p0, take part in
    // both recurrences and add nothing to dF/dp
    template <bool CHK>
    __device__ __forceinline__ real reverse_block_t(const real (&ein)[NVR], real p, real p0, const real (&recv)[C],
                                                    bool seed, real gk, real (&accL)[R + 1], real& corner,
                                                    real (&up)[C]) const
    {
        real e[R + 1][C + 1];
#pragma unroll
        for (int cc = 0; cc <= C; ++cc) e[0][cc] = ein[cc];
#pragma unroll
        for (int rr = 1; rr <= R; ++rr) e[rr][0] = ein[C + rr];
        if constexpr (CHK) block_forward_ll(e, p, p0);
        else block_forward(e, p);
        const real q2 = p * p, q0 = p0 * p0;
        const real Bc = fma(q2, -1.0 / 12.0, 1.0), B0 = fma(q0, -1.0 / 12.0, 1.0);
        const real Ac = fma(p, 0.5, fma(q2, 1.0 / 12.0, 1.0)), A0 = fma(p0, 0.5, fma(q0, 1.0 / 12.0, 1.0));
        const real dA = fma(p, 1.0 / 6.0, 0.5);   // A'(p)
        const real dB = p * (1.0 / 6.0);          // -B'(p)
        real gn[R + 1][C + 1];
#pragma unroll
        for (int rr = 0; rr <= R; ++rr)
#pragma unroll
            for (int cc = 0; cc <= C; ++cc) gn[rr][cc] = 0.0;
#pragma unroll
        for (int rr = 1; rr <= R; ++rr) gn[rr][C] = accL[rr];
#pragma unroll
        for (int cc = 0; cc < C; ++cc) gn[R][cc + 1] += recv[cc];
        gn[0][C] = corner;
        if (seed) gn[R][C] = gk;
        real accP = 0.0;
#pragma unroll
        for (int rr = R - 1; rr >= 0; --rr)
#pragma unroll
            for (int cc = C - 1; cc >= 0; --cc) {
                const bool off = CHK && cell_off(rr, cc);
                const real Aq = off ? A0 : Ac, Bq = off ? B0 : Bc;
                const real go = gn[rr + 1][cc + 1];
                gn[rr + 1][cc] = fma(go, Aq, gn[rr + 1][cc]);
                gn[rr][cc + 1] = fma(go, Aq, gn[rr][cc + 1]);
                gn[rr][cc] = fma(-go, Bq, gn[rr][cc]);
                if (off) continue;
                const real loc = fma(e[rr + 1][cc] + e[rr][cc + 1], dA, e[rr][cc] * dB);
                accP = fma(go, loc, accP);
            }
#pragma unroll
        for (int cc = 0; cc < C; ++cc) up[cc] = gn[0][cc + 1];
        corner = gn[0][0];
#pragma unroll
        for (int rr = 1; rr <= R; ++rr) accL[rr] = gn[rr][0];
        return accP;
    }

    // The linear map of Section 3.4 for one block: accP = sum of dF/dp over the block's cells.
    __device__ __forceinline__ void accumulate_grads(real accP, int b, const real (&yv)[DN], real (&gacc)[DN],
                                                     SK_LDS real* glds, real* gdx, real* gdy) const
    {
        if constexpr (D > 0) {
#pragma unroll
            for (int c = 0; c < D; ++c) gacc[c] = fma(accP, yv[c], gacc[c]);
            if (a.want_gy) {
                if constexpr (YLDS) {
                    SK_LDS real* gp = glds + b * DSc;
#pragma unroll
                    for (int c = 0; c < D; ++c) lds_atomic_add(gp + c, accP * dxr[c]);
                } else {
                    real* gp = gdy + (long)b * DSc;
#pragma unroll
                    for (int c = 0; c < D; ++c) unsafeAtomicAdd(gp + c, accP * dxr[c]);
                }
            }
        } else {
            const real ap = accP * a.sc;
            const real* xp = dxp + (long)arow * a.DS;
            const real* yp = dyg + (long)b * a.DS;
            for (int c = 0; c < a.d; ++c) {
                if (a.want_gx) unsafeAtomicAdd(&gdx[(long)arow * a.DS + c], ap * yp[c]);
                if (a.want_gy) unsafeAtomicAdd(&gdy[(long)b * a.DS + c], ap * xp[c]);
            }
        }
    }

    __device__ __forceinline__ void flush_gdx(const real (&gacc)[DN], real* gdx) const
    {
        if constexpr (D > 0) {
            if (a.want_gx && rowvalid()) {
                real* gp = gdx + (long)arow * DSc;
#pragma unroll
                for (int c = 0; c < D; ++c) unsafeAtomicAdd(gp + c, gacc[c] * a.sc);
            }
        }
    }
};

struct NoHook {
    template <class E> __device__ __forceinline__ void operator()(int, bool, E&) const {}
};


// ------------------------------------------------------------------------------------------------
// forward kernel: one wave per pair, kWavesPerWG independent waves per workgroup
// ------------------------------------------------------------------------------------------------
template <int BL, int D, bool YLDS>
__global__ __launch_bounds__(kWavesPerWG* kWave) void sweep_fwd_kernel(SweepArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    using SW = Sweep<BL, D, YLDS>;
    constexpr int C = SW::C;
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave index: uniform, and known to be
    const long slot = (long)blockIdx.x * kWavesPerWG + w;
    const long nslots = (long)gridDim.x * kWavesPerWG;
    SK_LDS real* ylds = (SK_LDS real*)(smem + (size_t)w * a.lds_wave);
    real* rows = a.rows + slot * a.rows_slot;
    SW sw(a, lane);

    for (long pid = slot; pid < a.npairs; pid += nslots) {
        long xi, yi;
        pair_ids(a, pid, xi, yi);
        sw.dxp = a.dx + xi * a.xstride;
        sw.dyg = a.dy + yi * a.ystride;
        sw.dyl = ylds;
        if constexpr (YLDS) {
            const int n = a.q * a.DS;
            for (int t = lane; t < n; t += kWave) ylds[t] = sw.dyg[t];
        }
        for (int s = 0; s < a.ns; ++s) {
            const bool last = s == a.ns - 1;
            sw.begin_strip(s, rows, !last);
            const int NT = sw.strip_steps();
            real topn[C];
            sw.load_top(0, sw.topc);
            for (int Tc = 0; Tc < NT; Tc += kWave) {
                if (Tc > 0) {
#pragma unroll
                    for (int cc = 0; cc < C; ++cc) sw.topc[cc] = topn[cc];
                }
                sw.load_top(Tc + kWave, topn);   // one chunk ahead
                const int Te = Tc + kWave < NT ? Tc + kWave : NT;
                sw.forward_run(Tc, Te, NoHook());
            }
            if (last) {
                if (lane == sw.lb) a.k_out[pid] = sw.bot[C - 1];
            } else {
                scratch_fence();
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// backward kernel: forward with checkpoints, then reverse sweep with segment replay
// ------------------------------------------------------------------------------------------------
template <int BL, int D, bool YLDS>
__global__ __launch_bounds__(kWavesPerWG* kWave) void sweep_bwd_kernel(SweepArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    using SW = Sweep<BL, D, YLDS>;
    constexpr int R = SW::R, C = SW::C, NVR = SW::NVR, NVC = SW::NVC, DN = SW::DN;
    // fetch ring entries and y increments one reverse step ahead, unless the block is so large that the
    // second register set would not fit
    constexpr bool LOOKAHEAD = BL < 2;
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave index: uniform, and known to be
    const long slot = (long)blockIdx.x * kWavesPerWG + w;
    const long nslots = (long)gridDim.x * kWavesPerWG;
    unsigned char* mylds = smem + (size_t)w * a.lds_wave;
    SK_LDS real* ylds = (SK_LDS real*)mylds;
    SK_LDS real* glds = ylds + (size_t)a.q * a.DS;              // gradient accumulators for dy (YLDS)
    SK_LDS real* ring = (SK_LDS real*)(mylds + a.ring_off);
    real* rows = a.rows + slot * a.rows_slot;
    real* adj = a.adj + slot * a.adj_slot;
    real* ckpt = a.ckpt + slot * a.ckpt_slot;
    const int S = a.S;
    SW sw(a, lane);
    // As the launch that solves drifted pairs once more, the kernel works through the list the reverse sweep left
    // (through every pair if that sweep could not tell which ones drifted); an empty list ends it at once.
    const bool listed = a.second_chance != 0 && *a.err != 2;
    const long count = a.second_chance == 0 ? a.npairs : (listed ? (long)*a.bad_count : a.npairs);
    const bool own_edges = a.second_chance == 2;   // a call that works on the caller's arrays (pairs of double paths)

    for (long it = slot; it < count; it += nslots) {
        const long pid = listed ? (long)a.bad_list[it] : it;
        long xi, yi;
        pair_ids(a, pid, xi, yi);
        sw.dxp = a.dx + xi * a.xstride;
        sw.dyg = a.dy + yi * a.ystride;
        sw.dyl = ylds;
        real* gdx = a.gdx + xi * a.xstride;
        real* gdy = a.gdy + yi * a.ystride;
        if (own_edges) {
            // increments of the pair (first line of the paper's forward listing), zero padded, and cleared sums
            real* dxw = const_cast<real*>(a.dx) + xi * a.xstride;
            real* dyw = const_cast<real*>(a.dy) + yi * a.ystride;
            const real* xp = a.xraw + xi * (long)a.L1 * a.d;
            const real* yp = a.yraw + yi * (long)a.L2 * a.d;
            for (int t = lane; t < a.rpad * a.DS; t += kWave) {
                const int r_ = t / a.DS, c = t - r_ * a.DS;
                dxw[t] = (r_ < a.r && c < a.d) ? xp[(long)(r_ + 1) * a.d + c] - xp[(long)r_ * a.d + c] : 0.0;
                gdx[t] = 0.0;
            }
            for (int t = lane; t < a.qpad * a.DS; t += kWave) {
                const int r_ = t / a.DS, c = t - r_ * a.DS;
                dyw[t] = (r_ < a.q && c < a.d) ? yp[(long)(r_ + 1) * a.d + c] - yp[(long)r_ * a.d + c] : 0.0;
                gdy[t] = 0.0;
            }
            // the sweep reads the increments with ordinary loads: make the stores visible to them
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        }
        if constexpr (YLDS) {
            const int n = a.q * a.DS;
            for (int t = lane; t < n; t += kWave) { ylds[t] = ld_scratch(sw.dyg + t); glds[t] = 0.0; }
        }
        const real gk = a.grad_k[pid];

        // ---- phase 1: forward, boundary rows of every strip and a checkpoint every S macro-steps ----
        for (int s = 0; s < a.ns; ++s) {
            sw.begin_strip(s, rows, true);
            const int NT = sw.strip_steps();
            real topn[C];
            sw.load_top(0, sw.topc);
            for (int Tc = 0; Tc < NT; Tc += kWave) {
                if (Tc > 0) {
#pragma unroll
                    for (int cc = 0; cc < C; ++cc) sw.topc[cc] = topn[cc];
                }
                sw.load_top(Tc + kWave, topn);
                const int Te = Tc + kWave < NT ? Tc + kWave : NT;
                for (int T0 = Tc; T0 < Te; T0 += S) {
                    sw.store_ckpt(ckpt + ((long)(s * a.nseg + T0 / S) * NVC) * kWave + lane);
                    sw.forward_run(T0, T0 + S < Te ? T0 + S : Te, NoHook());
                }
            }
            if (s == a.ns - 1 && lane == sw.lb && a.k_out) a.k_out[pid] = sw.bot[C - 1];
            scratch_fence();
        }

        // ---- phase 2: strips bottom-up, segments right-to-left ----
        for (int s = a.ns - 1; s >= 0; --s) {
            sw.begin_strip(s, rows, false);
            const int NT = sw.strip_steps();
            const int lb = sw.lb;
            const bool has_below = s < a.ns - 1;   // then lb == 63
            const real* adjr = adj + (long)((s + 1) & 1) * a.rowlen;   // written by the strip below
            real* adjw = adj + (long)(s & 1) * a.rowlen;
            // adjoint lane state
            real accL[R + 1];
            real up[C];
            real corner = 0.0;
            // Bottom edge feed of lane 63 (adjoint messages of the strip below): lane q of adjc holds the
            // entry of block column (column of lane 63 at the current step) - (63 - q); it shifts up by
            // one lane per step and is refilled every 64 steps from adjn, loaded one chunk ahead.
            real adjc[C], adjn[C];
            int adj_end = 0;
            real gacc[DN];
#pragma unroll
            for (int i = 0; i <= R; ++i) accL[i] = 0.0;
#pragma unroll
            for (int i = 0; i < C; ++i) up[i] = 0.0;
#pragma unroll
            for (int i = 0; i < DN; ++i) gacc[i] = 0.0;
            auto load_adj = [&](int Jb, real (&dst)[C]) {
                const int Jq = Jb - (kWave - 1 - lane);
                const bool ok = has_below && Jq >= 0 && Jq < a.nb;
#pragma unroll
                for (int cc = 0; cc < C; ++cc) dst[cc] = ok ? ld_scratch(adjr + (long)Jq * C + 1 + cc) : 0.0;
            };
            {
                const int Jb0 = NT - 1 - lb;   // block column of lane lb at the first reverse step
                load_adj(Jb0, adjc);
                load_adj(Jb0 - kWave, adjn);
                adj_end = NT - 1 - kWave;
            }

            const int nsegs = (NT + S - 1) / S;
            // checkpoint and top feed of a segment are loaded one segment ahead
            real cpn[NVC], topn[C];
            auto load_segment = [&](int g) {
                const real* cp = ckpt + ((long)(s * a.nseg + g) * NVC) * kWave + lane;
#pragma unroll
                for (int i = 0; i < NVC; ++i) cpn[i] = ld_scratch(cp + i * kWave);
                sw.load_top(g * S, topn);
            };
            load_segment(nsegs - 1);
            for (int g = nsegs - 1; g >= 0; --g) {
                const int T0 = g * S;
                const int T1 = T0 + S < NT ? T0 + S : NT;
                // restore the forward lane state at T0 and replay the segment into the ring
#pragma unroll
                for (int i = 0; i <= R; ++i) sw.left[i] = cpn[i];
#pragma unroll
                for (int i = 0; i < C; ++i) { sw.bot[i] = cpn[R + 1 + i]; sw.topc[i] = topn[i]; }
                if (g > 0) load_segment(g - 1);
                sw.forward_run(T0, T1, [&](int Tstep, bool act, real (&e)[R + 1][C + 1]) {
                    if (act) {
                        // keep the block input edges (the step leaves e[0][*] and e[*][0] untouched)
                        SK_LDS real* rp = ring + ((Tstep - T0) * NVR) * kWave + lane;
#pragma unroll
                        for (int cc = 0; cc <= C; ++cc) rp[cc * kWave] = e[0][cc];
#pragma unroll
                        for (int rr = 1; rr <= R; ++rr) rp[(C + rr) * kWave] = e[rr][0];
                    }
                });

                // walk the segment backwards; ring entries and y increments are fetched one step ahead
                auto fetch_ring = [&](int Tstep, real (&ein)[NVR]) {
                    const SK_LDS real* rp = ring + ((Tstep - T0) * NVR) * kWave + lane;
#pragma unroll
                    for (int v = 0; v < NVR; ++v) ein[v] = rp[v * kWave];
                };
                auto reverse_step = [&](int Tstep, const real (&ein)[NVR], const real (&yv)[DN], real (&einn)[NVR],
                                        real (&yvn)[DN]) {
                    if (Tstep == adj_end) {
#pragma unroll
                        for (int cc = 0; cc < C; ++cc) adjc[cc] = adjn[cc];
                        load_adj(Tstep - lb - kWave, adjn);
                        adj_end = Tstep - kWave;
                    }
                    real recv[C];
#pragma unroll
                    for (int cc = 0; cc < C; ++cc) {
                        const real anext = wave_shift_up(adjc[cc]);
                        recv[cc] = wave_from_below_or(up[cc], adjc[cc]);
                        adjc[cc] = anext;
                    }
                    const int J = Tstep - lane;
                    if constexpr (LOOKAHEAD) {
                        if (Tstep > T0) {
                            fetch_ring(Tstep - 1, einn);
                            sw.fetch_y(J - 1, yvn);
                        }
                    }
                    const bool active = (unsigned)J < (unsigned)sw.nbl;
                    if (active) {
                        const int b = J >> a.rs2;
                        const real p = sw.p_block(J, yv);
                        const bool seed = s == a.ns - 1 && lane == lb && J == a.nb - 1;
                        real accP = sw.reverse_block(ein, p, recv, seed, gk, accL, corner, up);
                        if (sw.ll_off_block(J)) accP = 0.0;   // the block's p is a constant
                        if (lane == 0 && s > 0) {
                            real* wp = adjw + (J * C + 1);
#pragma unroll
                            for (int cc = 0; cc < C; ++cc) wp[cc] = up[cc];
                        }
                        sw.accumulate_grads(accP, b, yv, gacc, glds, gdx, gdy);
                    }
                };
                if constexpr (LOOKAHEAD) {
                    real ea[NVR], eb[NVR], ya[DN], yb[DN];
                    fetch_ring(T1 - 1, ea);
                    sw.fetch_y(T1 - 1 - lane, ya);
                    int Tstep = T1 - 1;
                    for (; Tstep - 1 >= T0; Tstep -= 2) {
                        reverse_step(Tstep, ea, ya, eb, yb);
                        reverse_step(Tstep - 1, eb, yb, ea, ya);
                    }
                    if (Tstep >= T0) reverse_step(Tstep, ea, ya, eb, yb);
                } else {
                    for (int Tstep = T1 - 1; Tstep >= T0; --Tstep) {
                        real ea[NVR], ya[DN];
                        fetch_ring(Tstep, ea);
                        sw.fetch_y(Tstep - lane, ya);
                        reverse_step(Tstep, ea, ya, ea, ya);
                    }
                }
            }
            sw.flush_gdx(gacc, gdx);
            scratch_fence();
        }
        if constexpr (YLDS) {
            if (a.want_gy) {
                const int n = a.q * a.DS;
                for (int t = lane; t < n; t += kWave) {
                    const real v = glds[t];
                    if (v != 0.0) unsafeAtomicAdd(&gdy[t], v);
                }
            }
        }
        if (own_edges) {
            // the gradient of a point collects the two increments it touches (the linear map of Section 3.4)
            scratch_fence();
            const int d = a.d;
            if (a.gxraw) {
                real* go = a.gxraw + xi * (long)a.L1 * d;
                for (int t = lane; t < a.L1 * d; t += kWave) {
                    const int pt = t / d, c = t - pt * d;
                    const real hi = pt >= 1 ? ld_scratch(gdx + (long)(pt - 1) * a.DS + c) : 0.0;
                    const real lo = pt < a.L1 - 1 ? ld_scratch(gdx + (long)pt * a.DS + c) : 0.0;
                    go[t] = hi - lo;
                }
            }
            if (a.gyraw) {
                real* go = a.gyraw + yi * (long)a.L2 * d;
                for (int t = lane; t < a.L2 * d; t += kWave) {
                    const int pt = t / d, c = t - pt * d;
                    const real hi = pt >= 1 ? ld_scratch(gdy + (long)(pt - 1) * a.DS + c) : 0.0;
                    const real lo = pt < a.L2 - 1 ? ld_scratch(gdy + (long)pt * a.DS + c) : 0.0;
                    go[t] = hi - lo;
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// backward kernel, un-compute variant: forward with checkpoints, then ONE reverse sweep that recovers
// the forward values by inverting Eq. (1) block by block (no replay, no ring)
// ------------------------------------------------------------------------------------------------
// The reverse sweep starts every segment of S macro-steps from the exact lane state of a checkpoint
// (right edge, bottom edge and bottom-left corner of each lane's last block) and walks backwards: a lane
// recovers all nodes of its block from the right and bottom edges, which leaves it with the right edge
// of its previous block; the bottom edge of that block is the top edge the lane below recovered one
// step earlier (one more DPP hand-over, next to the adjoint messages).  Rounding errors of the inverse
// recurrence grow with the number of steps, so S is short, and at every checkpoint the recovered state
// is compared with the exact one (at the left end: with the boundary value 1): a drift above kDriftTol of the
// row's largest value raises the flag that makes the call solve every pair once more with the replay kernel
// above (this kernel's gradient sums are on their way by then, so it cannot leave out the one pair); such
// inputs have increment inner products of order one.
template <int BL, int D, bool YLDS>
__global__ __launch_bounds__(kWavesPerWG* kWave) void sweep_bwdu_kernel(SweepArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    using SW = Sweep<BL, D, YLDS>;
    constexpr int R = SW::R, C = SW::C, NVC = SW::NVC, DN = SW::DN;
    constexpr int C2 = 2 * C;   // feed width: adjoint messages and recovered top edge
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave index: uniform, and known to be
    const long slot = (long)blockIdx.x * kWavesPerWG + w;
    const long nslots = (long)gridDim.x * kWavesPerWG;
    unsigned char* mylds = smem + (size_t)w * a.lds_wave;
    SK_LDS real* ylds = (SK_LDS real*)mylds;
    SK_LDS real* glds = ylds + (size_t)a.q * a.DS;
    real* rows = a.rows + slot * a.rows_slot;
    real* adj = a.adj + slot * a.adj_slot;
    real* ckpt = a.ckpt + slot * a.ckpt_slot;
    const int S = a.S;
    const int nck = a.nseg + 1;   // checkpoints per strip
    const long adjlen = 2L * a.rowlen;
    SW sw(a, lane);

    for (long pid = slot; pid < a.npairs; pid += nslots) {
        long xi, yi;
        pair_ids(a, pid, xi, yi);
        sw.dxp = a.dx + xi * a.xstride;
        sw.dyg = a.dy + yi * a.ystride;
        sw.dyl = ylds;
        real* gdx = a.gdx + xi * a.xstride;
        real* gdy = a.gdy + yi * a.ystride;
        if constexpr (YLDS) {
            const int n = a.q * a.DS;
            for (int t = lane; t < n; t += kWave) { ylds[t] = sw.dyg[t]; glds[t] = 0.0; }
        }
        const real gk = a.grad_k[pid];

        // ---- phase 1: forward; boundary rows of every strip, a checkpoint every S macro-steps and one
        // at the end of the strip ----
        for (int s = 0; s < a.ns; ++s) {
            sw.begin_strip(s, rows, true);
            if (lane == sw.lb) sw.rowcur[0] = 1.0;   // node column 0 of the boundary row
            const int NT = sw.strip_steps();
            real topn[C];
            sw.load_top(0, sw.topc);
            for (int Tc = 0; Tc < NT; Tc += kWave) {
                if (Tc > 0) {
#pragma unroll
                    for (int cc = 0; cc < C; ++cc) sw.topc[cc] = topn[cc];
                }
                sw.load_top(Tc + kWave, topn);
                const int Te = Tc + kWave < NT ? Tc + kWave : NT;
                for (int T0 = Tc; T0 < Te; T0 += S) {
                    sw.store_ckpt(ckpt + ((long)(s * nck + T0 / S) * NVC) * kWave + lane);
                    sw.forward_run(T0, T0 + S < Te ? T0 + S : Te, NoHook());
                }
            }
            sw.store_ckpt(ckpt + ((long)(s * nck + (NT + S - 1) / S) * NVC) * kWave + lane);
            if (s == a.ns - 1 && lane == sw.lb && a.k_out) a.k_out[pid] = sw.bot[C - 1];
            scratch_fence();
        }

        // ---- phase 2: strips bottom-up, segments right-to-left ----
        bool drift = false;
        for (int s = a.ns - 1; s >= 0; --s) {
            real kscale = 1.0;
            sw.begin_strip(s, rows, false);
            const int NT = sw.strip_steps();
            const int lb = sw.lb;
            const bool full = lb == kWave - 1;
            const bool is_lb = lane == lb;
            const bool has_below = s < a.ns - 1;   // then lb == 63
            const real* adjr = adj + (long)((s + 1) & 1) * adjlen;   // written by the strip below: [J][2C]
            real* adjw = adj + (long)(s & 1) * adjlen;
            const real* krow = rows + (long)(a.ns - 1) * a.rowlen;   // bottom row of the grid
            real accL[R + 1], up[C], ktop[C];
            real corner = 0.0;
            real gacc[DN];
#pragma unroll
            for (int i = 0; i <= R; ++i) accL[i] = 0.0;
            // dF/dk at the far corner enters as the carried adjoint of the last lane's first block
            if (s == a.ns - 1 && is_lb) accL[R] = gk;
#pragma unroll
            for (int i = 0; i < C; ++i) { up[i] = 0.0; ktop[i] = 0.0; }
#pragma unroll
            for (int i = 0; i < DN; ++i) gacc[i] = 0.0;
            // Feed of the strip's last lane: lane q <= lb of fc holds, for block column
            // (column of lane lb at the current step) - (lb - q), the C adjoint messages of the strip below
            // followed by the C node values under the strip; it shifts up one lane per step and is
            // refilled every lb + 1 steps from fn, loaded one chunk ahead.
            real fc[C2], fn[C2];
            const int CL = lb + 1;
            int f_end = 0;
            auto load_feed = [&](int Jb, real (&dst)[C2]) {
                const int Jq = Jb - (lb - lane);
                const bool ok = lane <= lb && Jq >= 0 && Jq < a.nb;
#pragma unroll
                for (int cc = 0; cc < C; ++cc) {
                    dst[cc] = (ok && has_below) ? ld_scratch(adjr + (long)Jq * C2 + cc) : 0.0;
                    dst[C + cc] = !ok ? 0.0
                                      : (has_below ? ld_scratch(adjr + (long)Jq * C2 + C + cc)
                                                   : ld_scratch(krow + (long)Jq * C + cc));
                }
            };
            load_feed(NT - 1 - lb, fc);
            load_feed(NT - 1 - lb - CL, fn);
            f_end = NT - 1 - CL;

            const int nsegs = (NT + S - 1) / S;
            real cpn[R + 1 + C];
            // right edge of this lane's last block, and the bottom edge (with its left corner) of the block of the
            // lane above: that lane takes its bottom edge from this lane's ktop at the first step of a segment
            auto load_ckpt = [&](int j) {
                const real* cp = ckpt + ((long)(s * nck + j) * NVC) * kWave + lane;
                const int up1 = lane > 0 ? -1 : 0;
#pragma unroll
                for (int q = 0; q <= R; ++q) cpn[q] = ld_scratch(cp + q * kWave);
                cpn[R + 1] = ld_scratch(cp + (R + 1 + C) * kWave + up1);
#pragma unroll
                for (int q = 1; q < C; ++q) cpn[R + 1 + q] = ld_scratch(cp + (R + 1 + q - 1) * kWave + up1);
            };
            load_ckpt(nsegs);
            for (int g = nsegs - 1; g >= 0; --g) {
                const int T0 = g * S;
                const int T1 = T0 + S < NT ? T0 + S : NT;
                // the recovered right edge must agree with the exact one of the checkpoint, measured against
                // the largest forward value this lane has met in the strip (NaN counts as drift)
#pragma unroll
                for (int i = 0; i <= R; ++i) kscale = fmax(kscale, fabs(cpn[i]));
                if (g < nsegs - 1) {
                    const int Jp = T1 - lane;   // block this lane un-computed last
                    if (Jp >= 1 && Jp < sw.nbl) {
#pragma unroll
                        for (int i = 0; i <= R; ++i)
                            if (!(fabs(sw.left[i] - cpn[i]) <= kDriftTol * kscale)) drift = true;
                    }
                }
#pragma unroll
                for (int i = 0; i <= R; ++i) sw.left[i] = cpn[i];
#pragma unroll
                for (int i = 0; i < C; ++i) ktop[i] = cpn[R + 1 + i];
                load_ckpt(g);   // for the next segment (to the left)

                auto reverse_step = [&](auto fullc, int Tstep, const real (&yv)[DN], real (&yvn)[DN]) {
                    constexpr bool FULL = decltype(fullc)::value;
                    if (Tstep == f_end) {
#pragma unroll
                        for (int cc = 0; cc < C2; ++cc) fc[cc] = fn[cc];
                        load_feed(Tstep - lb - CL, fn);
                        f_end = Tstep - CL;
                    }
                    real recv[C], recvk[C];
#pragma unroll
                    for (int cc = 0; cc < C; ++cc) {
                        recv[cc] = recv_from_below<FULL>(up[cc], fc[cc], is_lb);
                        recvk[cc] = recv_from_below<FULL>(ktop[cc], fc[C + cc], is_lb);
                    }
#pragma unroll
                    for (int cc = 0; cc < C2; ++cc) fc[cc] = wave_shift_up(fc[cc]);
                    const int J = Tstep - lane;
                    sw.fetch_y(J - 1, yvn);
                    const bool active = (unsigned)J < (unsigned)sw.nbl;
                    if (active) {
                        const int b = J >> a.rs2;
                        const real p = sw.p_block(J, yv);
                        real e[R + 1][C + 1];
#pragma unroll
                        for (int rr = 0; rr <= R; ++rr) e[rr][C] = sw.left[rr];
#pragma unroll
                        for (int cc = 0; cc < C; ++cc) e[R][cc] = recvk[cc];
                        real accP = sw.uncompute_adjoint(e, p, recv, accL, corner, up);
                        if (sw.ll_off_block(J)) accP = 0.0;   // the block's p is a constant
#pragma unroll
                        for (int rr = 0; rr <= R; ++rr) sw.left[rr] = e[rr][0];
#pragma unroll
                        for (int cc = 0; cc < C; ++cc) ktop[cc] = e[0][cc];
                        if (lane == 0 && s > 0) {
                            real* wp = adjw + (long)J * C2;
#pragma unroll
                            for (int cc = 0; cc < C; ++cc) { wp[cc] = up[cc]; wp[C + cc] = ktop[cc]; }
                        }
                        sw.accumulate_grads(accP, b, yv, gacc, glds, gdx, gdy);
                    }
                };
                auto run_segment = [&](auto fullc) {
                    real ya[DN], yb[DN];
                    sw.fetch_y(T1 - 1 - lane, ya);
                    int Tstep = T1 - 1;
                    for (; Tstep - 1 >= T0; Tstep -= 2) {
                        reverse_step(fullc, Tstep, ya, yb);
                        reverse_step(fullc, Tstep - 1, yb, ya);
                    }
                    if (Tstep >= T0) reverse_step(fullc, Tstep, ya, yb);
                };
                if (full) run_segment(std::true_type()); else run_segment(std::false_type());
            }
            // the left end: the recovered left edge of the strip against the boundary value 1
#pragma unroll
            for (int i = 0; i <= R; ++i)
                if (!(fabs(sw.left[i] - 1.0) <= kDriftTol * kscale)) drift = true;
            // this kernel's sums are already on their way: every pair of the call is then solved once more
            if (drift) atomicCAS(a.err, 0, 2);   // (an error already raised stays)
            sw.flush_gdx(gacc, gdx);
            scratch_fence();
        }
        if constexpr (YLDS) {
            if (a.want_gy) {
                const int n = a.q * a.DS;
                for (int t = lane; t < n; t += kWave) {
                    const real v = glds[t];
                    if (v != 0.0) unsafeAtomicAdd(&gdy[t], v);
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------------------------
// cooperative kernels: one workgroup per pair, the strips of the pair pipelined over its waves
// ------------------------------------------------------------------------------------------------
// The strips of a pair are processed in rounds of nw consecutive strips, one per wave, separated by
// workgroup barriers.  Inside a round wave w hands the row below its last block row to wave w + 1
// through an outbox ring in LDS; two monotonic flags per wave carry the progress: prod = block columns
// written to the own outbox, cons = block columns read from the upstream outbox.  Wave w only ever
// waits for wave w - 1 (data) and wave w + 1 (ring space), both of which run concurrently and never wait
// for a later round, so the waits cannot form a cycle; every wait is bounded all the same and raises an
// error flag instead of spinning for ever.  The first wave of a round takes its top row from the global
// boundary row that the last wave of the previous round wrote (staged through a small private ring so
// that the step code is the same), or all ones in the very first round.
struct Link {
    SK_LDS int* prod_me;
    SK_LDS int* cons_me;
    const SK_LDS int* prod_up;
    const SK_LDS int* cons_dn;
    bool has_up, has_dn;
    int nb, RB, lane;
    int* err;
    bool* dead;   // set once a wait of this wave has run out: later waits return at once

    __device__ __forceinline__ void setup(int w, bool up, bool dn, SK_LDS int* prod, SK_LDS int* cons, int nb_,
                                          int RB_, int lane_, int* err_, bool* dead_)
    {
        nb = nb_; RB = RB_; lane = lane_; err = err_; dead = dead_;
        has_up = up;
        has_dn = dn;
        prod_me = prod + w;
        cons_me = cons + w;
        prod_up = prod + (w > 0 ? w - 1 : 0);
        cons_dn = cons + w + 1;
    }
    __device__ __forceinline__ void spin_until(const SK_LDS int* f, int need) const
    {
        if (*dead) return;
        for (int it = 0; it < (1 << 22); ++it) {
            const int v = __hip_atomic_load(f, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            lds_order();
            if (v >= need) return;
            __builtin_amdgcn_s_sleep(1);
        }
        *dead = true;
        if (lane == 0) atomicExch(err, 1);   // give up: the results are invalid but the kernel ends
    }
    __device__ __forceinline__ void wait_cols(int count) const
    {
        if (has_up) spin_until(prod_up, count < nb ? count : nb);
    }
    __device__ __forceinline__ void consumed(int count) const
    {
        if (has_up && RB < nb) {
            lds_order();
            __hip_atomic_store(cons_me, count < nb ? count : nb, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
    }
    // before writing outbox columns below `upto`: the ring slots they reuse must have been read
    __device__ __forceinline__ void reserve(int upto) const
    {
        if (!has_dn) return;
        const int need = (upto < nb ? upto : nb) - RB;
        if (need > 0) spin_until(cons_dn, need);
    }
    __device__ __forceinline__ void publish(int count) const
    {
        if (has_dn && count > 0) {
            lds_order();
            __hip_atomic_store(prod_me, count < nb ? count : nb, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
    }
};

template <int BL, bool BWD> struct CoopCfg {
    // waves per workgroup the kernel is compiled for: 8 (two per SIMD) unless the backward kernel's
    // register need at the largest block size asks for a whole SIMD's register file per wave
    static constexpr int kMaxWaves = (BWD && BL == 2) ? 4 : 8;
};

struct CoopLds {
    SK_LDS real* y;
    SK_LDS real* gy;
    SK_LDS int* prod;
    SK_LDS int* cons;
    SK_LDS real* ones;
    SK_LDS real* zeros;
    SK_LDS real* stage;  // this wave's private staging ring (global boundary row -> LDS)
    SK_LDS real* obox;   // this wave's outbox
    SK_LDS real* oboxes;
    SK_LDS real* ring;   // this wave's replay ring
};

__device__ __forceinline__ CoopLds carve_coop_lds(unsigned char* smem, const SweepArgs& a, int w, int Cc)
{
    CoopLds l;
    const int rs = a.RB * Cc;
    l.y = (SK_LDS real*)smem;
    l.gy = (SK_LDS real*)(smem + a.coop_off_gdy);
    l.prod = (SK_LDS int*)(smem + a.coop_off_flags);
    l.cons = l.prod + 32;
    l.ones = (SK_LDS real*)(smem + a.coop_off_obox);
    l.zeros = l.ones + rs;
    l.oboxes = l.zeros + rs;
    l.obox = l.oboxes + w * rs;
    l.stage = l.oboxes + (a.nw + w) * rs;
    l.ring = (SK_LDS real*)(smem + a.coop_off_ring + (size_t)w * a.coop_ring_stride);
    return l;
}

// Staging of a global boundary row into a private LDS ring, CH block columns per chunk, loaded one chunk
// ahead: lets the first wave of a round read its edge values exactly like the other waves do.
// src(J, cc) gives the global address of value cc of ring column J, or nullptr past the end.
template <int C>
struct Stager {
    real pre[C];
    SK_LDS real* ring;
    int rbmask, CH, lane;

    template <class Src>
    __device__ __forceinline__ void load(int col0, Src&& src)
    {
        const int J = col0 + lane;
#pragma unroll
        for (int cc = 0; cc < C; ++cc) {
            const real* g = lane < CH ? src(J, cc) : nullptr;
            pre[cc] = g ? ld_scratch(g) : 0.0;
        }
    }
    __device__ __forceinline__ void store(int col0)
    {
        if (lane < CH) {
            SK_LDS real* rp = ring + ((col0 + lane) & rbmask) * C;
#pragma unroll
            for (int cc = 0; cc < C; ++cc) rp[cc] = pre[cc];
        }
    }
    // columns [0, 2 CH) into the ring, [2 CH, 3 CH) into registers
    template <class Src>
    __device__ __forceinline__ void prime(Src&& src)
    {
        load(0, src);
        store(0);
        load(CH, src);
        store(CH);
        load(2 * CH, src);
    }
    // at the start of the chunk beginning at column Tc > 0
    template <class Src>
    __device__ __forceinline__ void advance(int Tc, Src&& src)
    {
        store(Tc + CH);
        load(Tc + 2 * CH, src);
    }
};

template <int BL, int D, bool YLDS>
__global__ __launch_bounds__((CoopCfg<BL, false>::kMaxWaves) * 64) void sweep_fwd_coop_kernel(SweepArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    using SW = Sweep<BL, D, YLDS>;
    constexpr int C = SW::C;
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave index: uniform, and known to be
    const int nw = a.nw;
    CoopLds l = carve_coop_lds(smem, a, w, C);
    real* rows = a.rows + (long)blockIdx.x * a.rows_slot;
    SW sw(a, lane);
    sw.rbmask = a.RB - 1;
    const int CH = a.CH;
    bool dead = false;

    for (int t = threadIdx.x; t < a.RB * C; t += blockDim.x) { l.ones[t] = 1.0; l.zeros[t] = 0.0; }
    for (long pid = blockIdx.x; pid < a.npairs; pid += gridDim.x) {
        long xi, yi;
        pair_ids(a, pid, xi, yi);
        sw.dxp = a.dx + xi * a.xstride;
        sw.dyg = a.dy + yi * a.ystride;
        sw.dyl = l.y;
        __syncthreads();   // the previous pair is done with y
        if constexpr (YLDS) {
            const int n = a.q * a.DS;
            for (int t = threadIdx.x; t < n; t += blockDim.x) l.y[t] = sw.dyg[t];
        }
        for (int s0 = 0; s0 < a.ns; s0 += nw) {
            if (s0 > 0) scratch_fence();   // boundary row of the previous round
            __syncthreads();
            if (threadIdx.x < 64) l.prod[threadIdx.x] = 0;
            __syncthreads();
            const int s = s0 + w;
            if (s >= a.ns) continue;
            const bool last = s == a.ns - 1;
            // the last wave of a round leaves its bottom row in global memory for the next round
            sw.begin_strip(s, rows, !last && w == nw - 1);
            Link lk;
            lk.setup(w, w > 0, !last && w < nw - 1, l.prod, l.cons, a.nb, a.RB, lane, a.err, &dead);
            sw.obox = l.obox;
            sw.lbo = lk.has_dn ? sw.lb : -1;
            if (sw.lbo >= 0) sw.lbany = sw.lb;
            const bool staged = w == 0 && s > 0;
            sw.ibox = w > 0 ? l.oboxes + (w - 1) * a.RB * C : (staged ? l.stage : l.ones);
            Stager<C> stg;
            stg.ring = l.stage; stg.rbmask = sw.rbmask; stg.CH = CH; stg.lane = lane;
            auto src = [&](int J, int cc) -> const real* {
                return J < a.nb ? sw.rowprev + (long)J * C + 1 + cc : nullptr;
            };
            if (staged) stg.prime(src);
            const int NT = sw.strip_steps();
            real edge[C];
            lk.wait_cols(CH + 1);
            sw.read_edge(0, edge);
            for (int Tc = 0; Tc < NT; Tc += CH) {
                const int Te = Tc + CH < NT ? Tc + CH : NT;
                if (Tc > 0) {
                    if (Tc < a.nb) {
                        lk.consumed(Tc);
                        lk.wait_cols(Tc + CH + 1);
                        if (staged) stg.advance(Tc, src);
                    }
                    lk.publish(Tc - sw.lb);
                }
                lk.reserve(Tc - sw.lb + CH);
                sw.forward_run_coop(Tc, Te, edge, NoHook());
            }
            lk.publish(a.nb);
            lk.consumed(a.nb);
            if (last && lane == sw.lb) a.k_out[pid] = *(volatile int*)a.err ? __builtin_nan("") : sw.bot[C - 1];
        }
    }
}

template <int BL, int D, bool YLDS>
__global__ __launch_bounds__((CoopCfg<BL, true>::kMaxWaves) * 64) void sweep_bwd_coop_kernel(SweepArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    using SW = Sweep<BL, D, YLDS>;
    constexpr int R = SW::R, C = SW::C, NVR = SW::NVR, NVC = SW::NVC, DN = SW::DN;
    constexpr bool LOOKAHEAD = BL < 2;
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave index: uniform, and known to be
    const int nw = a.nw;
    CoopLds l = carve_coop_lds(smem, a, w, C);
    real* rows = a.rows + (long)blockIdx.x * a.rows_slot;
    real* adj = a.adj + (long)blockIdx.x * a.adj_slot;
    real* ckpt = a.ckpt + (long)blockIdx.x * a.ckpt_slot;
    const int S = a.S;
    const int CH = a.CH < S ? a.CH : S;   // checkpoints fall on chunk starts
    SW sw(a, lane);
    sw.rbmask = a.RB - 1;
    bool dead = false;

    for (int t = threadIdx.x; t < a.RB * C; t += blockDim.x) { l.ones[t] = 1.0; l.zeros[t] = 0.0; }
    for (long pid = blockIdx.x; pid < a.npairs; pid += gridDim.x) {
        long xi, yi;
        pair_ids(a, pid, xi, yi);
        sw.dxp = a.dx + xi * a.xstride;
        sw.dyg = a.dy + yi * a.ystride;
        sw.dyl = l.y;
        real* gdx = a.gdx + xi * a.xstride;
        real* gdy = a.gdy + yi * a.ystride;
        __syncthreads();
        if constexpr (YLDS) {
            const int n = a.q * a.DS;
            for (int t = threadIdx.x; t < n; t += blockDim.x) { l.y[t] = sw.dyg[t]; l.gy[t] = 0.0; }
        }
        const real gk = a.grad_k[pid];

        // ---- phase 1: forward in rounds; boundary rows of every strip and checkpoints to global ----
        for (int s0 = 0; s0 < a.ns; s0 += nw) {
            if (s0 > 0) scratch_fence();
            __syncthreads();
            if (threadIdx.x < 64) l.prod[threadIdx.x] = 0;
            __syncthreads();
            const int s = s0 + w;
            if (s >= a.ns) continue;
            const bool last = s == a.ns - 1;
            sw.begin_strip(s, rows, true);
            Link lk;
            lk.setup(w, w > 0, !last && w < nw - 1, l.prod, l.cons, a.nb, a.RB, lane, a.err, &dead);
            sw.obox = l.obox;
            sw.lbo = lk.has_dn ? sw.lb : -1;
            if (sw.lbo >= 0) sw.lbany = sw.lb;
            const bool staged = w == 0 && s > 0;
            sw.ibox = w > 0 ? l.oboxes + (w - 1) * a.RB * C : (staged ? l.stage : l.ones);
            Stager<C> stg;
            stg.ring = l.stage; stg.rbmask = sw.rbmask; stg.CH = CH; stg.lane = lane;
            auto src = [&](int J, int cc) -> const real* {
                return J < a.nb ? sw.rowprev + (long)J * C + 1 + cc : nullptr;
            };
            if (staged) stg.prime(src);
            const int NT = sw.strip_steps();
            real edge[C];
            lk.wait_cols(CH + 1);
            sw.read_edge(0, edge);
            for (int Tc = 0; Tc < NT; Tc += CH) {
                const int Te = Tc + CH < NT ? Tc + CH : NT;
                if (Tc > 0) {
                    if (Tc < a.nb) {
                        lk.consumed(Tc);
                        lk.wait_cols(Tc + CH + 1);
                        if (staged) stg.advance(Tc, src);
                    }
                    lk.publish(Tc - sw.lb);
                }
                lk.reserve(Tc - sw.lb + CH);
                if (Tc % S == 0) {
                    sw.store_ckpt(ckpt + ((long)(s * a.nseg + Tc / S) * NVC) * kWave + lane);
                }
                sw.forward_run_coop(Tc, Te, edge, NoHook());
            }
            lk.publish(a.nb);
            lk.consumed(a.nb);
            if (last && lane == sw.lb && a.k_out) a.k_out[pid] = sw.bot[C - 1];
        }

        // ---- phase 2: strips bottom-up in rounds (processing index i = ns - 1 - s) ----
        for (int i0 = 0; i0 < a.ns; i0 += nw) {
            scratch_fence();   // phase 1 output, or the adjoint boundary row of the previous round
            __syncthreads();
            if (threadIdx.x < 64) l.prod[threadIdx.x] = 0;
            __syncthreads();
            const int i = i0 + w;
            if (i >= a.ns) continue;
            const int s = a.ns - 1 - i;
            sw.begin_strip(s, rows, false);
            Link lk;
            lk.setup(w, w > 0, s > 0 && w < nw - 1, l.prod, l.cons, a.nb, a.RB, lane, a.err, &dead);
            SK_LDS real* obox = l.obox;
            const int NT = sw.strip_steps();
            const int lb = sw.lb;
            const int lane_out = lk.has_dn ? 0 : -1;                   // lane 0 -> outbox of this wave
            const int lane_outg = (s > 0 && w == nw - 1) ? 0 : -1;     // lane 0 -> global row for the next round
            const bool staged = w == 0 && i > 0;
            sw.ibox = w > 0 ? l.oboxes + (w - 1) * a.RB * C : (staged ? l.stage : l.zeros);
            // adjoint boundary rows in global memory, indexed by reverse column (nb - 1 - J)
            const real* adjr = adj + (long)(((i0 / nw) + 1) & 1) * a.rowlen;
            real* adjw = adj + (long)((i0 / nw) & 1) * a.rowlen;
            Stager<C> stg;
            stg.ring = l.stage; stg.rbmask = sw.rbmask; stg.CH = CH; stg.lane = lane;
            auto src = [&](int c, int cc) -> const real* { return c < a.nb ? adjr + (long)c * C + cc : nullptr; };
            if (staged) stg.prime(src);
            real accL[R + 1];
            real up[C];
            real corner = 0.0;
            real gacc[DN];
#pragma unroll
            for (int k = 0; k <= R; ++k) accL[k] = 0.0;
#pragma unroll
            for (int k = 0; k < C; ++k) up[k] = 0.0;
#pragma unroll
            for (int k = 0; k < DN; ++k) gacc[k] = 0.0;

            const int nsegs = (NT + S - 1) / S;
            real cpn[NVC], topn[C];
            auto load_segment = [&](int g) {
                const real* cp = ckpt + ((long)(s * a.nseg + g) * NVC) * kWave + lane;
#pragma unroll
                for (int k = 0; k < NVC; ++k) cpn[k] = ld_scratch(cp + k * kWave);
                sw.load_top(g * S, topn);
            };
            load_segment(nsegs - 1);
            real edge[C];   // adjoint messages for lane 63 at the coming reverse step
            lk.wait_cols(CH + 1);
            sw.read_edge(0, edge);
            for (int g = nsegs - 1; g >= 0; --g) {
                const int T0 = g * S;
                const int T1 = T0 + S < NT ? T0 + S : NT;
#pragma unroll
                for (int k = 0; k <= R; ++k) sw.left[k] = cpn[k];
#pragma unroll
                for (int k = 0; k < C; ++k) { sw.bot[k] = cpn[R + 1 + k]; sw.topc[k] = topn[k]; }
                if (g > 0) load_segment(g - 1);
                sw.forward_run(T0, T1, [&](int Tstep, bool act, real (&e)[R + 1][C + 1]) {
                    if (act) {
                        SK_LDS real* rp = l.ring + ((Tstep - T0) * NVR) * kWave + lane;
#pragma unroll
                        for (int cc = 0; cc <= C; ++cc) rp[cc * kWave] = e[0][cc];
#pragma unroll
                        for (int rr = 1; rr <= R; ++rr) rp[(C + rr) * kWave] = e[rr][0];
                    }
                });
                auto fetch_ring = [&](int Tstep, real (&ein)[NVR]) {
                    const SK_LDS real* rp = l.ring + ((Tstep - T0) * NVR) * kWave + lane;
#pragma unroll
                    for (int v = 0; v < NVR; ++v) ein[v] = rp[v * kWave];
                };
                // reverse time t = NT - 1 - Tstep: lane lb needs reverse column t, lane 0 writes t - lb
                auto reverse_step = [&](int Tstep, const real (&ein)[NVR], const real (&yv)[DN], real (&einn)[NVR],
                                        real (&yvn)[DN]) {
                    const int t = NT - 1 - Tstep;
                    if ((t & (CH - 1)) == 0) {
                        if (t > 0) {
                            if (t < a.nb) {
                                lk.consumed(t);
                                lk.wait_cols(t + CH + 1);
                                if (staged) stg.advance(t, src);
                            }
                            lk.publish(t - lb);
                        }
                        lk.reserve(t - lb + CH);
                    }
                    real recv[C];
#pragma unroll
                    for (int cc = 0; cc < C; ++cc) recv[cc] = wave_from_below_or(up[cc], edge[cc]);
                    sw.read_edge(t + 1, edge);   // for the next reverse step
                    const int J = Tstep - lane;
                    if constexpr (LOOKAHEAD) {
                        if (Tstep > T0) {
                            fetch_ring(Tstep - 1, einn);
                            sw.fetch_y(J - 1, yvn);
                        }
                    }
                    const bool active = (unsigned)J < (unsigned)sw.nbl;
                    if (active) {
                        const int b = J >> a.rs2;
                        const real p = sw.p_block(J, yv);
                        const bool seed = s == a.ns - 1 && lane == lb && J == a.nb - 1;
                        real accP = sw.reverse_block(ein, p, recv, seed, gk, accL, corner, up);
                        if (sw.ll_off_block(J)) accP = 0.0;   // the block's p is a constant
                        if (lane == lane_out) {
                            SK_LDS real* op = obox + ((a.nb - 1 - J) & sw.rbmask) * C;
#pragma unroll
                            for (int cc = 0; cc < C; ++cc) op[cc] = up[cc];
                        }
                        if (lane == lane_outg) {
                            real* wp = adjw + (long)(a.nb - 1 - J) * C;
#pragma unroll
                            for (int cc = 0; cc < C; ++cc) wp[cc] = up[cc];
                        }
                        sw.accumulate_grads(accP, b, yv, gacc, l.gy, gdx, gdy);
                    }
                };
                if constexpr (LOOKAHEAD) {
                    real ea[NVR], eb[NVR], ya[DN], yb[DN];
                    fetch_ring(T1 - 1, ea);
                    sw.fetch_y(T1 - 1 - lane, ya);
                    int Tstep = T1 - 1;
                    for (; Tstep - 1 >= T0; Tstep -= 2) {
                        reverse_step(Tstep, ea, ya, eb, yb);
                        reverse_step(Tstep - 1, eb, yb, ea, ya);
                    }
                    if (Tstep >= T0) reverse_step(Tstep, ea, ya, eb, yb);
                } else {
                    for (int Tstep = T1 - 1; Tstep >= T0; --Tstep) {
                        real ea[NVR], ya[DN];
                        fetch_ring(Tstep, ea);
                        sw.fetch_y(Tstep - lane, ya);
                        reverse_step(Tstep, ea, ya, ea, ya);
                    }
                }
            }
            lk.publish(a.nb);
            lk.consumed(a.nb);
            if (*(volatile int*)a.err) {
#pragma unroll
                for (int k = 0; k < DN; ++k) gacc[k] = __builtin_nan("");
            }
            sw.flush_gdx(gacc, gdx);
        }
        __syncthreads();
        if constexpr (YLDS) {
            if (a.want_gy) {
                const int n = a.q * a.DS;
                for (int t = threadIdx.x; t < n; t += blockDim.x) {
                    const real v = l.gy[t];
                    if (v != 0.0) unsafeAtomicAdd(&gdy[t], v);
                }
            }
        }
    }
}

// Cooperative backward kernel, un-compute variant (see sweep_bwdu_kernel for the method and
// sweep_bwd_coop_kernel for the hand-over between waves).  The messages that travel upwards from strip to
// strip are 2C wide: the adjoint messages and the recovered top edge of the lower strip.
template <int BL, int D, bool YLDS>
__global__ __launch_bounds__((CoopCfg<BL, true>::kMaxWaves) * 64) void sweep_bwdu_coop_kernel(SweepArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    using SW = Sweep<BL, D, YLDS>;
    constexpr int R = SW::R, C = SW::C, NVC = SW::NVC, DN = SW::DN;
    constexpr int C2 = 2 * C;
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave index: uniform, and known to be
    const int nw = a.nw;
    CoopLds l = carve_coop_lds(smem, a, w, C2);
    real* rows = a.rows + (long)blockIdx.x * a.rows_slot;
    real* adj = a.adj + (long)blockIdx.x * a.adj_slot;
    real* ckpt = a.ckpt + (long)blockIdx.x * a.ckpt_slot;
    const int S = a.S;
    const int CH = a.CH < S ? a.CH : S;   // checkpoints fall on chunk starts
    const int nck = a.nseg + 1;
    const long adjlen = 2L * a.rowlen;
    const int rbmask = a.RB - 1;
    SW sw(a, lane);
    sw.rbmask = rbmask;
    bool dead = false;

    for (int t = threadIdx.x; t < a.RB * C2; t += blockDim.x) { l.ones[t] = 1.0; l.zeros[t] = 0.0; }
    for (long pid = blockIdx.x; pid < a.npairs; pid += gridDim.x) {
        long xi, yi;
        pair_ids(a, pid, xi, yi);
        sw.dxp = a.dx + xi * a.xstride;
        sw.dyg = a.dy + yi * a.ystride;
        sw.dyl = l.y;
        real* gdx = a.gdx + xi * a.xstride;
        real* gdy = a.gdy + yi * a.ystride;
        __syncthreads();
        if constexpr (YLDS) {
            const int n = a.q * a.DS;
            for (int t = threadIdx.x; t < n; t += blockDim.x) { l.y[t] = sw.dyg[t]; l.gy[t] = 0.0; }
        }
        const real gk = a.grad_k[pid];

        // ---- phase 1: forward in rounds; boundary rows and checkpoints to global ----
        for (int s0 = 0; s0 < a.ns; s0 += nw) {
            if (s0 > 0) scratch_fence();
            __syncthreads();
            if (threadIdx.x < 64) l.prod[threadIdx.x] = 0;
            __syncthreads();
            const int s = s0 + w;
            if (s >= a.ns) continue;
            const bool last = s == a.ns - 1;
            // global boundary rows are needed below the last wave of a round (next round's top feed) and
            // below the last strip (bottom row of the grid, where the reverse sweep starts)
            sw.begin_strip(s, rows, last || w == nw - 1);
            if (last && lane == sw.lb) sw.rowcur[0] = 1.0;
            Link lk;
            lk.setup(w, w > 0, !last && w < nw - 1, l.prod, l.cons, a.nb, a.RB, lane, a.err, &dead);
            sw.obox = l.obox;
            sw.lbo = lk.has_dn ? sw.lb : -1;
            if (sw.lbo >= 0) sw.lbany = sw.lb;
            const bool staged = w == 0 && s > 0;
            sw.ibox = w > 0 ? l.oboxes + (w - 1) * a.RB * C2 : (staged ? l.stage : l.ones);
            Stager<C> stg;
            stg.ring = l.stage; stg.rbmask = rbmask; stg.CH = CH; stg.lane = lane;
            auto src = [&](int J, int cc) -> const real* {
                return J < a.nb ? sw.rowprev + (long)J * C + 1 + cc : nullptr;
            };
            if (staged) stg.prime(src);
            const int NT = sw.strip_steps();
            real edge[C];
            lk.wait_cols(CH + 1);
            sw.read_edge(0, edge);
            for (int Tc = 0; Tc < NT; Tc += CH) {
                const int Te = Tc + CH < NT ? Tc + CH : NT;
                if (Tc > 0) {
                    if (Tc < a.nb) {
                        lk.consumed(Tc);
                        lk.wait_cols(Tc + CH + 1);
                        if (staged) stg.advance(Tc, src);
                    }
                    lk.publish(Tc - sw.lb);
                }
                lk.reserve(Tc - sw.lb + CH);
                if (Tc % S == 0) sw.store_ckpt(ckpt + ((long)(s * nck + Tc / S) * NVC) * kWave + lane);
                sw.forward_run_coop(Tc, Te, edge, NoHook());
            }
            sw.store_ckpt(ckpt + ((long)(s * nck + (NT + S - 1) / S) * NVC) * kWave + lane);
            lk.publish(a.nb);
            lk.consumed(a.nb);
            if (last && lane == sw.lb && a.k_out) a.k_out[pid] = sw.bot[C - 1];
        }

        // ---- phase 2: strips bottom-up in rounds (processing index i = ns - 1 - s) ----
        bool drift = false;
        for (int i0 = 0; i0 < a.ns; i0 += nw) {
            scratch_fence();   // phase 1 output, or the boundary row of the previous round
            __syncthreads();
            if (threadIdx.x < 64) l.prod[threadIdx.x] = 0;
            __syncthreads();
            const int i = i0 + w;
            if (i >= a.ns) continue;
            const int s = a.ns - 1 - i;
            real kscale = 1.0;
            sw.begin_strip(s, rows, false);
            Link lk;
            lk.setup(w, w > 0, s > 0 && w < nw - 1, l.prod, l.cons, a.nb, a.RB, lane, a.err, &dead);
            SK_LDS real* obox = l.obox;
            const int NT = sw.strip_steps();
            const int lb = sw.lb;
            const bool full = lb == kWave - 1;
            const bool is_lb = lane == lb;
            const int lane_out = lk.has_dn ? 0 : -1;                   // lane 0 -> outbox of this wave
            const int lane_outg = (s > 0 && w == nw - 1) ? 0 : -1;     // lane 0 -> global row for the next round
            const bool staged = w == 0;   // the first wave of a round reads its feed from global memory
            const SK_LDS real* ibox = w > 0 ? l.oboxes + (w - 1) * a.RB * C2 : l.stage;
            // boundary rows in global memory, indexed by reverse column c = nb - 1 - J, 2C values each
            const real* adjr = adj + (long)(((i0 / nw) + 1) & 1) * adjlen;
            real* adjw = adj + (long)((i0 / nw) & 1) * adjlen;
            const real* krow = rows + (long)(a.ns - 1) * a.rowlen;   // bottom row of the grid
            Stager<C2> stg;
            stg.ring = l.stage; stg.rbmask = rbmask; stg.CH = CH; stg.lane = lane;
            auto src = [&](int c, int cc) -> const real* {
                if (c >= a.nb) return nullptr;
                if (i > 0) return adjr + (long)c * C2 + cc;
                return cc < C ? nullptr : krow + (long)(a.nb - 1 - c) * C + (cc - C);
            };
            if (staged) stg.prime(src);
            auto read_feed = [&](int col, real (&dst)[C2]) {
                const int cidx = col < a.nb ? col : a.nb - 1;
                const SK_LDS real* ip = ibox + (cidx & rbmask) * C2;
#pragma unroll
                for (int cc = 0; cc < C2; ++cc) dst[cc] = ip[cc];
            };
            real accL[R + 1], up[C], ktop[C];
            real corner = 0.0;
            real gacc[DN];
#pragma unroll
            for (int k = 0; k <= R; ++k) accL[k] = 0.0;
            // dF/dk at the far corner enters as the carried adjoint of the last lane's first block
            if (s == a.ns - 1 && is_lb) accL[R] = gk;
#pragma unroll
            for (int k = 0; k < C; ++k) { up[k] = 0.0; ktop[k] = 0.0; }
#pragma unroll
            for (int k = 0; k < DN; ++k) gacc[k] = 0.0;

            const int nsegs = (NT + S - 1) / S;
            real cpn[R + 1 + C];
            // right edge of this lane's last block, and the bottom edge (with its left corner) of the block of the
            // lane above: that lane takes its bottom edge from this lane's ktop at the first step of a segment
            auto load_ckpt = [&](int j) {
                const real* cp = ckpt + ((long)(s * nck + j) * NVC) * kWave + lane;
                const int up1 = lane > 0 ? -1 : 0;
#pragma unroll
                for (int q = 0; q <= R; ++q) cpn[q] = ld_scratch(cp + q * kWave);
                cpn[R + 1] = ld_scratch(cp + (R + 1 + C) * kWave + up1);
#pragma unroll
                for (int q = 1; q < C; ++q) cpn[R + 1 + q] = ld_scratch(cp + (R + 1 + q - 1) * kWave + up1);
            };
            load_ckpt(nsegs);
            real feed[C2];   // messages for the strip's last lane at the coming reverse step
            lk.wait_cols(CH + 1);
            read_feed(0, feed);
            for (int g = nsegs - 1; g >= 0; --g) {
                const int T0 = g * S;
                const int T1 = T0 + S < NT ? T0 + S : NT;
#pragma unroll
                for (int k = 0; k <= R; ++k) kscale = fmax(kscale, fabs(cpn[k]));
                if (g < nsegs - 1) {
                    const int Jp = T1 - lane;
                    if (Jp >= 1 && Jp < sw.nbl) {
#pragma unroll
                        for (int k = 0; k <= R; ++k)
                            if (!(fabs(sw.left[k] - cpn[k]) <= kDriftTol * kscale)) drift = true;
                    }
                }
#pragma unroll
                for (int k = 0; k <= R; ++k) sw.left[k] = cpn[k];
#pragma unroll
                for (int k = 0; k < C; ++k) ktop[k] = cpn[R + 1 + k];
                load_ckpt(g);
                // reverse time t = NT - 1 - Tstep: lane lb needs reverse column t, lane 0 writes t - lb
                auto reverse_step = [&](auto fullc, int Tstep, const real (&yv)[DN], real (&yvn)[DN]) {
                    constexpr bool FULL = decltype(fullc)::value;
                    const int t = NT - 1 - Tstep;
                    if ((t & (CH - 1)) == 0) {
                        if (t > 0) {
                            if (t < a.nb) {
                                lk.consumed(t);
                                lk.wait_cols(t + CH + 1);
                                if (staged) stg.advance(t, src);
                            }
                            lk.publish(t - lb);
                        }
                        lk.reserve(t - lb + CH);
                    }
                    real recv[C], recvk[C];
#pragma unroll
                    for (int cc = 0; cc < C; ++cc) {
                        recv[cc] = recv_from_below<FULL>(up[cc], feed[cc], is_lb);
                        recvk[cc] = recv_from_below<FULL>(ktop[cc], feed[C + cc], is_lb);
                    }
                    read_feed(t + 1, feed);   // for the next reverse step
                    const int J = Tstep - lane;
                    sw.fetch_y(J - 1, yvn);
                    const bool active = (unsigned)J < (unsigned)sw.nbl;
                    if (active) {
                        const int b = J >> a.rs2;
                        const real p = sw.p_block(J, yv);
                        real e[R + 1][C + 1];
#pragma unroll
                        for (int rr = 0; rr <= R; ++rr) e[rr][C] = sw.left[rr];
#pragma unroll
                        for (int cc = 0; cc < C; ++cc) e[R][cc] = recvk[cc];
                        real accP = sw.uncompute_adjoint(e, p, recv, accL, corner, up);
                        if (sw.ll_off_block(J)) accP = 0.0;   // the block's p is a constant
#pragma unroll
                        for (int rr = 0; rr <= R; ++rr) sw.left[rr] = e[rr][0];
#pragma unroll
                        for (int cc = 0; cc < C; ++cc) ktop[cc] = e[0][cc];
                        if (lane == 0 && (lane_out == 0 || lane_outg == 0)) {
                            const int c = a.nb - 1 - J;
                            if (lane_out == 0) {
                                SK_LDS real* op = obox + (c & rbmask) * C2;
#pragma unroll
                                for (int cc = 0; cc < C; ++cc) { op[cc] = up[cc]; op[C + cc] = ktop[cc]; }
                            }
                            if (lane_outg == 0) {
                                real* wp = adjw + (long)c * C2;
#pragma unroll
                                for (int cc = 0; cc < C; ++cc) { wp[cc] = up[cc]; wp[C + cc] = ktop[cc]; }
                            }
                        }
                        sw.accumulate_grads(accP, b, yv, gacc, l.gy, gdx, gdy);
                    }
                };
                auto run_segment = [&](auto fullc) {
                    real ya[DN], yb[DN];
                    sw.fetch_y(T1 - 1 - lane, ya);
                    int Tstep = T1 - 1;
                    for (; Tstep - 1 >= T0; Tstep -= 2) {
                        reverse_step(fullc, Tstep, ya, yb);
                        reverse_step(fullc, Tstep - 1, yb, ya);
                    }
                    if (Tstep >= T0) reverse_step(fullc, Tstep, ya, yb);
                };
                if (full) run_segment(std::true_type()); else run_segment(std::false_type());
            }
            lk.publish(a.nb);
            lk.consumed(a.nb);
            // the left end: the recovered left edge of the strip against the boundary value 1
#pragma unroll
            for (int k = 0; k <= R; ++k)
                if (!(fabs(sw.left[k] - 1.0) <= kDriftTol * kscale)) drift = true;
            // this kernel's sums are already on their way: every pair of the call is then solved once more
            if (drift) atomicCAS(a.err, 0, 2);   // (an error already raised stays)
            sw.flush_gdx(gacc, gdx);
        }
        __syncthreads();
        if constexpr (YLDS) {
            if (a.want_gy) {
                const int n = a.q * a.DS;
                for (int t = threadIdx.x; t < n; t += blockDim.x) {
                    const real v = l.gy[t];
                    if (v != 0.0) unsafeAtomicAdd(&gdy[t], v);
                }
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

hipError_t launch_keep_tag(unsigned long long* tag, unsigned long long val, int check, int* err, hipStream_t st)
{
    hipLaunchKernelGGL(keep_tag_kernel, dim3(1), dim3(1), 0, st, tag, val, check, err);
    return hipGetLastError();
}

hipError_t launch_second_chance_reset(real* g1, long n1, real* g2, long n2, const int* err, hipStream_t st)
{
    if (!g1) n1 = 0;
    if (!g2) n2 = 0;
    if (n1 + n2 == 0) return hipSuccess;
    long blocks = (n1 + n2 + 255) / 256;
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(second_chance_reset_kernel, dim3((unsigned)blocks), dim3(256), 0, st, g1, n1, g2, n2, err);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_mmd2_reduce(const T* Kxx, const T* Kxy, const T* Kyy, long nxx, long nxy, long nyy, T* out,
                              hipStream_t st)
{
    hipLaunchKernelGGL(mmd2_reduce_kernel<T>, dim3(1), dim3(1024), 0, st, Kxx, Kxy, Kyy, nxx, nxy, nyy, out);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_add_inplace(T* dst, const T* src, long n, hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    long blocks = (n + 255) / 256;
    if (blocks > 4096) blocks = 4096;
    hipLaunchKernelGGL(add_inplace_kernel<T>, dim3((unsigned)blocks), dim3(256), 0, st, dst, src, n);
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
hipError_t launch_prepare(const T* x, real* dx, real* gdx, long nx, int L1, int rpad, const T* y, real* dy, real* gdy,
                          long ny, int L2, int qpad, int d, int DS, int* err, int nclear, hipStream_t st)
{
    PathSet<T> px{x, nullptr, dx, gdx, nx, L1, rpad};
    PathSet<T> py{y, nullptr, dy, gdy, ny, L2, qpad};
    long total = (dx ? nx * (long)rpad * DS : 0) + (dy ? ny * (long)qpad * DS : 0);
    if (total <= 0) total = 1;
    long blocks = (total + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(prepare_kernel<T>, dim3((unsigned)blocks), dim3(256), 0, st, px, py, d, DS, err, nclear);
    return hipGetLastError();
}

template <typename T>
hipError_t launch_finalize(const real* gdx, T* grad_x, long nx, int L1, int rpad, const real* gdy, T* grad_y, long ny,
                           int L2, int qpad, int d, int DS, const int* err, hipStream_t st)
{
    PathSet<T> px{nullptr, grad_x, nullptr, const_cast<real*>(gdx), nx, L1, rpad};
    PathSet<T> py{nullptr, grad_y, nullptr, const_cast<real*>(gdy), ny, L2, qpad};
    long total = (grad_x ? nx * (long)L1 * d : 0) + (grad_y ? ny * (long)L2 * d : 0);
    if (total <= 0) return hipSuccess;
    long blocks = (total + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    hipLaunchKernelGGL(finalize_kernel<T>, dim3((unsigned)blocks), dim3(256), 0, st, px, py, d, DS, err);
    return hipGetLastError();
}

template <int BL, int D, bool YLDS>
hipError_t launch_sweep_coop(bool backward, const SweepArgs& a, int grid, size_t lds, hipStream_t st)
{
    hipError_t e;
    const int maxw = backward ? CoopCfg<BL, true>::kMaxWaves : CoopCfg<BL, false>::kMaxWaves;
    if (a.nw < 1 || a.nw > maxw) return hipErrorInvalidValue;
    if (backward) {
        e = allow_full_lds(reinterpret_cast<const void*>(&sweep_bwd_coop_kernel<BL, D, YLDS>));
        if (e != hipSuccess) return e;
        if (a.uncompute) {
            e = allow_full_lds(reinterpret_cast<const void*>(&sweep_bwdu_coop_kernel<BL, D, YLDS>));
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL((sweep_bwdu_coop_kernel<BL, D, YLDS>), dim3(grid), dim3(a.nw * kWave), lds, st, a);
        } else {
            hipLaunchKernelGGL((sweep_bwd_coop_kernel<BL, D, YLDS>), dim3(grid), dim3(a.nw * kWave), lds, st, a);
        }
    } else {
        e = allow_full_lds(reinterpret_cast<const void*>(&sweep_fwd_coop_kernel<BL, D, YLDS>));
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((sweep_fwd_coop_kernel<BL, D, YLDS>), dim3(grid), dim3(a.nw * kWave), lds, st, a);
    }
    return hipGetLastError();
}

template <int BL, int D, bool YLDS>
hipError_t launch_sweep_one(bool backward, const SweepArgs& a, int grid, size_t lds, hipStream_t st)
{
    hipError_t e;
    if (a.coop) return launch_sweep_coop<BL, D, YLDS>(backward, a, grid, lds, st);
    if (backward) {
        e = allow_full_lds(reinterpret_cast<const void*>(&sweep_bwd_kernel<BL, D, YLDS>));
        if (e != hipSuccess) return e;
        if (a.uncompute) {
            e = allow_full_lds(reinterpret_cast<const void*>(&sweep_bwdu_kernel<BL, D, YLDS>));
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL((sweep_bwdu_kernel<BL, D, YLDS>), dim3(grid), dim3(kWavesPerWG * kWave), lds, st, a);
        } else {
            hipLaunchKernelGGL((sweep_bwd_kernel<BL, D, YLDS>), dim3(grid), dim3(kWavesPerWG * kWave), lds, st, a);
        }
    } else {
        e = allow_full_lds(reinterpret_cast<const void*>(&sweep_fwd_kernel<BL, D, YLDS>));
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((sweep_fwd_kernel<BL, D, YLDS>), dim3(grid), dim3(kWavesPerWG * kWave), lds, st, a);
    }
    return hipGetLastError();
}

template <int BL, int D>
hipError_t launch_sweep_y(bool backward, bool ylds, const SweepArgs& a, int grid, size_t lds, hipStream_t st)
{
    if constexpr (D > 0) {
        if (ylds) return launch_sweep_one<BL, D, true>(backward, a, grid, lds, st);
    }
    return launch_sweep_one<BL, D, false>(backward, a, grid, lds, st);
}

template <int BL>
hipError_t launch_sweep_bl(bool backward, int DT, bool ylds, const SweepArgs& a, int grid, size_t lds,
                           hipStream_t st)
{
    switch (DT) {
#ifndef SK_ONLY_C2   /* development builds instantiate a single shape */
        case 0: return launch_sweep_y<BL, 0>(backward, ylds, a, grid, lds, st);
        case 2: return launch_sweep_y<BL, 2>(backward, ylds, a, grid, lds, st);
        case 3: return launch_sweep_y<BL, 3>(backward, ylds, a, grid, lds, st);
        case 4: return launch_sweep_y<BL, 4>(backward, ylds, a, grid, lds, st);
        case 6: return launch_sweep_y<BL, 6>(backward, ylds, a, grid, lds, st);
        case 8: return launch_sweep_y<BL, 8>(backward, ylds, a, grid, lds, st);
        case 16: return launch_sweep_y<BL, 16>(backward, ylds, a, grid, lds, st);
#endif
        case 5: return launch_sweep_y<BL, 5>(backward, ylds, a, grid, lds, st);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_sweep(bool backward, int BL, int DT, const SweepArgs& a, int grid, size_t lds, hipStream_t st)
{
    const bool ylds = a.y_lds != 0;
    // the lead-lag form of the sweep: the level lies inside the blocks (which then hold every refined cell of a pair of
    // increments) or above them
    if (a.ll == 1 && (BL < 1 || a.rs1 != 0 || a.rs2 != 0)) return hipErrorInvalidValue;
    if (a.ll == 2 && (a.rs1 < 1 || a.rs2 < 1)) return hipErrorInvalidValue;
    if (a.ll < 0 || a.ll > 2) return hipErrorInvalidValue;
    switch (BL) {
#ifndef SK_ONLY_C2
        case 0: return launch_sweep_bl<0>(backward, DT, ylds, a, grid, lds, st);
        case 2: return launch_sweep_bl<2>(backward, DT, ylds, a, grid, lds, st);
#endif
        case 1: return launch_sweep_bl<1>(backward, DT, ylds, a, grid, lds, st);
        default: return hipErrorInvalidValue;
    }
}

template hipError_t launch_mmd2_reduce<float>(const float*, const float*, const float*, long, long, long, float*, hipStream_t);
template hipError_t launch_mmd2_reduce<double>(const double*, const double*, const double*, long, long, long, double*,
                                               hipStream_t);
template hipError_t launch_add_inplace<float>(float*, const float*, long, hipStream_t);
template hipError_t launch_add_inplace<double>(double*, const double*, long, hipStream_t);
template hipError_t launch_fill<int>(int*, long, int, hipStream_t);
template hipError_t launch_fill<float>(float*, long, float, hipStream_t);
template hipError_t launch_fill<double>(double*, long, double, hipStream_t);
template hipError_t launch_convert<float, double>(const float*, double*, long, hipStream_t);
template hipError_t launch_convert<double, float>(const double*, float*, long, hipStream_t);
template hipError_t launch_prepare<float>(const float*, real*, real*, long, int, int, const float*, real*, real*, long,
                                          int, int, int, int, int*, int, hipStream_t);
template hipError_t launch_prepare<double>(const double*, real*, real*, long, int, int, const double*, real*, real*,
                                           long, int, int, int, int, int*, int, hipStream_t);
template hipError_t launch_finalize<float>(const real*, float*, long, int, int, const real*, float*, long, int, int, int,
                                           int, const int*, hipStream_t);
template hipError_t launch_finalize<double>(const real*, double*, long, int, int, const real*, double*, long, int, int,
                                            int, int, const int*, hipStream_t);

}  // namespace sk

// Quad sweep (gfx950), forward: four path pairs per wavefront, for forward calls on Gram matrices of many short paths
// (at most 64 or 128 block rows per pair; no residual refinement: the blocks hold all of it).
//
// A wavefront that gives one lane to every block row of one pair walks 64 lanes over the pair's columns: the skew of
// the anti-diagonal sweep (Section 3.3) leaves 63 of its macro-steps per lane outside the grid, half of them all for
// 63 columns.  Here a pair has 16 lanes, each with M = 4 or 8 consecutive block rows, and the wavefront's four groups
// of 16 lanes work on four pairs at once, in lock-step, so that a sweep takes nb + 15 macro-steps of M blocks per lane
// instead of nb + 63 of one or two:
//
//  * the four pairs of a wavefront share the y path (pairs are taken in y-major order, four x paths at a time):
//    its increments sit in the wavefront's LDS once, and the four groups read the same addresses (broadcast);
//  * p = <dx[a], dy[b]> (Eq. (1), third line) is formed in registers: the lane keeps the increments of its rows
//    (M x D doubles) and reads the D increments of its column once per macro-step (for an even D 16 bytes at a time,
//    with a row stride of the y copy that keeps those reads free of bank conflicts);
//  * the bottom edge of a lane goes to the lane below by a DPP shift inside its row of 16 lanes; the first lane of
//    a group holds the top of the grid (boundary value 1);
//  * nothing is masked: a lane whose column lies outside the grid reads a row of zeros behind the y copy and works
//    with p = 0, i.e. A = B = 1, and the macro-steps whose 16 columns all lie inside the grid run without clamping.
//
// The rows of a pair are aligned to the bottom of its 16 M lane-rows (rows above the grid have zero increments), so the
// result leaves through the last lane of the group.  The registers of a wavefront leave room for two per SIMD.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "sk_dev.h"
#include "sk_kernels.h"
#include "sk_lane.h"

namespace sk {

// lane i of a row of 16 lanes receives v of lane i - 1; the row's first lane receives edge (its own lane's value)
__device__ __forceinline__ real row_from_above_or(real v, real edge)
{
    int lo = __double2loint(v), hi = __double2hiint(v);
    int elo = __double2loint(edge), ehi = __double2hiint(edge);
    lo = __builtin_amdgcn_update_dpp(elo, lo, 0x111, 0xf, 0xf, false);
    hi = __builtin_amdgcn_update_dpp(ehi, hi, 0x111, 0xf, 0xf, false);
    return __hiloint2double(hi, lo);
}

// Quad q of the sequence a launch works through: row yi of the Gram matrix in groups of four x paths, rows in
// ascending order.  A row has N pairs, or, for a symmetric Gram matrix K(X, X), the yi + 1 pairs n <= yi.
struct QuadCursor {
    long yi, xi0, npr;
    __device__ __forceinline__ void locate(const SweepArgs& a, long u)
    {
        if (!a.tri) {
            const long per_row = (a.gramN + kQuadPairs - 1) / kQuadPairs;
            yi = u / per_row;
            xi0 = (u - yi * per_row) * kQuadPairs;
            npr = a.gramN;
        } else {
            // rows 4 j .. 4 j + 3 hold j + 1 quads each: 2 j (j + 1) quads lie before row 4 j
            long j = (long)((sqrt(2.0 * (double)u + 1.0) - 1.0) * 0.5);
            while (2 * (j + 1) * (j + 2) <= u) ++j;
            while (2 * j * (j + 1) > u) --j;
            const long rest = u - 2 * j * (j + 1);
            yi = 4 * j + rest / (j + 1);
            xi0 = (rest % (j + 1)) * kQuadPairs;
            npr = yi + 1;
        }
    }
    __device__ __forceinline__ void next(const SweepArgs& a)
    {
        xi0 += kQuadPairs;
        if (xi0 >= npr) {
            xi0 = 0;
            ++yi;
            if (a.tri) npr = yi + 1;
        }
    }
};

template <int BL, int D, int M>
__global__ __launch_bounds__(kWavesPerWG* kWave, 2) void quad_fwd_kernel(SweepArgs a)
{
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int LP = kWave / kQuadPairs, YS = quad_y_stride(D);
    using LK = Lock<BL, D, M>;
    constexpr int C = LK::C;
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int g = lane >> 4, r = lane & (LP - 1);
    const long slot = (long)blockIdx.x * kWavesPerWG + w;
    const long nslots = (long)gridDim.x * kWavesPerWG;
    SK_LDS real* ylds = (SK_LDS real*)(smem + (size_t)w * a.lds_wave);
    const long u0 = slot * a.qd_nquads / nslots, u1 = (slot + 1) * a.qd_nquads / nslots;
    const int nb = a.nb;
    const int NT = nb + LP - 1;
    long cur_y = -1;
    if (u0 >= u1) return;

    QuadCursor cur;
    cur.locate(a, u0);
    typename LK::Fwd f;
    for (long u = u0; u < u1; ++u, cur.next(a)) {
        const long yi = cur.yi;
        if (yi != cur_y) {
            // the y increments, row stride YS: a lane's 16-byte reads of its column meet no other lane's banks
            const real* dyg = a.dy + yi * a.ystride;
            for (int t = lane; t < (a.q + 1) * D; t += kWave) {   // and a row of zeros behind the last one
                const int b = t / D, c = t - b * D;
                ylds[b * YS + c] = b < a.q ? dyg[(long)b * a.DS + c] : 0.0;
            }
            cur_y = yi;
        }
        const bool valid = cur.xi0 + g < cur.npr;
        const long xi = valid ? cur.xi0 + g : cur.npr - 1;   // a group beyond the row's end repeats its last pair
        // increments of the lane's rows (zero above the grid) and the time channel's constant product
        real dxr[M][D];
        const int nabove = a.lk_padb - r * M;   // the lane's rows m < nabove lie above the grid
        {
            const real* dxp = a.dx + xi * a.xstride;
            // (every load is issued before the first value is used, from a row inside the array: a load under a
            // condition would be waited for on the spot)
#pragma unroll
            for (int m = 0; m < M; ++m) {
                const int I = r * M + m - a.lk_padb;
                const real* xp = dxp + (long)(I >= 0 ? I : 0) * a.DS;
#pragma unroll
                for (int c = 0; c < D; ++c) dxr[m][c] = xp[c];
            }
#pragma unroll
            for (int m = 0; m < M; ++m) {
                const int I = r * M + m - a.lk_padb;
                const real s = I >= 0 ? a.sc : 0.0;
#pragma unroll
                for (int c = 0; c < D; ++c) dxr[m][c] *= s;
            }
        }
        f.init();

        // Channels [c0, c1) of the increments of the column the lane is at in macro-step T.
        auto fetch = [&](auto edge_c, int T, int& J, real (&y)[D], auto c0_c, auto c1_c) __attribute__((always_inline)) {
            constexpr bool EDGE = decltype(edge_c)::value;
            constexpr int c0 = decltype(c0_c)::value, c1 = decltype(c1_c)::value;
            J = T - r;
            const int b = EDGE ? (int)min((unsigned)J, (unsigned)nb) : J;   // outside the grid: the row of zeros
            if constexpr (D % 2 == 0) {
                static_assert(c0 % 2 == 0 && c1 % 2 == 0, "16 bytes at a time");
                const SK_LDS real2* yp = (const SK_LDS real2*)(ylds + __mul24(b, YS));
#pragma unroll
                for (int c = c0 / 2; c < c1 / 2; ++c) {
                    const real2 v = yp[c];
                    y[2 * c] = v.x;
                    y[2 * c + 1] = v.y;
                }
            } else {
                const SK_LDS real* yp = ylds + __mul24(b, YS);
#pragma unroll
                for (int c = c0; c < c1; ++c) y[c] = yp[c];
            }
        };
        using c_0 = std::integral_constant<int, 0>;
        using c_d = std::integral_constant<int, D>;
        // p of the lane's M blocks in column J (Eq. (1), third line), from the column's increments y
        auto inner = [&](auto edge_c, auto tc_c, int J, const real (&y)[D], real (&p)[M]) __attribute__((always_inline)) {
            constexpr bool EDGE = decltype(edge_c)::value;
#pragma unroll
            for (int m = 0; m < M; ++m) {
                real t = dxr[m][0] * y[0];
#pragma unroll
                for (int c = 1; c < D; ++c) t = fma(dxr[m][c], y[c], t);
                // (outside the grid the column's increments read as zeros, so only the time constant is left to mask)
                if constexpr (decltype(tc_c)::value) t += (m >= nabove && (!EDGE || (unsigned)J < (unsigned)nb)) ? a.tc : 0.0;
                p[m] = t;
            }
        };
        // Eq. (1) on the lane's M blocks, top to bottom (LK::Fwd::step with the coefficients of a block formed when its
        // turn comes: fewer values alive at once)
        auto cells = [&](const real (&p)[M]) __attribute__((always_inline)) {
            constexpr int R = 1 << BL;
            real top[C + 1];
            top[0] = f.left[0];
#pragma unroll
            for (int cc = 0; cc < C; ++cc) top[cc + 1] = row_from_above_or(f.bot[cc], 1.0);
            const real tr = top[C];
#pragma unroll
            for (int m = 0; m < M; ++m) {
                real Ac, Bc;
                LK::coef_fwd(p[m], Ac, Bc);
#pragma unroll
                for (int rb = 0; rb < R; ++rb) {
                    const int rr = m * R + rb;
                    real cur[C + 1];
                    cur[0] = f.left[rr + 1];
#pragma unroll
                    for (int cc = 0; cc < C; ++cc) cur[cc + 1] = fma(cur[cc] + top[cc + 1], Ac, -(top[cc] * Bc));
                    f.left[rr + 1] = cur[C];
#pragma unroll
                    for (int cc = 0; cc <= C; ++cc) top[cc] = cur[cc];
                }
            }
            f.blc = top[0];
#pragma unroll
            for (int cc = 0; cc < C; ++cc) f.bot[cc] = top[cc + 1];
            f.left[0] = tr;
        };
        // macro-steps [T0, T1).  Few channels: the increments of the next step's column are fetched as soon as this
        // step's have been used, into the same registers, and arrive while the cells are updated.  Many channels: that
        // is not long enough, and they are fetched a whole step ahead into a second set of registers.  (The step after
        // the last one of a range reads a row that exists: the next range's, or the row of zeros.)
        auto run = [&](auto edge_c, auto tc_c, int T0, int T1) __attribute__((always_inline)) {
            if (T0 >= T1) return;
            real p[M];
            if constexpr (D < 16) {
                int J, Jn;
                real y[D];
                fetch(edge_c, T0, J, y, c_0(), c_d());
                for (int T = T0; T < T1; ++T) {
                    inner(edge_c, tc_c, J, y, p);
                    fetch(edge_c, T + 1, Jn, y, c_0(), c_d());
                    J = Jn;
                    cells(p);
                }
            } else {
                int Ja, Jb;
                real ya[D], yb[D];
                fetch(edge_c, T0, Ja, ya, c_0(), c_d());
                int T = T0;
                for (; T + 2 <= T1; T += 2) {
                    fetch(edge_c, T + 1, Jb, yb, c_0(), c_d());
                    inner(edge_c, tc_c, Ja, ya, p);
                    cells(p);
                    fetch(edge_c, T + 2, Ja, ya, c_0(), c_d());
                    inner(edge_c, tc_c, Jb, yb, p);
                    cells(p);
                }
                if (T < T1) {
                    inner(edge_c, tc_c, Ja, ya, p);
                    cells(p);
                }
            }
        };
        // (tc_c: whether there is a time channel; without one its constant is not added)
        auto sweep = [&](auto tc_c) __attribute__((always_inline)) {
            const int Ti = nb > LP - 1 ? LP - 1 : NT;   // end of the leading edge range
            run(std::true_type(), tc_c, 0, Ti);
            if (nb > LP - 1) {
                run(std::false_type(), tc_c, LP - 1, nb);
                run(std::true_type(), tc_c, nb, NT);
            }
        };
        if (a.tc != 0.0) sweep(std::true_type());
        else sweep(std::false_type());
        if (r == LP - 1 && valid) {
            const long N = a.gramN;
            const long pid = a.tri ? xi * N + yi : xi * a.gramM + yi;
            a.k_out[pid] = f.bot[C - 1];
            if (a.tri && xi != yi) a.k_out[yi * N + xi] = f.bot[C - 1];
        }
    }
}

// ------------------------------------------------------------------------------------------------
// launcher
// ------------------------------------------------------------------------------------------------
template <int BL, int D, int M>
static hipError_t launch_quad_fwd_t(const SweepArgs& a, int grid, size_t lds, hipStream_t st)
{
    if (hipError_t e = allow_full_lds(reinterpret_cast<const void*>(&quad_fwd_kernel<BL, D, M>)); e != hipSuccess) return e;
    hipLaunchKernelGGL((quad_fwd_kernel<BL, D, M>), dim3(grid), dim3(kWavesPerWG * kWave), lds, st, a);
    return hipGetLastError();
}

template <int BL, int D>
static hipError_t launch_quad_fwd_m(const SweepArgs& a, int grid, size_t lds, hipStream_t st)
{
    if (a.lk_M == 4) return launch_quad_fwd_t<BL, D, 4>(a, grid, lds, st);
    if constexpr (quad_max_rows(BL, D) >= 8) {
        if (a.lk_M == 8) return launch_quad_fwd_t<BL, D, 8>(a, grid, lds, st);
    }
    return hipErrorInvalidValue;
}

template <int BL>
static hipError_t launch_quad_fwd_bl(int DT, const SweepArgs& a, int grid, size_t lds, hipStream_t st)
{
    switch (DT) {
        case 2: return launch_quad_fwd_m<BL, 2>(a, grid, lds, st);
        case 3: return launch_quad_fwd_m<BL, 3>(a, grid, lds, st);
        case 4: return launch_quad_fwd_m<BL, 4>(a, grid, lds, st);
        case 5: return launch_quad_fwd_m<BL, 5>(a, grid, lds, st);
        case 6: return launch_quad_fwd_m<BL, 6>(a, grid, lds, st);
        case 8: return launch_quad_fwd_m<BL, 8>(a, grid, lds, st);
        case 16:
            if constexpr (BL == 0) return launch_quad_fwd_m<BL, 16>(a, grid, lds, st);
            return hipErrorInvalidValue;
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_sweep_quad(int BL, int DT, const SweepArgs& a, int grid, size_t lds, hipStream_t st)
{
    // what the kernel assumes about the launch
    const int rows = (kWave / kQuadPairs) * a.lk_M;
    if (!a.gramM || !a.k_out || a.rs1 != 0 || a.rs2 != 0 || a.ll != 0 || a.mb < 1 || a.mb > rows || a.nb < 1 || a.q != a.nb ||
        a.lk_padb != rows - a.mb || a.DS < DT || a.d > DT || a.qd_nquads < 1 || a.lk_M > quad_max_rows(BL, DT) ||
        (size_t)(a.nb + 1) * quad_y_stride(DT) * sizeof(real) > a.lds_wave || (size_t)a.lds_wave * kWavesPerWG > lds)
        return hipErrorInvalidValue;
    switch (BL) {
        case 0: return launch_quad_fwd_bl<0>(DT, a, grid, lds, st);
        case 1: return launch_quad_fwd_bl<1>(DT, a, grid, lds, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace sk

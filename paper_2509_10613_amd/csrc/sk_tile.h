// Shared by the tile kernels (sk_tile.hip: forward; sk_tile_bwd.hip: backward): operand layouts of the MFMA tiles and
// the column clamp of the sweeps.  The two kernels are compiled in files of their own: in one file the compiler's
// choices for the one changed with the other's code (the forward kernel lost 12 % that way).
#pragma once
#include <hip/hip_runtime.h>

#include <type_traits>

#include "sk_dev.h"
#include "sk_kernels.h"
#include "sk_lane.h"

namespace sk {


typedef double real4 __attribute__((ext_vector_type(4)));

// Column a lane reads p from: J inside the grid, else the zero column nb (J < 0 is a huge unsigned number).
__device__ __forceinline__ int read_col(int J, int nb) { return (int)min((unsigned)J, (unsigned)nb); }
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
            // (rowoff is at most 32, the tile kernels' shapes: only the first two row tiles can reach above the grid)
            if (T < 2) {
#pragma unroll
                for (int kc = 0; kc < KC; ++kc) v[T][kc] = row >= 0 ? t[kc] : 0.0;
            } else {
#pragma unroll
                for (int kc = 0; kc < KC; ++kc) v[T][kc] = t[kc];
            }
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
            // (rowoff is at most 32: rows 4 kk + g16 with kk >= 8 lie inside the grid)
            if (kk < 8) v[kk] = (row >= 0 && n16 < D) ? t[kk] : 0.0;
            else v[kk] = n16 < D ? t[kk] : 0.0;
        }
    }
    // Delta tiles into P.  Result register r of lane l of tile (J, I) is Delta[a = 16 I + l % 16][b = 16 J + l / 16 + 4 r].
    // The time channel adds its constant product inside the grid only (TC = false: there is none, tc is zero).
    template <bool TC = true>
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
                    real v = acc[r];
                    if constexpr (TC) v += (al >= padb && b < nb) ? tc : 0.0;
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


// defined in sk_tile_bwd.hip; grid counts workgroups of kWavesPerWG waves, as the launch plan does
hipError_t launch_tile_bwd(int DT, const SweepArgs& a, int grid, hipStream_t st);

}  // namespace sk

// Kernel arguments and launchers of the truncated-signature path (Section 2.3), shared by the entry points and the
// kernel file.
#pragma once
#include <hip/hip_runtime.h>

#include "sg_plan.h"

namespace sg {

struct Args {
    const double* dz;   // [B][np][Dpad] increments of the transformed paths, rows n..np-1 zero
    double* out;        // [B][sig_len]
    long B;
    long n;             // segments per path
    long np;            // stored rows per path: n rounded up to an odd number (0 if n = 0)
    int D, Dpad, N, Q, NB;
    long LP, WP;        // lanes and waves per path
    long sig_len;
    int PW;             // paths per wave (1, or several short paths side by side in a wave: then WP = 1)
    long NW;            // waves of the launch
    int leadlag;        // rows alternate between moves of the lead and of the lag half of the channels (n is even)
};

struct BwdArgs {
    const double* dz;    // [B][np][Dpad] increments of the transformed paths
    double* gz;          // [B][np][Dpad] dF/dz, zero on entry, accumulated by atomics
    const double* sig;   // [B][sig_len] signatures of the whole paths
    const double* gout;  // [B][sig_len] upstream gradient
    long B;
    long n, np;
    int D, Dpad, N, Q, NB;
    long LP, WP;
    long sig_len;
    size_t lds_wave;     // doubles of LDS per wave
    int PW;              // paths per wave (several short paths side by side: then WP = 1)
    long NW;             // waves of the launch
    int leadlag;         // rows alternate between moves of the lead and of the lag half of the channels (n is even)
};

hipError_t launch_horner(int DT, int M, int S, const Args& a, long grid, hipStream_t st);
hipError_t launch_horner_bwd(int DT, int M, int S, const BwdArgs& a, long grid, size_t lds_bytes, hipStream_t st);

template <typename TO>
hipError_t launch_point_gradients(const double* gz, TO* gx, long B, long L, int d, int Dpad, int P, long Lc, long np,
                                  int lead_lag, hipStream_t st);

// adjoints of the two factors of each pair product: Gc[2 i] = adjoint of X[2 i], Gc[2 i + 1] = adjoint of X[2 i + 1],
// given the adjoint Gp[i] of X[2 i] (x) X[2 i + 1]
hipError_t launch_chen_pairs_adjoint(const double* X, const double* Gp, double* Gc, long pairs, int D, int N, long sig_len,
                                     hipStream_t st);

template <typename TI>
hipError_t launch_increments(const TI* x, double* dz, long B, long L, int d, int D, int Dpad, long n, int P, long Lc,
                             long np, int time_aug, int lead_lag, hipStream_t st);

// out[i] = in[2 i] (x) in[2 i + 1] for i < pairs, signatures of sig_len entries (levels 0..N over D channels)
hipError_t launch_chen_pairs(const double* in, double* out, long pairs, int D, int N, long sig_len, hipStream_t st);

}  // namespace sg

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
};

hipError_t launch_horner(int DT, int M, int S, const Args& a, long grid, hipStream_t st);

template <typename TI>
hipError_t launch_increments(const TI* x, double* dz, long B, long L, int d, int D, int Dpad, long n, long np,
                             int time_aug, int lead_lag, hipStream_t st);

}  // namespace sg

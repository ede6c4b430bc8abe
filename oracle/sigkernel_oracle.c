/*
 * TEST INFRASTRUCTURE - not part of the product path.  Only the tests, the smoke check and the
 * benchmark's cpu_baseline leg may load this library.
 *
 * CPU oracle for signature kernels (paper Section 3).  The arithmetic lives in
 * sigkernel_oracle_impl.h; this file instantiates it for double (_f64) and long double (_f80).
 * Build: gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC (see oracle/build.py).
 */
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define REAL double
#define SUFFIX _f64
#include "sigkernel_oracle_impl.h"
#undef REAL
#undef SUFFIX

#define REAL long double
#define SUFFIX _f80
#include "sigkernel_oracle_impl.h"
#undef REAL
#undef SUFFIX

/* Number of threads the batch entry points will use. */
int osk_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

// Solo kernels: the backward kernels that could share a SIMD, built for one wave per SIMD (see sk_solo_impl.h).
#define SK_SOLO_ONE 1
#include "sk_solo_impl.h"

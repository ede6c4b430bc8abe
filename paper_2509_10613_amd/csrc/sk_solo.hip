// Solo kernels: the forward kernels and the backward kernels at the occupancy the launch plan allows them at most.
#include "sk_solo_impl.h"

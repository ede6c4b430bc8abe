// Device-side helpers shared by the sweep kernels: LDS-typed pointers, lane exchange by DPP, scratch loads
// and fences, LDS atomics.
#pragma once
#include <hip/hip_runtime.h>

#include "sk_kernels.h"

namespace sk {

// Pointers into LDS keep their address space in the type, so that every access is a ds_* instruction.
#define SK_LDS __attribute__((address_space(3)))

// ------------------------------------------------------------------------------------------------
// lane exchange helpers (must be called with all 64 lanes active)
// ------------------------------------------------------------------------------------------------
// lane i receives v of lane i-1; lane 0 receives edge (its own lane's value of that argument)
__device__ __forceinline__ real wave_from_above_or(real v, real edge)
{
    int lo = __double2loint(v), hi = __double2hiint(v);
    int elo = __double2loint(edge), ehi = __double2hiint(edge);
    lo = __builtin_amdgcn_update_dpp(elo, lo, 0x138, 0xf, 0xf, false);
    hi = __builtin_amdgcn_update_dpp(ehi, hi, 0x138, 0xf, 0xf, false);
    return __hiloint2double(hi, lo);
}
// lane i receives v of lane i+1; lane 63 receives edge
__device__ __forceinline__ real wave_from_below_or(real v, real edge)
{
    int lo = __double2loint(v), hi = __double2hiint(v);
    int elo = __double2loint(edge), ehi = __double2hiint(edge);
    lo = __builtin_amdgcn_update_dpp(elo, lo, 0x130, 0xf, 0xf, false);
    hi = __builtin_amdgcn_update_dpp(ehi, hi, 0x130, 0xf, 0xf, false);
    return __hiloint2double(hi, lo);
}
// shifts of the feed registers: the lane that has no source receives zero
__device__ __forceinline__ real wave_shift_down(real v)   // lane i receives lane i+1
{
    int lo = __double2loint(v), hi = __double2hiint(v);
    lo = __builtin_amdgcn_update_dpp(0, lo, 0x130, 0xf, 0xf, true);
    hi = __builtin_amdgcn_update_dpp(0, hi, 0x130, 0xf, 0xf, true);
    return __hiloint2double(hi, lo);
}
__device__ __forceinline__ real wave_shift_up(real v)     // lane i receives lane i-1
{
    int lo = __double2loint(v), hi = __double2hiint(v);
    lo = __builtin_amdgcn_update_dpp(0, lo, 0x138, 0xf, 0xf, true);
    hi = __builtin_amdgcn_update_dpp(0, hi, 0x138, 0xf, 0xf, true);
    return __hiloint2double(hi, lo);
}

// Lane i receives v of lane i+1, except the strip's last lane lb, which receives edge (its own lane's
// value of that argument).  full = (lb == 63) is wave-uniform.
template <bool FULL>
__device__ __forceinline__ real recv_from_below(real v, real edge, bool is_lb)
{
    if constexpr (FULL) {
        return wave_from_below_or(v, edge);
    } else {
        const real t = wave_shift_down(v);
        return is_lb ? edge : t;
    }
}

// Device-scope load that bypasses the per-CU vector cache: used for data this wave wrote to global
// scratch earlier in the same kernel.
__device__ __forceinline__ real ld_scratch(const real* p)
{
    unsigned long long u = __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p), __ATOMIC_RELAXED,
                                             __HIP_MEMORY_SCOPE_AGENT);
    return __longlong_as_double((long long)u);
}

// Scratch written by a wave is only ever read back by waves of the same workgroup (same CU, hence the same
// L2): it is enough that the stores have completed (they write through to L2) and that the reads bypass the
// per-CU vector cache (ld_scratch).  An agent-scope fence would write back and invalidate the whole L2.
__device__ __forceinline__ void scratch_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

__device__ __forceinline__ void lds_atomic_add(SK_LDS real* p, real v)
{
    (void)__hip_atomic_fetch_add(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
}

// Ordering of LDS traffic only: the hardware executes the LDS instructions of a wave in order, so all that is
// needed around a flag access is that the compiler keeps the order and that outstanding LDS operations
// have completed.  (A workgroup-scope release/acquire would also wait for every global load and store in
// flight, which here includes checkpoint traffic with microseconds of latency.)
__device__ __forceinline__ void lds_order() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }


// Pair q of the sequence a launch of the solo / tile kernels works through: the identity for pair batches, y-major
// for Gram matrices (q = m N + n: consecutive pairs share the y path), and for a symmetric Gram matrix K(X, X)
// only the pairs n <= m (k(x, y) = k(y, x) holds bit for bit, Section 3.1: the other half is a copy).  There the
// rows m and N - 1 - m, which hold m + 1 and N - m such pairs, form one virtual row of N + 1 pairs, so that
// contiguous runs of the sequence are equally long whatever the row.  pid / pid2: where K[n, m] and its mirror
// image live (equal on the diagonal).
__device__ __forceinline__ void gram_pair(const SweepArgs& a, long q, long& xi, long& yi, long& pid, long& pid2)
{
    if (!a.gramM) {
        xi = yi = pid = pid2 = q;
    } else if (!a.tri) {
        yi = q / a.gramN;
        xi = q - yi * a.gramN;
        pid = pid2 = xi * a.gramM + yi;
    } else {
        const long N = a.gramN;
        const long vr = q / (N + 1), t = q - vr * (N + 1);
        if (t <= vr) { yi = vr; xi = t; }
        else { yi = N - 1 - vr; xi = t - vr - 1; }
        pid = xi * N + yi;
        pid2 = yi * N + xi;
    }
}
// The same sequence walked pair by pair: locate() divides once, next() adds and compares.
struct PairCursor {
    long xi, yi, pid, pid2;
    long vr, t;   // symmetric case: virtual row and place in it
    __device__ __forceinline__ void locate(const SweepArgs& a, long q)
    {
        gram_pair(a, q, xi, yi, pid, pid2);
        vr = t = 0;
        if (a.gramM && a.tri) {
            vr = q / (a.gramN + 1);
            t = q - vr * (a.gramN + 1);
        }
    }
    __device__ __forceinline__ void next(const SweepArgs& a)
    {
        if (!a.gramM) {
            ++xi; ++yi; ++pid; ++pid2;
        } else if (!a.tri) {
            ++xi;
            pid += a.gramM;
            if (xi == a.gramN) { xi = 0; ++yi; pid = yi; }
            pid2 = pid;
        } else {
            const long N = a.gramN;
            if (++t > N) { t = 0; ++vr; }
            if (t <= vr) { yi = vr; xi = t; }
            else { yi = N - 1 - vr; xi = t - vr - 1; }
            pid = xi * N + yi;
            pid2 = yi * N + xi;
        }
    }
};
// Upstream gradient of the pair: in the symmetric case the pair stands for both (n, m) and (m, n).
__device__ __forceinline__ real gram_weight(const SweepArgs& a, long pid, long pid2)
{
    const real g = a.grad_k[pid];
    return pid2 != pid ? g + a.grad_k[pid2] : g;
}

// Called by one lane: the pair's inverse recurrence drifted, list it for the replay kernel.
__device__ __forceinline__ void list_drifted(const SweepArgs& a, long pid, long pid2)
{
    const int n = pid2 != pid ? 2 : 1;
    const int at = atomicAdd(a.bad_count, n);
    a.bad_list[at] = pid;
    if (n == 2) a.bad_list[at + 1] = pid2;
}

__device__ __forceinline__ void pair_ids(const SweepArgs& a, long pid, long& xi, long& yi)
{
    xi = a.gramM ? pid / a.gramM : pid;
    yi = a.gramM ? pid % a.gramM : pid;
}

}  // namespace sk

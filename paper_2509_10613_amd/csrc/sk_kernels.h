// Kernel argument block and launcher declarations shared by the HIP kernels and the C-ABI layer.
#pragma once
#include <hip/hip_runtime.h>

#include <mutex>
#include <set>
#include <utility>

#include "sk_plan.h"

namespace sk {

// Lets a kernel use the whole LDS of a compute unit as dynamic shared memory.  The attribute belongs to the kernel
// on one device, so it is set once per (device, kernel); safe to call from several host threads.
inline hipError_t allow_full_lds(const void* kernel)
{
    static std::mutex mu;
    static std::set<std::pair<int, const void*>> done;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(mu);
    if (done.count({dev, kernel})) return hipSuccess;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLdsPerCU);
    if (e == hipSuccess) done.insert({dev, kernel});
    return e;
}

using real = double;   // arithmetic type of every sweep

struct SweepArgs {
    const real* dx;      // [nx][rpad][DS] zero-padded x increments
    const real* dy;      // [ny][qpad][DS]
    long xstride, ystride;
    int rpad, qpad, DS;
    real* k_out;         // [npairs] (may be null in the backward kernel)
    const real* grad_k;  // [npairs] upstream gradients (backward)
    real* gdx;           // gradient accumulators in the layout of dx / dy (backward)
    real* gdy;
    int want_gx, want_gy;
    real* rows;          // per wave slot: ns boundary rows of rowlen elements
    long rows_slot;
    int rowlen;
    real* adj;           // per wave slot: two adjoint boundary rows
    long adj_slot;
    real* ckpt;          // per wave slot: ns * nseg checkpoints of the lane state
    long ckpt_slot;
    long npairs;
    long gramM;          // > 0: pair id -> (id / gramM, id % gramM)
    long gramN;          // rows of the Gram matrix
    int tri;             // symmetric Gram matrix in the solo / tile kernels: npairs = N (N + 1) / 2 pairs n <= m (sk_dev.h)
    int r, q;            // coarse cells per side
    int rs1, rs2;        // residual refinement shifts of block row / column to coarse index
    int mb, nb;          // block rows / columns
    int ns;              // strips
    int S, nseg;         // replay segment length, segments per strip
    int d;               // channels (runtime loop when the kernel has no compile-time count)
    real tc;             // scaled product of the two time-channel increments (0 without time augmentation)
    real sc;             // 2^-(lam1+lam2)
    // Lead-lag paths (Section 4) swept on the grid of the original increments with one more level of refinement:
    // of the 2 x 2 quadrants of that level the diagonal ones carry p, the others the time constant alone.
    // 0: no transform; 1: the level lies inside a block (rs1 = rs2 = 0); 2: above the blocks (rs1, rs2 >= 1)
    int ll;
    int y_lds;
    unsigned lds_wave;   // LDS bytes per wave
    unsigned ring_off;   // byte offset of the replay ring inside a wave's LDS
    // cooperative mode (one workgroup per pair, strips pipelined over its nw waves)
    int coop;
    int nw;              // waves per workgroup
    int RB, CH;          // outbox ring length and hand-over chunk, in block columns (powers of two)
    unsigned coop_off_gdy, coop_off_flags, coop_off_obox, coop_off_ring, coop_ring_stride;   // LDS bytes
    int uncompute;       // backward: recover forward values by inverting Eq. (1) instead of replaying segments
    // lock-step mode (one workgroup per pair: a stencil wave and a coefficient wave per strip, all waves
    // advancing in barrier-separated chunks of macro-steps)
    int lock;
    int lk_M;            // block rows per lane
    int lk_ns;           // strips of 64 * lk_M block rows
    int lk_NT;           // macro-steps per strip (a multiple of 8)
    int lk_padb;         // virtual block rows above the grid (the strips are aligned to its bottom)
    int lk_rowlen;       // doubles per hand-over row in LDS
    unsigned lk_off_y, lk_off_gy, lk_off_cring, lk_off_gp, lk_off_krows, lk_off_arows, lk_off_dump;   // LDS bytes
    unsigned lk_cring_stride, lk_gp_stride;   // LDS bytes per strip
    unsigned lk_off_ck, lk_ck_stride;         // checkpoint staging (backward)
    unsigned lk_off_gyp;                      // solo kernels, backward: y-side gradient sums of the pair in work
    int solo;            // 1: solo kernels (one wave per pair, a single strip of 64 * lk_M block rows; uses lk_M,
                         // lk_NT, lk_padb and, as offsets inside a wave's LDS, lk_off_gy / lk_off_krows / lk_off_dump)
    int band;            // 1: band kernels (a pair's strips spread over bd_nbands workgroups; uses lk_ns, lk_NT, lk_padb)
    int bd_nbands;
    int bd_spin;         // polls of another workgroup's counter before a wait gives up
    int* bd_flags;       // [2][npairs][bd_nbands] progress counters (forward, reverse), zero at launch
    unsigned bd_off_y, bd_off_gy, bd_off_rings;   // LDS bytes
    int tile;            // 1: tile kernels (one wave per pair, increment Gram matrix in LDS, contractions by MFMA; uses
                         // lk_NT, lk_padb, lk_off_krows / lk_off_dump as offsets inside a wave's LDS)
    int quad;            // 1: quad kernel (forward Gram calls: four pairs per wave; uses lk_M, lk_padb)
    long qd_nquads;      // groups of four pairs of one Gram row in the launch's sequence
    // lock-step mode on a batch of pairs of double paths: the kernels read the caller's points and write the
    // caller's gradients themselves (no preparation and finalisation launches, no global accumulators)
    int fused;
    const real* xraw;    // [npairs][L1][d]
    const real* yraw;    // [npairs][L2][d]
    real* gxraw;         // [npairs][L1][d] or null
    real* gyraw;         // [npairs][L2][d] or null
    int L1, L2;
    // the two halves of the fused backward call as launches of their own: 1 = the forward sweep only, leaving the
    // checkpoints and the strips' bottom rows in global memory; 2 = the reverse sweep only, from what 1 left; 0 = both
    int lk_phase;
    real* lk_keep;       // [npairs][lk_ns + 1][lk_rowlen]: the hand-over rows between the two launches
                         // (solo kernels: [npairs][keep_len], the pair's bottom row)
    long keep_len;
    // A kept forward sweep is signed with a hash of the call's arguments; the reverse sweep that takes it over compares
    // (a mismatch gives NaN gradients), and a backward call that sweeps forward itself erases the signature.
    unsigned long long* keep_tag;
    unsigned long long keep_tag_val;
    int* err;            // device int: 1 = a bounded wait between waves ran out, 2 = the un-compute drifted in a
                         // launch mode that cannot tell which pair (every pair is then solved once more), 3 = the
                         // workspace does not hold the forward sweep the call was told to take over
    // Pairs whose inverse recurrence drifted (solo, tile and lock-step kernels): the reverse sweep adds nothing to
    // the gradients for them and lists them here; the replay kernel then solves the listed pairs (sk_api.hip).
    long long* bad_list; // [kcount] pair ids (a pair of a symmetric Gram matrix is listed as (n, m) and (m, n))
    int* bad_count;      // entries of bad_list, zero at launch
    // the replay kernel as that second launch: 0 = an ordinary backward call over all pairs; 1 = the listed pairs
    // (all pairs if *err == 2); 2 = the listed pairs of a call that works on the caller's arrays: the wave forms the
    // pair's increments, clears its accumulators and differences them into the caller's gradients itself
    int second_chance;
};

template <typename T> hipError_t launch_fill(T* p, long n, T v, hipStream_t st);
// tag[0] = val (check == 0), or: *err = 3 if tag[0] != val, and an earlier 3 taken back if it is equal (check != 0)
hipError_t launch_keep_tag(unsigned long long* tag, unsigned long long val, int check, int* err, hipStream_t st);
template <typename TA, typename TB> hipError_t launch_convert(const TA* in, TB* out, long n, hipStream_t st);
template <typename T>
hipError_t launch_mmd2_reduce(const T* Kxx, const T* Kxy, const T* Kyy, long nxx, long nxy, long nyy, T* out,
                              hipStream_t st);
template <typename T> hipError_t launch_add_inplace(T* dst, const T* src, long n, hipStream_t st);
// dx/dy null = that side is not (re)computed (symmetric Gram); gdx/gdy null = no accumulator to clear.
template <typename T>
hipError_t launch_prepare(const T* x, real* dx, real* gdx, long nx, int L1, int rpad, const T* y, real* dy, real* gdy,
                          long ny, int L2, int qpad, int d, int DS, int* err, int nclear, hipStream_t st);
// band mode (a.band != 0), defined in sk_band.hip; phase 0: forward sweep, 1: forward sweep of the backward
// pass (checkpoints), 2: reverse sweep
hipError_t launch_sweep_band(int phase, int BL, int DT, const SweepArgs& a, int grid, size_t lds, hipStream_t st);
template <typename T>
hipError_t launch_finalize(const real* gdx, T* grad_x, long nx, int L1, int rpad, const real* gdy, T* grad_y, long ny,
                           int L2, int qpad, int d, int DS, const int* err, hipStream_t st);
hipError_t launch_sweep(bool backward, int BL, int DT, const SweepArgs& a, int grid, size_t lds, hipStream_t st);
// clears the n doubles at g1 and at g2 (either may be null) if *err == 2: every pair is about to be solved once more
hipError_t launch_second_chance_reset(real* g1, long n1, real* g2, long n2, const int* err, hipStream_t st);
// solo mode (a.solo != 0), defined in sk_solo.hip
hipError_t launch_sweep_solo(bool backward, int BL, int DT, const SweepArgs& a, int grid, size_t lds, hipStream_t st);
// the one-wave builds of the solo backward kernels (sk_solo_one.hip), called by launch_sweep_solo
hipError_t launch_sweep_solo_one(bool backward, int BL, int DT, const SweepArgs& a, int grid, size_t lds, hipStream_t st);
// tile mode (a.tile != 0), defined in sk_tile.hip
hipError_t launch_sweep_tile(bool backward, int DT, const SweepArgs& a, int grid, size_t lds, hipStream_t st);
// quad mode (a.quad != 0; forward only), defined in sk_quad.hip
hipError_t launch_sweep_quad(int BL, int DT, const SweepArgs& a, int grid, size_t lds, hipStream_t st);
// lock-step mode (a.lock != 0), defined in sk_lockstep.hip
hipError_t launch_sweep_lockstep(bool backward, int BL, int DT, const SweepArgs& a, int grid, size_t lds,
                                 hipStream_t st);

}  // namespace sk

// C-ABI entry points (declared in include/sigkernel.h): argument validation, workspace carving and the
// sequence of kernel launches for each operation.  Everything here is host code; the arithmetic of the
// method lives in the kernels.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <vector>

#include "sigkernel.h"
#include "signature.h"
#include "sg_kernels.h"
#include "sk_kernels.h"

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

// Optional HIP-event timing of the sweep kernels (for benchmarks): one event pair per sweep launch,
// recorded on the caller's stream while enabled.
struct TimedLaunch { hipEvent_t start, stop; int backward; int tag; };
std::mutex g_timing_mu;
int g_timing_tag = 0;   // 0: off; otherwise the tag new launches are recorded under
std::vector<TimedLaunch> g_timed;

// The event pair of a launch that is being timed; an error return between the two records destroys the events.
struct EventPair {
    TimedLaunch tl{};
    bool live = false;
    ~EventPair()
    {
        if (live) {
            (void)hipEventDestroy(tl.start);
            (void)hipEventDestroy(tl.stop);
        }
    }
    hipError_t begin(int backward, int tag, hipStream_t st)
    {
        hipError_t e = hipEventCreate(&tl.start);
        if (e != hipSuccess) return e;
        e = hipEventCreate(&tl.stop);
        if (e != hipSuccess) { (void)hipEventDestroy(tl.start); return e; }
        live = true;
        tl.backward = backward;
        tl.tag = tag;
        return hipEventRecord(tl.start, st);
    }
    hipError_t end(hipStream_t st)
    {
        hipError_t e = hipEventRecord(tl.stop, st);
        if (e != hipSuccess) return e;
        std::lock_guard<std::mutex> lk(g_timing_mu);
        g_timed.push_back(tl);
        live = false;   // the reader releases them
        return hipSuccess;
    }
};

int timing_tag()
{
    std::lock_guard<std::mutex> lk(g_timing_mu);
    return g_timing_tag;
}

int validate(int64_t nx, int64_t ny, int64_t L1, int64_t L2, int64_t d, int lam1, int lam2, int flags, int dt)
{
    if (dt != SK_F32 && dt != SK_F64) return fail(SK_ERR_DTYPE, "dtype %d is neither SK_F32 nor SK_F64", dt);
    if (flags & ~(SK_FLAG_TIME_AUG | SK_FLAG_BWD_REPLAY | SK_FLAG_SHORT_WAITS | SK_FLAG_LEAD_LAG | SK_FLAG_KEEP_FORWARD |
                  SK_FLAG_HAVE_FORWARD))
        return fail(SK_ERR_DTYPE, "unknown flag bits 0x%x", flags);
    if (lam1 < 0 || lam2 < 0 || lam1 > 20 || lam2 > 20)
        return fail(SK_ERR_DYADIC, "dyadic orders (%d, %d) outside 0..20", lam1, lam2);
    if (nx < 0 || ny < 0) return fail(SK_ERR_SHAPE, "negative batch size");
    if (L1 < 1 || L2 < 1 || d < 1) return fail(SK_ERR_SHAPE, "need L1, L2, d >= 1 (got %lld, %lld, %lld)",
                                               (long long)L1, (long long)L2, (long long)d);
    const int64_t lim = (int64_t)1 << 29;
    if (L1 > lim || L2 > lim || ((L1 - 1) << lam1) >= lim || ((L2 - 1) << lam2) >= lim)
        return fail(SK_ERR_SHAPE, "refined grid side (L-1) << lambda must stay below 2^29");
    if (d > 65536) return fail(SK_ERR_SHAPE, "d above 65536");
    if ((flags & SK_FLAG_LEAD_LAG) && (2 * L1 - 1 > lim || 2 * L2 - 1 > lim || ((2 * L1 - 2) << lam1) >= lim ||
                                       ((2 * L2 - 2) << lam2) >= lim))
        return fail(SK_ERR_SHAPE, "lead-lag transform: refined grid side 2 (L-1) << lambda must stay below 2^29");
    if (nx > ((int64_t)1 << 40) || ny > ((int64_t)1 << 40)) return fail(SK_ERR_SHAPE, "batch too large");
    return SK_OK;
}

// The scratch of a call: the launch plan's, then (backward calls whose reverse sweep inverts Eq. (1)) that of the
// launch that solves drifted pairs once more with the replay kernel.
struct Layout {
    sk::Plan p;
    sk::Plan sc;          // the second launch (valid only if has_sc)
    bool has_sc = false;
    size_t off_sc = 0;
    size_t total = 0;
    // Lead-lag transform (Section 4): the plan is that of the caller's paths with one more dyadic level on either
    // side, swept in its lead-lag form (every kernel but the tile kernels has one, and such plans never choose those).
    bool ll = false;
};

// L1, L2, d, lam1, lam2 are the caller's.
Layout make_layout(bool backward, bool gram, bool symmetric, int64_t nx, int64_t ny, int64_t L1, int64_t L2, int64_t d,
                   int lam1, int lam2, int flags, int io_elem, bool uncompute, bool keep = false)
{
    Layout l;
    l.ll = (flags & SK_FLAG_LEAD_LAG) != 0;
    if (l.ll) { lam1 += 1; lam2 += 1; }
    l.p = sk::make_plan(backward, gram, symmetric, nx, ny, L1, L2, d, lam1, lam2, io_elem, uncompute, keep, false, l.ll);
    l.total = l.p.total;
    if (l.p.valid && backward && l.p.uncompute) {
        l.sc = sk::make_plan(true, gram, symmetric, nx, ny, L1, L2, d, lam1, lam2, io_elem, false, false, true, l.ll);
        l.has_sc = l.sc.valid;
        l.off_sc = l.p.total;
        l.total = l.p.total + l.sc.total;
    }
    return l;
}

// T is the element type of the caller's arrays.  The sweeps run in double whatever T is: non-packed
// single-precision vector instructions issue at the same rate as double ones on this chip, and the
// recurrence of Eq. (1) in single precision loses the low bits of p when forming 1 + p/2 + ..., an error
// that grows linearly with the number of cells.  Float callers get float storage at the edges only.
template <typename T>
int run(const Layout& lay, bool backward, const void* x, const void* y, void* k, const void* grad_k, void* grad_x,
        void* grad_y, int lam1, int lam2, int flags, void* ws, hipStream_t st, int phase = 0)
{
    using namespace sk;
    const Plan& p = lay.p;
    constexpr bool kIsDouble = sizeof(T) == 8;
    unsigned char* base = static_cast<unsigned char*>(ws);
    double* dxT = reinterpret_cast<double*>(base + p.off_dxT);
    double* dyT = reinterpret_cast<double*>(base + p.off_dyT);
    hipError_t e;
#define SK_CHECK(call)                                                                         \
    do {                                                                                       \
        e = (call);                                                                            \
        if (e != hipSuccess) return fail(SK_ERR_HIP, "%s: %s", #call, hipGetErrorString(e));   \
    } while (0)

    SweepArgs a;
    std::memset(&a, 0, sizeof(a));
    a.dx = dxT; a.dy = dyT;
    a.xstride = p.xstride; a.ystride = p.ystride;
    a.rpad = p.rpad; a.qpad = p.qpad; a.DS = p.DP;
    if (kIsDouble) {
        a.k_out = static_cast<double*>(k);
        a.grad_k = static_cast<const double*>(grad_k);
    } else {
        a.k_out = k ? reinterpret_cast<double*>(base + p.off_kio) : nullptr;
        if (backward && phase != 1) {
            double* gk64 = reinterpret_cast<double*>(base + p.off_gkio);
            SK_CHECK((launch_convert<T, double>(static_cast<const T*>(grad_k), gk64, p.kcount, st)));
            a.grad_k = gk64;
        }
    }
    a.rows = reinterpret_cast<double*>(base + p.off_rows);
    a.rows_slot = p.rows_slot;
    a.rowlen = p.rowlen;
    a.npairs = p.npairs;
    a.gramM = p.gramM;
    a.gramN = p.nx;
    a.tri = p.tri;
    a.r = p.r; a.q = p.q; a.rs1 = p.rs1; a.rs2 = p.rs2; a.mb = p.mb; a.nb = p.nb; a.ns = p.ns;
    a.S = p.S; a.nseg = p.nseg; a.d = p.d;
    const double sc = 1.0 / (double)((int64_t)1 << (lam1 + lam2));
    a.sc = sc;
    // the time channel t_i = i / (points - 1) of the paths the sweep stands for (lead-lag paths have 2L - 1 points)
    const int tsteps1 = lay.ll ? 2 * (p.L1 - 1) : p.L1 - 1, tsteps2 = lay.ll ? 2 * (p.L2 - 1) : p.L2 - 1;
    a.tc = (flags & SK_FLAG_TIME_AUG) ? sc * (1.0 / (double)tsteps1) * (1.0 / (double)tsteps2) : 0.0;
    a.ll = p.ll;
    a.y_lds = p.y_lds;
    a.lds_wave = (unsigned)p.lds_wave;
    a.ring_off = (unsigned)p.ring_off;
    a.coop = p.coop; a.nw = p.nw; a.RB = p.RB; a.CH = p.CH;
    a.uncompute = p.uncompute;
    a.coop_off_gdy = (unsigned)p.coop_off_gdy; a.coop_off_flags = (unsigned)p.coop_off_flags;
    a.coop_off_obox = (unsigned)p.coop_off_obox; a.coop_off_ring = (unsigned)p.coop_off_ring;
    a.coop_ring_stride = (unsigned)p.coop_ring_stride;
    a.solo = p.solo;
    a.tile = p.tile;
    a.quad = p.quad; a.qd_nquads = p.nquads;
    a.band = p.band; a.bd_nbands = p.bd_nbands;
    a.bd_off_y = (unsigned)p.bd_off_y; a.bd_off_gy = (unsigned)p.bd_off_gy; a.bd_off_rings = (unsigned)p.bd_off_rings;
    a.bd_flags = reinterpret_cast<int*>(base + p.off_flags);
    a.bd_spin = (flags & SK_FLAG_SHORT_WAITS) ? 1 : kBandSpin;
    a.lock = p.lock; a.lk_M = p.lk_M; a.lk_ns = p.lk_ns; a.lk_NT = p.lk_NT; a.lk_padb = p.lk_padb;
    a.lk_rowlen = p.lk_rowlen;
    a.lk_off_y = (unsigned)p.lk_off_y; a.lk_off_gy = (unsigned)p.lk_off_gy; a.lk_off_cring = (unsigned)p.lk_off_cring;
    a.lk_off_gp = (unsigned)p.lk_off_gp; a.lk_off_krows = (unsigned)p.lk_off_krows;
    a.lk_off_arows = (unsigned)p.lk_off_arows; a.lk_off_dump = (unsigned)p.lk_off_dump;
    a.lk_cring_stride = (unsigned)p.lk_cring_stride; a.lk_gp_stride = (unsigned)p.lk_gp_stride;
    a.lk_off_ck = (unsigned)p.lk_off_ck; a.lk_ck_stride = (unsigned)p.lk_ck_stride;

    if (backward) {
        a.gdx = reinterpret_cast<double*>(base + p.off_gdxT);
        a.gdy = reinterpret_cast<double*>(base + p.off_gdyT);
        a.want_gx = grad_x != nullptr;
        a.want_gy = p.symmetric ? (grad_x != nullptr) : (grad_y != nullptr);
        a.adj = reinterpret_cast<double*>(base + p.off_adj);
        a.adj_slot = p.adj_slot;
        a.ckpt = reinterpret_cast<double*>(base + p.off_ckpt);
        a.ckpt_slot = p.ckpt_slot;
    }
    a.err = reinterpret_cast<int*>(base + p.off_err);
    a.lk_off_gyp = (unsigned)p.lk_off_gyp;
    if (p.off_badlist != 0) {
        a.bad_count = reinterpret_cast<int*>(base + p.off_badcnt);
        a.bad_list = reinterpret_cast<long long*>(base + p.off_badlist);
    }
    // Lock-step mode on a batch of pairs of double paths works on the caller's arrays directly.
    const bool fused = p.lock && p.gramM == 0 && kIsDouble;
    if (fused) {
        a.fused = 1;
        a.xraw = static_cast<const double*>(x);
        a.yraw = static_cast<const double*>(y);
        a.gxraw = static_cast<double*>(grad_x);
        a.gyraw = static_cast<double*>(grad_y);
        a.L1 = p.L1; a.L2 = p.L2;
        a.lk_phase = phase;
        a.lk_keep = backward ? reinterpret_cast<double*>(base + p.off_keep) : nullptr;
    } else if (phase != 0 && p.keep_solo) {
        a.lk_phase = phase;
        a.lk_keep = reinterpret_cast<double*>(base + p.off_keep);
        a.keep_len = p.keep_len;
    } else if (phase != 0 && !p.band) {
        return fail(SK_ERR_SHAPE, "internal: no split form of this launch");
    }
    // Band mode is two launches anyway (forward sweep with checkpoints and bottom rows in global memory, reverse
    // sweep); a kept forward sweep is the first of them, and its kernel values wait in the workspace.
    double* keep_k = (p.band && phase != 0) ? reinterpret_cast<double*>(base + p.off_keep) : nullptr;
    const bool own_tag_launch = p.band || p.keep_solo;   // these sign, erase and check in launches of their own
    if (backward && ((p.gramM == 0 && (fused || p.band)) || p.keep_solo) && p.off_keep_tag != 0) {
        a.keep_tag = reinterpret_cast<unsigned long long*>(base + p.off_keep_tag);
        // FNV-1a over what the kept sweep depends on
        unsigned long long h = 1469598103934665603ull;
        auto mix = [&](unsigned long long v) {
            for (int i = 0; i < 8; ++i) { h ^= (v >> (8 * i)) & 0xffull; h *= 1099511628211ull; }
        };
        mix(reinterpret_cast<uintptr_t>(x)); mix(reinterpret_cast<uintptr_t>(y));
        mix((unsigned long long)p.npairs); mix((unsigned long long)p.nx); mix((unsigned long long)p.ny);
        mix((unsigned long long)p.L1); mix((unsigned long long)p.L2);
        mix((unsigned long long)p.d); mix((unsigned long long)lam1); mix((unsigned long long)lam2);
        mix((unsigned long long)(flags & (SK_FLAG_TIME_AUG | SK_FLAG_LEAD_LAG))); mix(sizeof(T));
        a.keep_tag_val = h | 1ull;
    }
    // one preparation launch: increments of both sides, cleared gradient accumulators, cleared error flag
    // (the reverse sweep of a kept forward sweep: the same increments once more, cleared accumulators, and only the
    // reverse sweep's progress counters cleared - the error flag still says how the forward sweep went)
    if (!fused)
    SK_CHECK(launch_prepare<T>(static_cast<const T*>(x), dxT, (backward && a.want_gx) ? a.gdx : nullptr, p.nx, p.L1,
                               p.rpad, static_cast<const T*>(y), p.symmetric ? nullptr : dyT,
                               (backward && a.want_gy && !p.symmetric) ? a.gdy : nullptr, p.ny, p.L2, p.qpad, p.d,
                               p.DP, phase == 2 ? a.bd_flags + p.nflags / 2 : a.err,
                               phase == 2 ? p.nflags / 2 + 1 : 1 + (int)((p.off_flags - p.off_err) / sizeof(int)) + p.nflags,
                               st));   // (both ranges end with the counter of drifted pairs, the int behind the flags)
    // the calls that work on the caller's arrays have no preparation launch: their counter of drifted pairs
    if (fused && backward && phase != 1 && a.bad_count) SK_CHECK(launch_fill<int>(a.bad_count, 1, 0, st));
    // band mode signs, erases and checks a kept sweep in launches of their own (the lock-step kernels do it themselves)
    if (own_tag_launch && phase == 2) SK_CHECK(launch_keep_tag(a.keep_tag, a.keep_tag_val, 1, a.err, st));
    const int ttag = timing_tag();
    EventPair ev;
    if (ttag) SK_CHECK(ev.begin((backward && phase != 1) ? 1 : 0, ttag, st));   // a kept forward sweep counts as a forward launch
    if (p.band) SK_CHECK(launch_sweep_band(phase ? phase + 1 : (backward ? 1 : 0), p.BL, p.DT, a, p.grid, p.lds_bytes, st));
    else if (p.lock) SK_CHECK(launch_sweep_lockstep(backward, p.BL, p.DT, a, p.grid, p.lds_bytes, st));
    else if (p.quad) SK_CHECK(launch_sweep_quad(p.BL, p.DT, a, p.grid, p.lds_bytes, st));
    else if (p.tile) SK_CHECK(launch_sweep_tile(backward, p.DT, a, p.grid, p.lds_bytes, st));
    else if (p.solo) SK_CHECK(launch_sweep_solo(backward, p.BL, p.DT, a, p.grid, p.lds_bytes, st));
    else SK_CHECK(launch_sweep(backward, p.BL, p.DT, a, p.grid, p.lds_bytes, st));
    if (ttag) SK_CHECK(ev.end(st));
    // Pairs whose inverse recurrence drifted were left out of the gradient sums and listed: the replay kernel solves
    // them once more (an empty list ends that launch at once).  Launch modes that cannot tell which pairs drifted
    // raise the flag instead; then the sums are cleared and every pair is solved again.
    if (backward && phase != 1 && lay.has_sc && a.bad_count) {
        const Plan& q = lay.sc;
        unsigned char* sbase = base + lay.off_sc;
        SweepArgs b = a;
        b.second_chance = fused ? 2 : 1;
        b.npairs = p.kcount;
        b.tri = 0;
        b.rows = reinterpret_cast<double*>(sbase + q.off_rows);
        b.rows_slot = q.rows_slot;
        b.rowlen = q.rowlen;
        b.adj = reinterpret_cast<double*>(sbase + q.off_adj);
        b.adj_slot = q.adj_slot;
        b.ckpt = reinterpret_cast<double*>(sbase + q.off_ckpt);
        b.ckpt_slot = q.ckpt_slot;
        b.ns = q.ns; b.S = q.S; b.nseg = q.nseg;
        b.y_lds = q.y_lds;
        b.lds_wave = (unsigned)q.lds_wave;
        b.ring_off = (unsigned)q.ring_off;
        b.coop = 0; b.uncompute = 0; b.lock = 0; b.solo = 0; b.tile = 0; b.band = 0;
        b.lk_phase = 0; b.keep_tag = nullptr;
        if (!(p.lock || p.solo || p.tile))
            SK_CHECK(launch_second_chance_reset(a.want_gx ? a.gdx : nullptr, (long)(p.nx * p.xstride),
                                                (a.want_gy && !p.symmetric) ? a.gdy : nullptr,
                                                (long)(p.ny * p.ystride), a.err, st));
        SK_CHECK(launch_sweep(true, q.BL, q.DT, b, q.grid, q.lds_bytes, st));
    }
    if (own_tag_launch && a.keep_tag && phase != 2) SK_CHECK(launch_keep_tag(a.keep_tag, phase == 1 ? a.keep_tag_val : 0ull, 0, a.err, st));
    if (keep_k && phase == 1)
        SK_CHECK(hipMemcpyAsync(keep_k, a.k_out, (size_t)p.kcount * sizeof(double), hipMemcpyDeviceToDevice, st));
    if (keep_k && phase == 2 && a.k_out)
        SK_CHECK(hipMemcpyAsync(a.k_out, keep_k, (size_t)p.kcount * sizeof(double), hipMemcpyDeviceToDevice, st));
    if (!kIsDouble && k) SK_CHECK((launch_convert<double, T>(a.k_out, static_cast<T*>(k), p.kcount, st)));
    if (backward && !fused && phase != 1) {
        SK_CHECK(launch_finalize<T>(a.gdx, static_cast<T*>(grad_x), p.nx, p.L1, p.rpad, a.gdy,
                                    p.symmetric ? nullptr : static_cast<T*>(grad_y), p.ny, p.L2, p.qpad, p.d, p.DP,
                                    a.err, st));
    }
#undef SK_CHECK
    return SK_OK;
}

// Degenerate shapes: no increments on one side -> k = 1 and zero gradients.
template <typename T>
int run_trivial(int64_t npairs, int64_t nx, int64_t ny, int64_t L1, int64_t L2, int64_t d, void* k, void* grad_x,
                void* grad_y, hipStream_t st)
{
    hipError_t e = hipSuccess;
    if (k) e = sk::launch_fill<T>(static_cast<T*>(k), npairs, T(1), st);
    if (e == hipSuccess && grad_x) e = sk::launch_fill<T>(static_cast<T*>(grad_x), nx * L1 * d, T(0), st);
    if (e == hipSuccess && grad_y) e = sk::launch_fill<T>(static_cast<T*>(grad_y), ny * L2 * d, T(0), st);
    if (e != hipSuccess) return fail(SK_ERR_HIP, "fill: %s", hipGetErrorString(e));
    return SK_OK;
}

int check_device()
{
    // per device: 0 unknown, 1 ok (a failed check is repeated, and reported, by the next call)
    constexpr int kKnown = 64;
    static std::atomic<int> state[kKnown];
    int dev = 0, lds = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(SK_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
    const bool tracked = dev >= 0 && dev < kKnown;
    if (tracked && state[dev].load(std::memory_order_acquire) == 1) return SK_OK;
    e = hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev);
    if (e != hipSuccess) return fail(SK_ERR_HIP, "hipDeviceGetAttribute: %s", hipGetErrorString(e));
    if ((size_t)lds < sk::kLdsPerCU)
        return fail(SK_ERR_HIP, "device offers %d bytes of LDS per workgroup, this library is built for %zu (gfx950)",
                    lds, sk::kLdsPerCU);
    if (tracked) state[dev].store(1, std::memory_order_release);
    return SK_OK;
}

// Whether the backward plan pb has its forward and reverse sweeps as launches of their own: the lock-step kernels that
// work on the caller's arrays (pairs of double paths), the band kernels, and the solo kernels
// (pb made with keep = true: checkpoints and bottom rows per pair).
bool split_forward(const sk::Plan& pb, sk_dtype dt)
{
    if (pb.keep_solo) return true;                     // pair batches and Gram matrices
    if (pb.gramM != 0) return false;
    return pb.band || (pb.lock && dt == SK_F64);
}

int dispatch(bool backward, bool gram, const void* x, const void* y, void* k, const void* grad_k, void* grad_x,
             void* grad_y, int64_t nx, int64_t ny, int64_t L1, int64_t L2, int64_t d, int lam1, int lam2, int flags,
             sk_dtype dt, void* ws, size_t ws_bytes, void* stream)
{
    int rc = validate(nx, ny, L1, L2, d, lam1, lam2, flags, (int)dt);
    if (rc != SK_OK) return rc;
    const int64_t npairs = gram ? nx * ny : nx;
    if (npairs == 0 && !(gram && backward)) return SK_OK;
    if (!x || !y) return fail(SK_ERR_NULL, "x / y is NULL");
    if (!backward && !k) return fail(SK_ERR_NULL, "output k is NULL");
    if (backward && !grad_k) return fail(SK_ERR_NULL, "grad_k is NULL");
    const bool symmetric = gram && x == y;
    if (symmetric && (nx != ny || L1 != L2)) return fail(SK_ERR_SHAPE, "Y == X needs N == M and L1 == L2");
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int elem = dt == SK_F64 ? 8 : 4;
    if (symmetric) grad_y = nullptr;

    if (L1 == 1 || L2 == 1 || npairs == 0) {
        if (dt == SK_F64) return run_trivial<double>(npairs, nx, ny, L1, L2, d, k, grad_x, grad_y, st);
        return run_trivial<float>(npairs, nx, ny, L1, L2, d, k, grad_x, grad_y, st);
    }
    rc = check_device();
    if (rc != SK_OK) return rc;
    Layout lay = make_layout(backward, gram, symmetric, nx, ny, L1, L2, d, lam1, lam2, flags, elem,
                             !(flags & SK_FLAG_BWD_REPLAY));
    if (!lay.p.valid) return fail(SK_ERR_SHAPE, "internal: plan invalid");
    if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255) != 0)
        return fail(SK_ERR_WORKSPACE, "workspace pointer is NULL or not 256-byte aligned");
    // A forward sweep kept for the backward call: the launch modes that have the two halves of the backward call as
    // launches of their own run the first half here and the second half there; the others ignore both flags.
    int phase = 0;
    if (flags & (backward ? SK_FLAG_HAVE_FORWARD : SK_FLAG_KEEP_FORWARD)) {
        const Layout lb = make_layout(true, gram, symmetric, nx, ny, L1, L2, d, lam1, lam2, flags, elem,
                                      !(flags & SK_FLAG_BWD_REPLAY), true);
        if (!lb.p.valid) return fail(SK_ERR_SHAPE, "internal: plan invalid");
        if (ws_bytes < lb.total)
            return fail(SK_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed (a kept forward sweep: the backward call's, "
                        "asked for with the flag)", ws_bytes, lb.total);
        if (split_forward(lb.p, dt)) {
            phase = backward ? 2 : 1;
            lay = lb;
        }
    }
    if (ws_bytes < lay.total)
        return fail(SK_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", ws_bytes, lay.total);
    if (phase != 0) {
        if (phase == 1) { grad_k = nullptr; grad_x = nullptr; grad_y = nullptr; }
        if (dt == SK_F64) return run<double>(lay, true, x, y, k, grad_k, grad_x, grad_y, lam1, lam2, flags, ws, st, phase);
        return run<float>(lay, true, x, y, k, grad_k, grad_x, grad_y, lam1, lam2, flags, ws, st, phase);
    }
    if (dt == SK_F64)
        return run<double>(lay, backward, x, y, k, grad_k, grad_x, grad_y, lam1, lam2, flags, ws, st);
    return run<float>(lay, backward, x, y, k, grad_k, grad_x, grad_y, lam1, lam2, flags, ws, st);
}

}  // namespace

extern "C" {

size_t sigkernel_workspace_bytes(int op, int64_t B_or_N, int64_t M, int64_t L1, int64_t L2, int64_t d, int lam1,
                                 int lam2, int flags, sk_dtype dt)
{
    const bool gram = op == SK_OP_GRAM || op == SK_OP_GRAM_BWD;
    // a forward call that keeps its sweep works in the backward call's workspace
    const bool fwd_op = op == SK_OP_FWD || op == SK_OP_GRAM;
    const bool kept = (flags & (fwd_op ? SK_FLAG_KEEP_FORWARD : SK_FLAG_HAVE_FORWARD)) != 0;
    const bool backward = !fwd_op || kept;
    if (op < SK_OP_FWD || op > SK_OP_GRAM_BWD) return 0;
    const int64_t ny = gram ? M : B_or_N;
    if (validate(B_or_N, ny, L1, L2, d, lam1, lam2, flags, (int)dt) != SK_OK) return 0;
    // The symmetric Gram case needs no more than the general one, so the query does not distinguish them.
    const Layout l = make_layout(backward, gram, false, B_or_N, ny, L1, L2, d, lam1, lam2, flags, dt == SK_F64 ? 8 : 4,
                                 !(flags & SK_FLAG_BWD_REPLAY), kept);
    return l.p.valid ? l.total : 0;
}

int sigkernel_fwd(const void* x, const void* y, void* k, int64_t B, int64_t L1, int64_t L2, int64_t d, int lam1,
                  int lam2, int flags, sk_dtype dt, void* ws, size_t ws_bytes, void* stream)
{
    return dispatch(false, false, x, y, k, nullptr, nullptr, nullptr, B, B, L1, L2, d, lam1, lam2, flags, dt, ws,
                    ws_bytes, stream);
}

int sigkernel_bwd(const void* x, const void* y, const void* grad_k, void* grad_x, void* grad_y, void* k_out,
                  int64_t B, int64_t L1, int64_t L2, int64_t d, int lam1, int lam2, int flags, sk_dtype dt, void* ws,
                  size_t ws_bytes, void* stream)
{
    return dispatch(true, false, x, y, k_out, grad_k, grad_x, grad_y, B, B, L1, L2, d, lam1, lam2, flags, dt, ws,
                    ws_bytes, stream);
}

int sigkernel_gram(const void* X, const void* Y, void* K, const void* grad_K, void* grad_X, void* grad_Y, int64_t N,
                   int64_t M, int64_t L1, int64_t L2, int64_t d, int lam1, int lam2, int flags, sk_dtype dt,
                   void* ws, size_t ws_bytes, void* stream)
{
    return dispatch(grad_K != nullptr, true, X, Y, K, grad_K, grad_X, grad_Y, N, M, L1, L2, d, lam1, lam2, flags,
                    dt, ws, ws_bytes, stream);
}

}  // extern "C"

// ---------------------------------------------------------------- sigkernel_bwd without a caller's workspace
// Scratch of sigkernel_bwd_static: one array per GPU, part of the library's code object, alive until the process
// ends.  In host code the array's name is only a handle for hipGetSymbolAddress; kernels are given the address that
// call returns for the device in use.
namespace {
constexpr size_t kStaticScratchBytes = (size_t)SK_STATIC_SCRATCH_BYTES;
}
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};   // per device: the address of that device's copy of the array

int static_scratch(void** out)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(SK_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return fail(SK_ERR_HIP, "device index %d outside 0..%d", dev, kMaxDevices - 1);
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));   // with device `dev` current: that device's copy
        if (e != hipSuccess || !ptr)
            return fail(SK_ERR_HIP, "hipGetSymbolAddress(scratch) on device %d: %s", dev, hipGetErrorString(e));
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return SK_OK;
}
}  // namespace

extern "C" int sigkernel_bwd_static(const void* x, const void* y, const void* grad_k, void* grad_x, void* grad_y,
                                    void* k_out, int64_t B, int64_t L1, int64_t L2, int64_t d, int lam1, int lam2,
                                    int flags, sk_dtype dt, void* stream)
{
    if (flags & (SK_FLAG_KEEP_FORWARD | SK_FLAG_HAVE_FORWARD))
        return fail(SK_ERR_DTYPE, "SK_FLAG_KEEP_FORWARD / SK_FLAG_HAVE_FORWARD do not apply to sigkernel_bwd_static "
                    "(its scratch is shared by every call on the device)");
    int rc = validate(B, B, L1, L2, d, lam1, lam2, flags, (int)dt);
    if (rc != SK_OK) return rc;
    const size_t need = B > 0 ? sigkernel_workspace_bytes(SK_OP_BWD, B, 0, L1, L2, d, lam1, lam2, flags, dt) : 0;
    if (need > kStaticScratchBytes)
        return fail(SK_ERR_WORKSPACE, "this shape needs %zu bytes of scratch, sigkernel_bwd_static holds %zu per device; "
                    "use sigkernel_bwd with a workspace of the caller's", need, kStaticScratchBytes);
    void* ptr = nullptr;
    rc = static_scratch(&ptr);
    if (rc != SK_OK) return rc;
    // The preparation launch of every call clears the accumulators, the error flag and the counters it uses, and a
    // call that sweeps forward itself erases the signature of a kept sweep: nothing of the previous call's contents
    // is read before it is written.
    return dispatch(true, false, x, y, k_out, grad_k, grad_x, grad_y, B, B, L1, L2, d, lam1, lam2, flags, dt, ptr,
                    kStaticScratchBytes, stream);
}

// Layout of the scratch of sigkernel_mmd2: the three Gram matrices, their constant upstream weights, the second
// halves of the two gradients (all in the caller's element type), then the scratch of the Gram calls.
namespace {
struct MmdLayout {
    size_t kxx, kxy, kyy, wxx, wxy, wyy, gx2, gy2, sub, sub_bytes, total;
};
MmdLayout mmd_layout(int64_t N, int64_t M, int64_t L1, int64_t L2, int64_t d, int lam1, int lam2, int flags,
                     sk_dtype dt, bool grads)
{
    MmdLayout l{};
    const size_t e = dt == SK_F64 ? 8 : 4;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = sk::align_up(off + bytes, 256); return o; };
    l.kxx = take((size_t)N * N * e);
    l.kxy = take((size_t)N * M * e);
    l.kyy = take((size_t)M * M * e);
    if (grads) {
        l.wxx = take((size_t)N * N * e);
        l.wxy = take((size_t)N * M * e);
        l.wyy = take((size_t)M * M * e);
        l.gx2 = take((size_t)N * L1 * d * e);
        l.gy2 = take((size_t)M * L2 * d * e);
    }
    const int op = grads ? SK_OP_GRAM_BWD : SK_OP_GRAM;
    size_t s = sigkernel_workspace_bytes(op, N, N, L1, L1, d, lam1, lam1, flags, dt);
    size_t t = sigkernel_workspace_bytes(op, N, M, L1, L2, d, lam1, lam2, flags, dt);
    if (t > s) s = t;
    t = sigkernel_workspace_bytes(op, M, M, L2, L2, d, lam2, lam2, flags, dt);
    if (t > s) s = t;
    l.sub_bytes = s;
    l.sub = take(s);
    l.total = off;
    return l;
}

template <typename T>
int run_mmd2(const MmdLayout& l, const void* X, const void* Y, void* loss, void* grad_X, void* grad_Y, int64_t N,
             int64_t M, int64_t L1, int64_t L2, int64_t d, int lam1, int lam2, int flags, sk_dtype dt, void* ws,
             void* stream)
{
    hipStream_t st = static_cast<hipStream_t>(stream);
    unsigned char* base = static_cast<unsigned char*>(ws);
    T* Kxx = reinterpret_cast<T*>(base + l.kxx);
    T* Kxy = reinterpret_cast<T*>(base + l.kxy);
    T* Kyy = reinterpret_cast<T*>(base + l.kyy);
    void* sub = base + l.sub;
    const bool grads = grad_X != nullptr || grad_Y != nullptr;
    T *Wxx = nullptr, *Wxy = nullptr, *Wyy = nullptr, *gx2 = nullptr, *gy2 = nullptr;
    hipError_t e = hipSuccess;
    if (grads) {
        Wxx = reinterpret_cast<T*>(base + l.wxx);
        Wxy = reinterpret_cast<T*>(base + l.wxy);
        Wyy = reinterpret_cast<T*>(base + l.wyy);
        gx2 = grad_X ? reinterpret_cast<T*>(base + l.gx2) : nullptr;
        gy2 = grad_Y ? reinterpret_cast<T*>(base + l.gy2) : nullptr;
        // d loss / dK of the three blocks: constants, generated where they are used
        e = sk::launch_fill<T>(Wxx, N * N, (T)(1.0 / ((double)N * (double)N)), st);
        if (e == hipSuccess) e = sk::launch_fill<T>(Wxy, N * M, (T)(-2.0 / ((double)N * (double)M)), st);
        if (e == hipSuccess) e = sk::launch_fill<T>(Wyy, M * M, (T)(1.0 / ((double)M * (double)M)), st);
        if (e != hipSuccess) return fail(SK_ERR_HIP, "fill: %s", hipGetErrorString(e));
    }
    int rc = SK_OK;
    // K(X, X): symmetric, grad_X receives the total derivative of this block
    if (grad_X || !grads)
        rc = dispatch(grad_X != nullptr, true, X, X, Kxx, grad_X ? Wxx : nullptr, grad_X, nullptr, N, N, L1, L1, d, lam1,
                      lam1, flags, dt, sub, l.sub_bytes, stream);
    else
        rc = dispatch(false, true, X, X, Kxx, nullptr, nullptr, nullptr, N, N, L1, L1, d, lam1, lam1, flags, dt, sub,
                      l.sub_bytes, stream);
    if (rc != SK_OK) return rc;
    rc = dispatch(grads, true, X, Y, Kxy, grads ? Wxy : nullptr, gx2, gy2, N, M, L1, L2, d, lam1, lam2, flags, dt, sub,
                  l.sub_bytes, stream);
    if (rc != SK_OK) return rc;
    rc = dispatch(grad_Y != nullptr, true, Y, Y, Kyy, grad_Y ? Wyy : nullptr, grad_Y, nullptr, M, M, L2, L2, d, lam2, lam2,
                  flags, dt, sub, l.sub_bytes, stream);
    if (rc != SK_OK) return rc;
    if (grad_X) e = sk::launch_add_inplace<T>(static_cast<T*>(grad_X), gx2, N * L1 * d, st);
    if (e == hipSuccess && grad_Y) e = sk::launch_add_inplace<T>(static_cast<T*>(grad_Y), gy2, M * L2 * d, st);
    if (e == hipSuccess) e = sk::launch_mmd2_reduce<T>(Kxx, Kxy, Kyy, N * N, N * M, M * M, static_cast<T*>(loss), st);
    if (e != hipSuccess) return fail(SK_ERR_HIP, "mmd2 reduction: %s", hipGetErrorString(e));
    return SK_OK;
}
}  // namespace

extern "C" {

size_t sigkernel_mmd2_workspace_bytes(int64_t N, int64_t M, int64_t L1, int64_t L2, int64_t d, int lam1, int lam2,
                                      int flags, sk_dtype dt, int with_grads)
{
    if (N < 1 || M < 1 || (flags & (SK_FLAG_KEEP_FORWARD | SK_FLAG_HAVE_FORWARD)) ||
        validate(N, M, L1, L2, d, lam1, lam2, flags, (int)dt) != SK_OK)
        return 0;
    return mmd_layout(N, M, L1, L2, d, lam1, lam2, flags, dt, with_grads != 0).total;
}

int sigkernel_mmd2(const void* X, const void* Y, void* loss, void* grad_X, void* grad_Y, int64_t N, int64_t M,
                   int64_t L1, int64_t L2, int64_t d, int lam1, int lam2, int flags, sk_dtype dt, void* ws,
                   size_t ws_bytes, void* stream)
{
    // one call computes everything: there is no forward sweep to keep or to take over
    if (flags & (SK_FLAG_KEEP_FORWARD | SK_FLAG_HAVE_FORWARD))
        return fail(SK_ERR_DTYPE, "SK_FLAG_KEEP_FORWARD / SK_FLAG_HAVE_FORWARD do not apply to sigkernel_mmd2");
    int rc = validate(N, M, L1, L2, d, lam1, lam2, flags, (int)dt);
    if (rc != SK_OK) return rc;
    if (N < 1 || M < 1) return fail(SK_ERR_SHAPE, "mmd2 needs at least one path on either side");
    if (!X || !Y || !loss) return fail(SK_ERR_NULL, "X / Y / loss is NULL");
    if (X == Y) return fail(SK_ERR_SHAPE, "mmd2 of a set with itself is zero; pass two arrays");
    const bool grads = grad_X != nullptr || grad_Y != nullptr;
    const MmdLayout l = mmd_layout(N, M, L1, L2, d, lam1, lam2, flags, dt, grads);
    if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255) != 0)
        return fail(SK_ERR_WORKSPACE, "workspace pointer is NULL or not 256-byte aligned");
    if (ws_bytes < l.total) return fail(SK_ERR_WORKSPACE, "workspace has %zu bytes, %zu needed", ws_bytes, l.total);
    if (dt == SK_F64)
        return run_mmd2<double>(l, X, Y, loss, grad_X, grad_Y, N, M, L1, L2, d, lam1, lam2, flags, dt, ws, stream);
    return run_mmd2<float>(l, X, Y, loss, grad_X, grad_Y, N, M, L1, L2, d, lam1, lam2, flags, dt, ws, stream);
}

int sigkernel_event_timing(int enable)
{
    std::lock_guard<std::mutex> lk(g_timing_mu);
    g_timing_tag = enable;
    return SK_OK;
}

int sigkernel_event_timing_read_tag(int tag, double* fwd_ms, int* fwd_launches, double* bwd_ms, int* bwd_launches)
{
    std::vector<TimedLaunch> v;
    {
        std::lock_guard<std::mutex> lk(g_timing_mu);
        if (tag == 0) {
            v.swap(g_timed);
        } else {
            std::vector<TimedLaunch> rest;
            for (auto& t : g_timed) (t.tag == tag ? v : rest).push_back(t);
            g_timed.swap(rest);
        }
    }
    double ms[2] = {0.0, 0.0};
    int cnt[2] = {0, 0};
    int rc = SK_OK;
    for (auto& t : v) {
        hipError_t e = hipEventSynchronize(t.stop);
        float f = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&f, t.start, t.stop);
        if (e != hipSuccess) rc = fail(SK_ERR_HIP, "event timing: %s", hipGetErrorString(e));
        else { ms[t.backward] += f; cnt[t.backward] += 1; }
        (void)hipEventDestroy(t.start);
        (void)hipEventDestroy(t.stop);
    }
    if (fwd_ms) *fwd_ms = ms[0];
    if (fwd_launches) *fwd_launches = cnt[0];
    if (bwd_ms) *bwd_ms = ms[1];
    if (bwd_launches) *bwd_launches = cnt[1];
    return rc;
}

int sigkernel_event_timing_read(double* fwd_ms, int* fwd_launches, double* bwd_ms, int* bwd_launches)
{
    return sigkernel_event_timing_read_tag(0, fwd_ms, fwd_launches, bwd_ms, bwd_launches);
}

int sigkernel_describe(int op, int64_t B_or_N, int64_t M, int64_t L1, int64_t L2, int64_t d, int lam1, int lam2,
                       int flags, sk_dtype dt, char* out, size_t out_bytes)
{
    if (!out || out_bytes == 0) return fail(SK_ERR_NULL, "out is NULL or empty");
    out[0] = 0;
    if (op < SK_OP_FWD || op > SK_OP_GRAM_BWD) return fail(SK_ERR_SHAPE, "unknown operation %d", op);
    const bool gram = op == SK_OP_GRAM || op == SK_OP_GRAM_BWD;
    const bool backward = op == SK_OP_BWD || op == SK_OP_GRAM_BWD;
    const int64_t ny = gram ? M : B_or_N;
    int rc = validate(B_or_N, ny, L1, L2, d, lam1, lam2, flags, (int)dt);
    if (rc != SK_OK) return rc;
    Layout lay = make_layout(backward, gram, false, B_or_N, ny, L1, L2, d, lam1, lam2, flags, dt == SK_F64 ? 8 : 4,
                             !(flags & SK_FLAG_BWD_REPLAY));
    if (!lay.p.valid) {
        std::snprintf(out, out_bytes, "mode=trivial (no cells to sweep)");
        return SK_OK;
    }
    // a kept forward sweep: the two halves of the backward call, where the launch mode has them
    int phase = 0;
    if (flags & (backward ? SK_FLAG_HAVE_FORWARD : SK_FLAG_KEEP_FORWARD)) {
        const Layout lb = make_layout(true, gram, false, B_or_N, ny, L1, L2, d, lam1, lam2, flags, dt == SK_F64 ? 8 : 4,
                                      !(flags & SK_FLAG_BWD_REPLAY), true);
        if (lb.p.valid && split_forward(lb.p, dt)) {
            phase = backward ? 2 : 1;
            lay = lb;
        } else if (lb.p.valid) {
            lay.total = lb.total > lay.total ? lb.total : lay.total;   // the caller still brings the backward call's workspace
        }
    }
    const sk::Plan& p = lay.p;
    char kern[128];
    int threads;
    const char* mode;
    if (p.band) {
        mode = "band";
        // backward: two launches, the forward sweep with checkpoints and then the reverse sweep (the larger one)
        if (phase == 1) std::snprintf(kern, sizeof(kern), "band_fwd_kernel<%d, %d, true, %d>", p.BL, p.DT, p.ll);
        else if (phase == 2) std::snprintf(kern, sizeof(kern), "band_rev_kernel<%d, %d, %d>", p.BL, p.DT, p.ll);
        else if (backward)
            std::snprintf(kern, sizeof(kern), "band_fwd_kernel<%d, %d, true, %d>+band_rev_kernel<%d, %d, %d>", p.BL, p.DT,
                          p.ll, p.BL, p.DT, p.ll);
        else
            std::snprintf(kern, sizeof(kern), "band_fwd_kernel<%d, %d, false, %d>", p.BL, p.DT, p.ll);
        threads = (sk::kBandStrips + 1) * sk::kWave;
    } else if (p.quad) {
        mode = "quad";
        std::snprintf(kern, sizeof(kern), "quad_fwd_kernel<%d, %d, %d>", p.BL, p.DT, p.lk_M);
        threads = sk::kWavesPerWG * sk::kWave;
    } else if (p.tile) {
        mode = "tile";
        // (backward: the second argument says whether the sweeps move two columns per LDS instruction, sk_tile_bwd.hip)
        if (backward) std::snprintf(kern, sizeof(kern), "tile_bwd_kernel<%d, %s>", p.DT / 4, p.nb + 1 < sk::kTileCols - 1 ? "true" : "false");
        else std::snprintf(kern, sizeof(kern), "tile_fwd_kernel<%d>", p.DT / 4);
        threads = sk::kWavesPerWG * sk::kWave;
    } else if (p.solo) {
        mode = "solo";
        if (backward || phase)
            std::snprintf(kern, sizeof(kern), "solo_bwd_kernel<%d, %d, %d, %d, %d, %d>", p.BL, p.DT, p.lk_M, phase, p.ll,
                          sk::solo_bwd_shares_simd(p.BL, p.lk_M, p.DT, p.lds_bytes) ? 2 : 1);
        else std::snprintf(kern, sizeof(kern), "solo_fwd_kernel<%d, %d, %d, %d>", p.BL, p.DT, p.lk_M, p.ll);
        threads = sk::kWavesPerWG * sk::kWave;
    } else if (p.lock) {
        mode = "lock-step";
        if (backward || phase)
            std::snprintf(kern, sizeof(kern), "lock_bwd_kernel<%d, %d, %d, %d, %d>", p.BL, p.DT, p.lk_M, phase, p.ll);
        else std::snprintf(kern, sizeof(kern), "lock_fwd_kernel<%d, %d, %d, %d>", p.BL, p.DT, p.lk_M, p.ll);
        threads = (p.lk_ns == 1 ? 3 : (p.lk_ns == 2 ? 8 : 12)) * sk::kWave;
    } else {
        const char* base = !backward ? "sweep_fwd" : (p.uncompute ? "sweep_bwdu" : "sweep_bwd");
        mode = p.coop ? "cooperative" : "wave-per-pair";
        std::snprintf(kern, sizeof(kern), "%s%s_kernel<%d, %d, %s>", base, p.coop ? "_coop" : "", p.BL, p.DT,
                      (p.y_lds && p.DT) ? "true" : "false");
        threads = (p.coop ? p.nw : sk::kWavesPerWG) * sk::kWave;
    }
    const bool fused = p.lock && !gram && dt == SK_F64;
    std::snprintf(out, out_bytes,
                  "mode=%s kernel=%s grid=%d threads=%d lds_bytes=%zu strips=%d rows_per_lane=%d fused=%d "
                  "kept_sweep_half=%d lead_lag_form=%s second_launch_lds_bytes=%zu workspace_bytes=%zu "
                  "drifted_pairs_counter_at=%zu",
                  mode, kern, p.grid, threads, p.lds_bytes, (p.lock || p.solo || p.tile || p.quad || p.band) ? p.lk_ns : p.ns,
                  (p.lock || p.solo || p.tile || p.quad || p.band) ? p.lk_M : 1,
                  fused ? 1 : 0, phase, lay.ll ? "checkerboard" : "none",
                  (lay.has_sc && backward && phase != 1) ? lay.sc.lds_bytes : (size_t)0, lay.total, p.off_badlist != 0 ? p.off_badcnt : (size_t)0);
    return SK_OK;
}

// ---------------------------------------------------------------- truncated signatures (signature.h)
}  // extern "C"

namespace {

int sig_validate(int64_t B, int64_t L, int64_t d, int N, int flags, int dt, sg::Plan* plan, bool backward = false,
                 bool have_sig = false)
{
    if (dt != SK_F32 && dt != SK_F64) return fail(SK_ERR_DTYPE, "dtype %d is neither SK_F32 nor SK_F64", dt);
    if (flags & ~(SK_FLAG_TIME_AUG | SK_FLAG_LEAD_LAG | SK_SIG_DEPTH_MASK)) return fail(SK_ERR_DTYPE, "unknown flag bits 0x%x", flags);
    const int force_M = ((flags & 0xf00) >> 8) - 1;
    const int force_S = (flags & 0xf000) >> 12;
    const int split = (flags & 0x1f0000) >> 16;          // SK_SIG_PIECES(log2 P) = (log2 P + 1) << 16
    const int force_P = split ? (1 << (split - 1)) : 0;
    if (split > 11) return fail(SK_ERR_SHAPE, "at most 2^10 pieces per path");
    if (B < 0) return fail(SK_ERR_SHAPE, "negative batch size");
    if (L < 1 || d < 1 || N < 1) return fail(SK_ERR_SHAPE, "need L, d, N >= 1 (got %lld, %lld, %d)", (long long)L,
                                             (long long)d, N);
    if (L > ((int64_t)1 << 29) || d > 32768 || N > 64 || B > ((int64_t)1 << 40))
        return fail(SK_ERR_SHAPE, "L above 2^29, d above 32768, N above 64 or B above 2^40");
    *plan = sg::make_plan(B, L, d, N, (flags & SK_FLAG_TIME_AUG) != 0, (flags & SK_FLAG_LEAD_LAG) != 0, dt == SK_F64,
                          force_M, backward, have_sig, force_S, force_P,
                          (flags & SK_SIG_ONE_PATH_PER_WAVE) ? 1 : 0);
    if (!plan->valid) return fail(SK_ERR_SHAPE, "%s: %s", backward ? "signature_bwd" : "signature_fwd", plan->why);
    return SK_OK;
}

template <typename T>
int run_signature(const sg::Plan& p, const void* x, void* out, int flags, void* ws, hipStream_t st)
{
    constexpr bool kIsDouble = sizeof(T) == 8;
    unsigned char* base = static_cast<unsigned char*>(ws);
    hipError_t e;
#define SK_CHECK(call)                                                                         \
    do {                                                                                       \
        e = (call);                                                                            \
        if (e != hipSuccess) return fail(SK_ERR_HIP, "%s: %s", #call, hipGetErrorString(e));   \
    } while (0)
    double* dz = reinterpret_cast<double*>(base + p.off_dz);
    SK_CHECK(sg::launch_increments<T>(static_cast<const T*>(x), dz, p.B, p.L, p.d, p.D, p.Dpad, p.n, p.P, p.Lc, p.np,
                                      (flags & SK_FLAG_TIME_AUG) ? 1 : 0, (flags & SK_FLAG_LEAD_LAG) ? 1 : 0, st));
    double* result = kIsDouble ? static_cast<double*>(out) : reinterpret_cast<double*>(base + p.off_out);
    sg::Args a;
    a.dz = dz;
    a.out = p.P > 1 ? reinterpret_cast<double*>(base + p.off_t0) : result;
    a.B = p.VB; a.n = p.Lc; a.np = p.np; a.D = p.D; a.Dpad = p.Dpad; a.N = p.N; a.Q = p.Q; a.NB = p.NB;
    a.LP = p.LP; a.WP = p.WP; a.sig_len = p.sig_len; a.PW = p.PW; a.NW = p.waves;
    a.leadlag = (flags & SK_FLAG_LEAD_LAG) ? 1 : 0;
    const int ttag = timing_tag();
    EventPair ev;
    if (ttag) SK_CHECK(ev.begin(0, ttag, st));
    SK_CHECK(sg::launch_horner(p.DT, p.M, p.S, a, p.grid, st));
    if (p.P > 1) {
        // the signatures of the pieces, multiplied pairwise until one per path is left (Chen's identity)
        double* t0 = reinterpret_cast<double*>(base + p.off_t0);
        double* t1 = reinterpret_cast<double*>(base + p.off_t1);
        const double* src = t0;
        for (int cur = p.P; cur > 1; cur /= 2) {
            double* dst = cur == 2 ? result : (src == t0 ? t1 : t0);
            SK_CHECK(sg::launch_chen_pairs(src, dst, p.B * (cur / 2), p.D, p.N, p.sig_len, st));
            src = dst;
        }
    }
    if (ttag) SK_CHECK(ev.end(st));
    if (!kIsDouble) SK_CHECK((sk::launch_convert<double, T>(result, static_cast<T*>(out), p.B * p.sig_len, st)));
#undef SK_CHECK
    return SK_OK;
}

// grad_x from the signatures and the upstream gradient.  The forward plan `pf` is used when the signatures have to be
// computed first (into the backward workspace).
template <typename T>
int run_signature_bwd(const sg::Plan& p, const sg::Plan& pf, const void* x, const void* sig, const void* grad_out,
                      void* grad_x, int flags, void* ws, hipStream_t st)
{
    constexpr bool kIsDouble = sizeof(T) == 8;
    unsigned char* base = static_cast<unsigned char*>(ws);
    hipError_t e;
#define SK_CHECK(call)                                                                         \
    do {                                                                                       \
        e = (call);                                                                            \
        if (e != hipSuccess) return fail(SK_ERR_HIP, "%s: %s", #call, hipGetErrorString(e));   \
    } while (0)
    double* dz = reinterpret_cast<double*>(base + p.off_dz);
    double* gz = reinterpret_cast<double*>(base + p.off_gz);
    const long count = p.B * p.sig_len;
    SK_CHECK(sg::launch_increments<T>(static_cast<const T*>(x), dz, p.B, p.L, p.d, p.D, p.Dpad, p.n, p.P, p.Lc, p.np,
                                      (flags & SK_FLAG_TIME_AUG) ? 1 : 0, (flags & SK_FLAG_LEAD_LAG) ? 1 : 0, st));
    SK_CHECK(sk::launch_fill<double>(gz, p.VB * p.np * p.Dpad, 0.0, st));
    const double* gout64;
    if (kIsDouble) {
        gout64 = static_cast<const double*>(grad_out);
    } else {
        double* g64 = reinterpret_cast<double*>(base + p.off_gout);
        SK_CHECK((sk::launch_convert<T, double>(static_cast<const T*>(grad_out), g64, count, st)));
        gout64 = g64;
    }
    const int ttag = timing_tag();
    const bool timed = ttag != 0;
    EventPair ev;
    auto forward_args = [&](double* out) {
        sg::Args f;
        f.dz = dz;
        f.out = out;
        f.B = pf.VB; f.n = pf.Lc; f.np = pf.np; f.D = pf.D; f.Dpad = pf.Dpad; f.N = pf.N; f.Q = pf.Q; f.NB = pf.NB;
        f.LP = pf.LP; f.WP = pf.WP; f.sig_len = pf.sig_len; f.PW = pf.PW; f.NW = pf.waves;
        f.leadlag = (flags & SK_FLAG_LEAD_LAG) ? 1 : 0;
        return f;
    };
    const double* sig64;
    if (p.P > 1) {
        // Paths cut into pieces: signatures of the pieces (level 0 of a tree), products of neighbouring pairs level by
        // level up to the whole paths, then the adjoints back down; the backward kernel then sees the pieces as paths
        // with their own signatures and upstream gradients.  Signatures the caller passed are not used.
        if (timed) SK_CHECK(ev.begin(1, ttag, st));
        double* tv = reinterpret_cast<double*>(base + p.off_t0);
        double* ta = reinterpret_cast<double*>(base + p.off_t1);
        sg::Args f = forward_args(tv);
        SK_CHECK(sg::launch_horner(pf.DT, pf.M, pf.S, f, pf.grid, st));
        // level j holds P >> j signatures per path, starting at lev[j] signatures into the tree buffers
        long lev[16];
        int nlev = 0;
        {
            long o = 0;
            for (int cur = p.P; cur > 1; cur /= 2) {
                lev[nlev++] = o;
                o += p.B * cur;
            }
        }
        for (int j = 0; j + 1 < nlev; ++j)      // the product of all pieces is not needed: its adjoint is grad_out
            SK_CHECK(sg::launch_chen_pairs(tv + lev[j] * p.sig_len, tv + lev[j + 1] * p.sig_len, p.B * (p.P >> (j + 1)), p.D,
                                           p.N, p.sig_len, st));
        for (int j = nlev - 1; j >= 0; --j) {
            const double* parent = j == nlev - 1 ? gout64 : ta + lev[j + 1] * p.sig_len;
            SK_CHECK(sg::launch_chen_pairs_adjoint(tv + lev[j] * p.sig_len, parent, ta + lev[j] * p.sig_len,
                                                   p.B * (p.P >> (j + 1)), p.D, p.N, p.sig_len, st));
        }
        sig64 = tv;
        gout64 = ta;
    } else if (!sig) {
        sg::Args f = forward_args(reinterpret_cast<double*>(base + p.off_sig));
        SK_CHECK(sg::launch_horner(pf.DT, pf.M, pf.S, f, pf.grid, st));
        sig64 = f.out;
    } else if (kIsDouble) {
        sig64 = static_cast<const double*>(sig);
    } else {
        double* s64 = reinterpret_cast<double*>(base + p.off_sig);
        SK_CHECK((sk::launch_convert<T, double>(static_cast<const T*>(sig), s64, count, st)));
        sig64 = s64;
    }
    sg::BwdArgs a;
    a.dz = dz; a.gz = gz; a.sig = sig64; a.gout = gout64;
    a.B = p.VB; a.n = p.Lc; a.np = p.np; a.D = p.D; a.Dpad = p.Dpad; a.N = p.N; a.Q = p.Q; a.NB = p.NB;
    a.LP = p.LP; a.WP = p.WP; a.sig_len = p.sig_len; a.lds_wave = p.lds_wave; a.PW = p.PW; a.NW = p.waves;
    a.leadlag = (flags & SK_FLAG_LEAD_LAG) ? 1 : 0;
    if (timed && p.P == 1) SK_CHECK(ev.begin(1, ttag, st));
    SK_CHECK(sg::launch_horner_bwd(p.DT, p.M, p.S, a, p.grid, p.lds_bytes, st));
    if (timed) SK_CHECK(ev.end(st));
    SK_CHECK(sg::launch_point_gradients<T>(gz, static_cast<T*>(grad_x), p.B, p.L, p.d, p.Dpad, p.P, p.Lc, p.np,
                                           (flags & SK_FLAG_LEAD_LAG) ? 1 : 0, st));
#undef SK_CHECK
    return SK_OK;
}

}  // namespace

extern "C" {

int64_t signature_length(int64_t d, int N, int flags)
{
    if (d < 1 || d > 32768 || N < 1 || (flags & ~(SK_FLAG_TIME_AUG | SK_FLAG_LEAD_LAG | SK_SIG_DEPTH_MASK))) return 0;
    const int64_t D = ((flags & SK_FLAG_LEAD_LAG) ? 2 * d : d) + ((flags & SK_FLAG_TIME_AUG) ? 1 : 0);
    return sg::sig_length(D, N);
}

size_t signature_workspace_bytes(int64_t B, int64_t L, int64_t d, int N, int flags, sk_dtype dt)
{
    sg::Plan p;
    if (sig_validate(B, L, d, N, flags, (int)dt, &p) != SK_OK || B == 0) return 0;
    return p.total;
}

int signature_fwd(const void* x, void* out, int64_t B, int64_t L, int64_t d, int N, int flags, sk_dtype dt, void* ws,
                  size_t ws_bytes, void* stream)
{
    sg::Plan p;
    int rc = sig_validate(B, L, d, N, flags, (int)dt, &p);
    if (rc != SK_OK) return rc;
    if (B == 0) return SK_OK;
    if (!x || !out) return fail(SK_ERR_NULL, "x or out is NULL");
    if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255) || ws_bytes < p.total)
        return fail(SK_ERR_WORKSPACE, "workspace is NULL, misaligned or smaller than %zu bytes", p.total);
    hipStream_t st = static_cast<hipStream_t>(stream);
    return dt == SK_F64 ? run_signature<double>(p, x, out, flags, ws, st) : run_signature<float>(p, x, out, flags, ws, st);
}

size_t signature_bwd_workspace_bytes(int64_t B, int64_t L, int64_t d, int N, int flags, sk_dtype dt, int have_sig)
{
    sg::Plan p;
    if (sig_validate(B, L, d, N, flags, (int)dt, &p, true, have_sig != 0) != SK_OK || B == 0) return 0;
    return p.total;
}

int signature_bwd(const void* x, const void* sig, const void* grad_out, void* grad_x, int64_t B, int64_t L, int64_t d,
                  int N, int flags, sk_dtype dt, void* ws, size_t ws_bytes, void* stream)
{
    sg::Plan p, pf;
    int rc = sig_validate(B, L, d, N, flags, (int)dt, &p, true, sig != nullptr);
    if (rc != SK_OK) return rc;
    if (B == 0) return SK_OK;
    if (!x || !grad_out || !grad_x) return fail(SK_ERR_NULL, "x, grad_out or grad_x is NULL");
    if (!sig || p.P > 1) {
        // the forward launch for the same paths, cut into the same pieces, its output in double whatever the caller's
        // type; a forced subtree depth applies to the backward kernel only
        int q = 0;
        while ((1 << q) < p.P) ++q;
        rc = sig_validate(B, L, d, N, (flags & (SK_FLAG_TIME_AUG | SK_FLAG_LEAD_LAG | SK_SIG_ONE_PATH_PER_WAVE)) | SK_SIG_PIECES(q),
                          SK_F64, &pf);
        if (rc != SK_OK) return rc;
        if (pf.P != p.P || pf.Lc != p.Lc || pf.np != p.np || pf.Dpad != p.Dpad)
            return fail(SK_ERR_SHAPE, "signature_bwd: forward and backward plans disagree on the pieces");
    }
    if (!ws || (reinterpret_cast<uintptr_t>(ws) & 255) || ws_bytes < p.total)
        return fail(SK_ERR_WORKSPACE, "workspace is NULL, misaligned or smaller than %zu bytes", p.total);
    hipStream_t st = static_cast<hipStream_t>(stream);
    return dt == SK_F64 ? run_signature_bwd<double>(p, pf, x, sig, grad_out, grad_x, flags, ws, st)
                        : run_signature_bwd<float>(p, pf, x, sig, grad_out, grad_x, flags, ws, st);
}

int signature_bwd_describe(int64_t B, int64_t L, int64_t d, int N, int flags, sk_dtype dt, char* out, size_t out_bytes)
{
    if (!out || out_bytes == 0) return fail(SK_ERR_NULL, "out is NULL or empty");
    out[0] = 0;
    sg::Plan p;
    int rc = sig_validate(B, L, d, N, flags, (int)dt, &p, true, true);
    if (rc != SK_OK) return rc;
    std::snprintf(out, out_bytes,
                  "kernel=horner_bwd_kernel<%d, %d, %d, %d, %s, %s> channels=%d prefix_letters=%d letter_blocks=%d "
                  "lanes_per_path=%lld waves_per_path=%lld paths_per_wave=%d pieces_per_path=%d segments_per_piece=%lld "
                  "grid=%lld threads=%d lds_bytes=%zu entries_per_path=%lld workspace_bytes=%zu",
                  p.DT, p.M, p.S, p.Q <= sg::kQExact ? p.Q : sg::kQMax, p.PW > 1 ? "true" : "false",
                  ((flags & SK_FLAG_LEAD_LAG) && p.DT >= 4 && p.M >= 1) ? "true" : "false", p.D, p.Q, p.NB,
                  (long long)p.LP, (long long)p.WP, p.PW, p.P, (long long)p.Lc, (long long)p.grid, sg::kWave * sg::kWavesPerWG, p.lds_bytes, (long long)p.sig_len,
                  B == 0 ? (size_t)0 : p.total);
    return SK_OK;
}

int signature_describe(int64_t B, int64_t L, int64_t d, int N, int flags, sk_dtype dt, char* out, size_t out_bytes)
{
    if (!out || out_bytes == 0) return fail(SK_ERR_NULL, "out is NULL or empty");
    out[0] = 0;
    sg::Plan p;
    int rc = sig_validate(B, L, d, N, flags, (int)dt, &p);
    if (rc != SK_OK) return rc;
    std::snprintf(out, out_bytes,
                  "kernel=horner_kernel<%d, %d, %d, %d, %s, %s> channels=%d prefix_letters=%d letter_blocks=%d lanes_per_path=%lld "
                  "waves_per_path=%lld paths_per_wave=%d pieces_per_path=%d segments_per_piece=%lld grid=%lld threads=%d "
                  "entries_per_path=%lld workspace_bytes=%zu",
                  p.DT, p.M, p.S, p.Q <= sg::kQExact ? p.Q : sg::kQMax, p.PW > 1 ? "true" : "false",
                  ((flags & SK_FLAG_LEAD_LAG) && p.DT >= 4 && p.M >= 1) ? "true" : "false", p.D, p.Q, p.NB,
                  (long long)p.LP, (long long)p.WP, p.PW, p.P, (long long)p.Lc, (long long)p.grid, sg::kWave * sg::kWavesPerWG, (long long)p.sig_len,
                  B == 0 ? (size_t)0 : p.total);
    return SK_OK;
}

const char* sigkernel_last_error(void) { return g_err; }

const char* sigkernel_version(void) { return "sigkernel-mi355x 0.1 (gfx950)"; }

}  // extern "C"

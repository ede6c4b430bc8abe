// Host-side launch plan for the signature-kernel sweeps: pure arithmetic, no HIP calls, so that the
// workspace query and the launches agree by construction.
//
// Geometry (paper Section 3.1/3.2): the refined grid has m = (L1-1) << lam1 by n = (L2-1) << lam2 cells.
// The sweep works on square blocks of 2^BL x 2^BL refined cells that share one entry of the increment
// Gram matrix (BL = min(lam1, lam2, 2)); the block grid has mb = (L1-1) << rs1 rows and
// nb = (L2-1) << rs2 columns, rs = lam - BL.  A strip is 64 consecutive block rows, one per lane.
#pragma once
#include <cstddef>
#include <cstdint>

namespace sk {

constexpr int kWave = 64;
constexpr int kWavesPerWG = 4;            // waves (independent pairs) per workgroup
constexpr size_t kLdsPerCU = 160 * 1024;  // gfx950: 160 KB of LDS per compute unit / workgroup
constexpr size_t kLdsPerWave = kLdsPerCU / kWavesPerWG - 1024;
constexpr int kNumCU = 256;
constexpr int kMaxBL = 2;

// Channel counts with a dedicated kernel instantiation (increments kept in registers).
constexpr int kTemplD[] = {2, 3, 4, 5, 6, 8, 16};

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct Plan {
    bool valid = false;
    bool backward = false;
    bool symmetric = false;     // Gram with Y == X: one increment buffer, one gradient accumulator
    int elem = 8;               // bytes per element of every internal buffer (sweeps run in double)
    int io_elem = 8;            // bytes per element of the caller's arrays
    int64_t nx = 0, ny = 0;     // number of x paths and y paths
    int64_t npairs = 0;         // pairs the sweep launch works through
    int64_t kcount = 0;         // entries of k / K (differs from npairs only for tri)
    int tri = 0;                // symmetric Gram matrix in solo / tile mode: only the pairs n <= m are solved
    int64_t gramM = 0;          // > 0: pair id -> (id / gramM, id % gramM); 0: pair id -> (id, id)
    int L1 = 0, L2 = 0, d = 0;
    int BL = 0, rs1 = 0, rs2 = 0;
    int r = 0, q = 0;           // coarse cells per side
    int rpad = 0, qpad = 0;
    int mb = 0, nb = 0;         // block rows / columns
    int ns = 0;                 // strips per pair
    int rowlen = 0;             // elements of one boundary row (node columns, padded)
    int DT = 0;                 // kernel template channel count (0 = runtime loop over d)
    int DP = 0;                 // channels stored per increment row (d padded to the kernel's count)
    int S = 0, nseg = 0;        // backward: macro-steps per replay segment, segments per strip
    int y_lds = 0;              // y increments (and their gradient accumulators) staged in LDS
    size_t lds_wave = 0, lds_bytes = 0, ring_off = 0;
    int grid = 0;
    int64_t nslots = 0;
    int64_t xstride = 0, ystride = 0, rows_slot = 0, ckpt_slot = 0, adj_slot = 0;
    size_t off_dxT = 0, off_dyT = 0, off_gdxT = 0, off_gdyT = 0, off_rows = 0, off_adj = 0, off_ckpt = 0;
    size_t off_kio = 0, off_gkio = 0;   // float callers: double staging of k and grad_k
    size_t off_keep_tag = 0;
    int keep_solo = 0;                  // solo backward plan with per-pair checkpoints and bottom rows
    int64_t keep_len = 0;               // doubles per kept bottom row (solo)
    size_t off_keep = 0;                // backward: what a kept forward sweep leaves besides rows and checkpoints
                                        // (lock-step: the hand-over rows; band: the kernel values)
    size_t off_err = 0;                 // one int: a bounded wait between cooperating waves ran out
    size_t total = 0;
    // cooperative mode: one workgroup per pair, its strips pipelined over nw waves
    int coop = 0, nw = 0, RB = 0, CH = 0;
    int uncompute = 0;   // backward: reverse sweep recovers forward values by inverting Eq. (1) (no replay ring)
    size_t coop_off_gdy = 0, coop_off_flags = 0, coop_off_obox = 0, coop_off_ring = 0, coop_ring_stride = 0;
    // lock-step mode: one workgroup per pair, per strip one stencil wave and one coefficient wave
    int band = 0, bd_nbands = 0;   // bands of kBandStrips strips on different compute units (sk_band.hip)
    size_t bd_off_y = 0, bd_off_gy = 0, bd_off_rings = 0, off_flags = 0;
    int nflags = 0;
    // Pairs whose inverse recurrence drifted are listed here by the reverse sweep and solved once more by the replay
    // kernel (sk_api.hip): a counter (the int behind the progress counters, cleared with them) and the pair ids.
    size_t off_badcnt = 0, off_badlist = 0;
    int ll = 0;     // lead-lag form of the sweep: 0 none, 1 the level lies inside a block, 2 above the blocks
    int tile = 0;   // one wave per pair, at most 64 x 64 cells, contractions on the matrix cores (sk_tile.hip)
    int quad = 0;   // four pairs per wave, forward Gram calls on the tile kernels' shapes (sk_quad.hip)
    int64_t nquads = 0;   // groups of four pairs of one Gram row the quad launch works through
    int solo = 0;   // one wave per pair, a single strip of 64 * lk_M block rows (many pairs of short paths)
    int lock = 0, lk_M = 0, lk_ns = 0, lk_NT = 0, lk_padb = 0, lk_rowlen = 0;
    size_t lk_off_y = 0, lk_off_gy = 0, lk_off_cring = 0, lk_off_gp = 0, lk_off_krows = 0, lk_off_arows = 0,
           lk_off_dump = 0, lk_cring_stride = 0, lk_gp_stride = 0, lk_off_ck = 0, lk_ck_stride = 0, lk_off_gyp = 0;
};

// Lock-step mode constants: chunk lengths (macro-steps between workgroup barriers) of the forward and the
// reverse sweep, checkpoint spacing, and the lag between consecutive strips.  A value written to a hand-over
// row in one chunk is read by the neighbouring strip in a later chunk if lag >= 63 + chunk.
constexpr int kLockCH1 = 8, kLockCH2 = 4, kLockS = 8;
constexpr int kLockLag1 = 72, kLockLag2 = 68;
constexpr int kLockMaxStrips = 4;      // forward: a stencil and a coefficient wave per strip
constexpr int kLockMaxStripsBwd = 2;   // backward: plus a gradient wave per strip

// Block rows per lane the lock-step kernels are built for: two, unless the lane state would not fit the
// register file (largest blocks or most channels in the backward kernel; both together in the forward one);
// zero: no lock-step kernel for this combination.
constexpr int lock_max_rows(bool backward, int BL, int DT)
{
    if (DT == 0) return 0;
    if (backward) return (BL >= 2 && DT >= 16) ? 0 : ((BL >= 2 || DT >= 16) ? 1 : 2);
    return (BL >= 2 && DT >= 16) ? 1 : 2;
}

// Block rows per lane of the solo kernels (one wave does the stencil, the coefficients and the gradients).
constexpr int solo_max_rows(bool backward, int BL, int DT)
{
    if (DT == 0) return 0;
    if (backward) return ((BL <= 1 && DT <= 8) || DT <= 4) ? 2 : 1;
    return (BL >= 2 && DT >= 16) ? 1 : 2;
}

// Wavefronts per SIMD the solo backward kernel is built for: two, or one where the lane state of two block rows of
// 4 x 4 cells, or the sums and increments of sixteen channels, need the whole register file (accumulation registers
// included: with 256 registers the sixteen-channel kernels spill a kilobyte per lane and run four times slower).
constexpr int solo_bwd_waves_per_simd(int BL, int M, int DT)
{
    return ((BL >= 2 && M >= 2) || DT >= 16 || (DT >= 8 && (M >= 2 || BL >= 2))) ? 1 : 2;
}
// Whether a launch of the solo backward kernel puts two workgroups on a compute unit (lds: bytes per workgroup); if
// not, the kernel's one-wave build is launched, which has the whole register file.
constexpr bool solo_bwd_shares_simd(int BL, int M, int DT, size_t lds)
{
    return solo_bwd_waves_per_simd(BL, M, DT) >= 2 && 2 * lds <= kLdsPerCU;
}

// Tile mode: the increment Gram matrix of a pair as a 64 x 64 array of doubles in LDS, column stride
// kTileStride (even, not a multiple of 4: row-contiguous, skewed and transposed accesses all stay at most
// two-way bank conflicted), kTileCols columns (-1 .. 64: a zero guard column on either side).
constexpr int kTileStride = 66, kTileCols = 66;
// Quad mode: a wavefront works on four pairs that share the y path, 16 lanes with four or eight block rows each.
constexpr int kQuadPairs = 4;
// Block rows per lane the quad kernel is built for (0: none): blocks of at most 2 x 2 cells, and the increments of a
// lane's rows in at most 128 registers.
constexpr int quad_max_rows(int BL, int DT)
{
    if (BL > 1 || DT == 0) return 0;
    if (DT == 16) return BL == 0 ? 4 : 0;
    return DT == 8 ? 4 : 8;
}
// Row stride of the y copy in LDS (doubles): for an even channel count a multiple of 16 bytes that spreads the
// 16-byte reads of lanes at consecutive rows over the banks; an odd count does that by itself.
constexpr int quad_y_stride(int DT) { return DT % 2 ? DT : (DT == 6 ? 10 : DT + 2); }
constexpr int kTileRowPad = 8;     // backward: node columns kept left of column 0 in the pair's bottom row (all 1)
constexpr int kTileCkChunks = 8;   // backward: chunks of 8 macro-steps between two checkpoints (kept in LDS)

// Band mode: strips per workgroup, block columns per hand-over ring, coarse y columns per y ring (powers of
// two), chunks the data-moving wave works ahead, and the bound on its polls of another workgroup's counter.
constexpr int kBandStrips = 4, kBandRing = 64, kBandYRing = 512, kBandLead = 2, kBandSpin = 1 << 22, kBandSlack = 8, kBandLeadRev = 3;

// Band mode takes over from three strips on (a single band then: measured a little ahead of the cooperative kernels).
constexpr int kBandMinStrips = 2;
constexpr int64_t kCoopMaxPairs = 1024;   // above this, one wave per pair already fills the chip

constexpr int kUncomputeS = 8;   // macro-steps between checkpoints when the reverse sweep inverts Eq. (1)
constexpr size_t kSecondChanceBytes = (size_t)8 << 20;   // scratch of the launch that solves drifted pairs once more
// A recovered forward value may differ from the exact checkpoint by this fraction of the lane's largest forward
// value; beyond it the pair is solved once more by the replay kernel.  Measured: on Brownian-like paths (the
// benchmark configurations) the differences stay below 3e-12 (a tolerance of 1e-12 already sends such pairs to
// the replay kernel) and the gradients agree with the reference to a few 1e-13; on paths with a few increments of
// order one a pair that passes can lose accuracy where its kernel values cancel (seen: 1.6e-10 of the gradient's
// largest entry, against 3e-12 from the replay kernel).  SK_FLAG_BWD_REPLAY is the choice for such data.
constexpr double kDriftTol = 1e-11;

inline Plan make_plan(bool backward, bool gram, bool symmetric, int64_t nx, int64_t ny, int64_t L1, int64_t L2,
                      int64_t d, int lam1, int lam2, int io_elem, bool uncompute = true, bool keep = false,
                      bool second_chance = false, bool lead_lag = false)
{
    // lead_lag: the sweep of two lead-lag paths (Section 4) on the grid of the original increments; lam1 and lam2 then
    // count the lead-lag level as one more dyadic level (the caller's orders plus one), L1, L2 and d are the caller's.
    // The level lies inside the blocks when these hold every refined cell of a pair of increments, above them
    // otherwise (Plan::ll); the tile kernels have no such form.
    // second_chance: the plan of the launch that solves the listed pairs once more (wave-per-pair replay kernel,
    // a bounded number of waves, no increment and accumulator areas of its own: it works on the main plan's).
    // keep: a backward plan whose forward sweep may be a launch of its own (a forward call that keeps its sweep for
    // the backward call).  Lock-step and band plans are laid out for that anyway; solo plans then get checkpoints and
    // a bottom row per pair instead of per wave.
    Plan p;
    p.uncompute = backward && uncompute;
    const int elem = 8;
    p.io_elem = io_elem;
    p.backward = backward;
    p.symmetric = symmetric;
    p.elem = elem;
    p.nx = nx;
    p.ny = ny;
    p.npairs = gram ? nx * ny : nx;
    p.kcount = p.npairs;
    p.gramM = gram ? ny : 0;
    p.L1 = (int)L1; p.L2 = (int)L2; p.d = (int)d;
    p.r = (int)L1 - 1; p.q = (int)L2 - 1;
    if (p.npairs <= 0 || p.r <= 0 || p.q <= 0) return p;   // nothing to sweep
    int mn = lam1 < lam2 ? lam1 : lam2;
    if (lead_lag) {
        if (mn < 1) return p;   // not valid: the lead-lag level counts as one dyadic level on either side
        // With unequal orders the blocks stay below the lead-lag level on both sides (a block then lies inside one
        // quadrant of that level, whichever side is refined more).
        if (lam1 != lam2) mn -= 1;
    }
    p.BL = mn < kMaxBL ? mn : kMaxBL;
    p.rs1 = lam1 - p.BL; p.rs2 = lam2 - p.BL;
    p.mb = p.r << p.rs1; p.nb = p.q << p.rs2;
    if (lead_lag) p.ll = (p.rs1 == 0 && p.rs2 == 0) ? 1 : 2;
    p.ns = (p.mb + kWave - 1) / kWave;
    const int C = 1 << p.BL, R = C;
    p.rowlen = (int)align_up((size_t)(p.nb + 8) * C + 1, 64);   // a few block columns beyond the grid (band mode)
    p.rpad = (int)align_up((size_t)p.r, 64);
    p.qpad = (int)align_up((size_t)p.q, 64);
    p.DT = 0;
    for (int t : kTemplD) if (d <= t) { p.DT = t; break; }
    p.DP = p.DT ? (p.DT | 1) : (int)d;   // odd row stride: LDS bank spread (see Sweep::DSc)
    p.xstride = (int64_t)p.DP * p.rpad;
    p.ystride = (int64_t)p.DP * p.qpad;

    const int NVR = R + C + 1;   // block input edges kept per macro-step in the ring
    const size_t ring_step = (size_t)kWave * NVR * elem;
    p.coop = (p.ns >= 2 && p.npairs <= kCoopMaxPairs && !second_chance) ? 1 : 0;
    if (p.coop) {
        // Workgroup-shared LDS: y (+ gradient accumulators), flags, ones/zeros/outbox rings; then one replay
        // ring per wave.
        const int maxw = (backward && p.BL == 2) ? 4 : 8;
        p.nw = p.ns < maxw ? p.ns : maxw;
        // Outbox rings long enough for a whole row need no back-pressure; otherwise 32 columns (set below).
        p.CH = 8;
        const int CW = backward ? 2 * C : C;   // values per column in the hand-over rings
        {
            int full = 32;
            while (full < p.nb + 1) full <<= 1;
            p.RB = ((size_t)(2 * p.nw + 2) * full * CW * elem <= 40 * 1024) ? full : 32;
        }
        const size_t ycopy = (size_t)p.q * p.DP * elem;
        const size_t fixed = 512 + (size_t)(2 * p.nw + 2) * p.RB * CW * elem;
        const size_t budget = kLdsPerCU - 1024;
        const size_t ring_min = (backward && !p.uncompute) ? (size_t)p.nw * 4 * ring_step : 0;
        const size_t yneed = ycopy * (backward ? 2 : 1);
        p.y_lds = (p.DT != 0 && align_up(yneed, 256) + fixed + ring_min <= budget) ? 1 : 0;
        size_t used = p.y_lds ? align_up(ycopy, 256) : 0;
        p.coop_off_gdy = used;
        if (p.y_lds && backward) used += align_up(ycopy, 256);
        p.coop_off_flags = used;
        used += 512;
        p.coop_off_obox = used;   // ones, zeros, nw outboxes, nw staging rings
        used += (size_t)(2 * p.nw + 2) * p.RB * CW * elem;
        used = align_up(used, 256);
        p.coop_off_ring = used;
        if (backward && p.uncompute) {
            p.S = kUncomputeS;
            p.nseg = (p.nb + kWave - 1 + p.S - 1) / p.S;
        } else if (backward) {
            int S = 64;
            while (S > 4 && used + (size_t)p.nw * S * ring_step > budget) S >>= 1;
            p.S = S;
            p.nseg = (p.nb + kWave - 1 + S - 1) / S;
            p.coop_ring_stride = (size_t)S * ring_step;
            used += (size_t)p.nw * p.coop_ring_stride;
        }
        p.lds_wave = 0;
        p.lds_bytes = align_up(used, 256);
        int wg_per_cu = (int)(kLdsPerCU / p.lds_bytes);
        if (wg_per_cu < 1) wg_per_cu = 1;
        if (wg_per_cu * p.nw > 8) wg_per_cu = 8 / p.nw > 0 ? 8 / p.nw : 1;
        int64_t cap = (int64_t)kNumCU * wg_per_cu;
        p.grid = (int)(p.npairs < cap ? p.npairs : cap);
        p.nslots = p.grid;
    } else {
        // LDS per wave: y increments (+ their gradient accumulators when going backward) and the replay ring.
        size_t ybytes = (size_t)p.DP * p.qpad * elem * (backward ? 2 : 1);
        p.y_lds = (p.DT != 0 && ybytes <= kLdsPerWave) ? 1 : 0;   // up to a whole compute unit for four waves
        size_t used = p.y_lds ? ybytes : 0;
        p.ring_off = used;
        if (backward && p.uncompute) {
            p.S = kUncomputeS;
            p.nseg = (p.nb + kWave - 1 + p.S - 1) / p.S;
        } else if (backward) {
            auto fit = [&](size_t before) {
                int S = 64;
                while (S > 4 && before + (size_t)S * ring_step > kLdsPerWave) S >>= 1;
                return S;
            };
            int S = fit(used);
            if (used + (size_t)S * ring_step > kLdsPerWave) {
                // not even the shortest ring fits next to the y increments: these stay in global memory
                p.y_lds = 0;
                used = 0;
                p.ring_off = 0;
                S = fit(0);
            }
            p.S = S;
            p.nseg = (p.nb + kWave - 1 + S - 1) / S;   // strips run nb + (lanes-1) macro-steps at most
            used += (size_t)S * ring_step;
        }
        p.lds_wave = align_up(used, 256);
        p.lds_bytes = p.lds_wave * kWavesPerWG;

        int wg_per_cu = (int)(kLdsPerCU / (p.lds_bytes ? p.lds_bytes : 1));
        if (wg_per_cu < 1) wg_per_cu = 1;
        if (wg_per_cu > 4) wg_per_cu = 4;
        if (backward && wg_per_cu > 2) wg_per_cu = 2;   // register file: the backward kernels run 2 waves per SIMD at most
        int64_t want = (p.npairs + kWavesPerWG - 1) / kWavesPerWG;
        int64_t cap = (int64_t)kNumCU * wg_per_cu;
        if (second_chance && cap > kNumCU) cap = kNumCU;
        p.grid = (int)(want < cap ? want : cap);
        p.nslots = (int64_t)p.grid * kWavesPerWG;
    }
    if (second_chance) {
        // rows, adjoint rows and checkpoints per wave slot, held to kSecondChanceBytes (at least one workgroup)
        const int C2 = 1 << p.BL;
        const size_t slot_bytes = ((size_t)p.ns * p.rowlen + 4 * (size_t)p.rowlen +
                                   (size_t)p.ns * (p.nseg + 1) * (2 * C2 + 2) * kWave) * elem;
        int64_t g = (int64_t)(kSecondChanceBytes / (slot_bytes * kWavesPerWG));
        if (g < 1) g = 1;
        if (g < p.grid) p.grid = (int)g;
        p.nslots = (int64_t)p.grid * kWavesPerWG;
    }

    // Lock-step mode replaces the modes above when every pair can have a workgroup of its own resident at
    // once: the chip is then under-filled and the time of a call is the latency of one pair's chain of
    // macro-steps, which this mode shortens (fewer instructions in the wave that carries the recurrence,
    // fewer strips, no waits).
    if (lock_max_rows(backward, p.BL, p.DT) > 0 && (!backward || p.uncompute) && !second_chance) {
        const int maxM = lock_max_rows(backward, p.BL, p.DT);
        int M = 1;
        while (M < maxM && (p.mb + kWave * M - 1) / (kWave * M) > 2) M *= 2;
        const int lns = (p.mb + kWave * M - 1) / (kWave * M);
        const int NT = (int)align_up((size_t)p.nb + kWave - 1, 8);
        const int lrow = (int)align_up((size_t)kWave * C + (size_t)NT * C + C + 2, 2);
        size_t used = 0;
        auto lds_take = [&](size_t bytes) { size_t o = used; used = align_up(used + bytes, 256); return o; };
        const size_t ycopy = (size_t)p.q * p.DP * elem;
        const size_t o_y = lds_take(ycopy);
        const size_t o_gy = backward ? lds_take(ycopy) : 0;
        const size_t cstride = (size_t)16384 * M;   // 2 chunks x (8 steps x 16 B | 4 steps x 32 B) x 64 lanes x M
        const size_t o_cr = lds_take(cstride * lns);
        const size_t gstride = (size_t)2 * kLockCH2 * M * kWave * elem;
        const size_t o_gp = backward ? lds_take(gstride * lns) : 0;
        const size_t o_kr = lds_take((size_t)(lns + 1) * lrow * elem);
        const size_t o_ar = backward ? lds_take((size_t)(lns + 1) * lrow * elem) : 0;
        const size_t o_dump = lds_take((size_t)(kWave + 8) * C * elem);
        const size_t kstride = (size_t)2 * (M * R + 1 + C) * kWave * elem;   // two staged checkpoints per strip
        const size_t o_ck = backward ? lds_take(kstride * lns) : 0;
        const int waves = lns == 1 ? 3 : (lns == 2 ? 8 : 12);
        int wgpc = used ? (int)(kLdsPerCU / used) : 0;
        if (wgpc * waves > 16) wgpc = 16 / waves;
        if (lns <= (backward ? kLockMaxStripsBwd : kLockMaxStrips) && used <= kLdsPerCU - 1024 && wgpc >= 1 && p.npairs <= (int64_t)kNumCU * wgpc) {
            p.lock = 1; p.coop = 0;
            p.lk_M = M; p.lk_ns = lns; p.lk_NT = NT; p.lk_rowlen = lrow;
            p.lk_padb = lns * kWave * M - p.mb;
            p.lk_off_y = o_y; p.lk_off_gy = o_gy; p.lk_off_cring = o_cr; p.lk_off_gp = o_gp;
            p.lk_off_krows = o_kr; p.lk_off_arows = o_ar; p.lk_off_dump = o_dump;
            p.lk_cring_stride = cstride; p.lk_gp_stride = gstride;
            p.lk_off_ck = o_ck; p.lk_ck_stride = kstride;
            p.y_lds = 1;
            p.lds_wave = 0;
            p.lds_bytes = align_up(used, 256);
            p.grid = (int)p.npairs;
            p.nslots = p.npairs;
            p.S = kLockS;
            p.nseg = NT / kLockS;
        }
    }

    // Solo mode: enough pairs to fill the chip, and all block rows of a pair fit one strip of 64 M rows.
    if (!p.lock && solo_max_rows(backward, p.BL, p.DT) > 0 && (!backward || p.uncompute) && !second_chance) {
        const int M = p.mb > kWave ? 2 : 1;
        const int NT = (int)align_up((size_t)p.nb + kWave - 1, 8);
        size_t used = 0;
        auto lds_take = [&](size_t bytes) { size_t o = used; used = align_up(used + bytes, 256); return o; };
        const size_t ycopy = (size_t)p.q * p.DP * elem;
        lds_take(ycopy);
        const size_t o_gy = backward ? lds_take(ycopy) : 0;
        const size_t o_gyp = backward ? lds_take(ycopy) : 0;   // y-side sums of the pair in work
        const size_t o_kr = backward ? lds_take(((size_t)kWave * C + (size_t)NT * C + 2) * elem) : 0;
        const size_t o_dump = backward ? lds_take((size_t)kWave * C * elem) : 0;
        const int maxwg = backward ? solo_bwd_waves_per_simd(p.BL, M, p.DT) : 4;   // register file of the backward kernel
        if (M <= solo_max_rows(backward, p.BL, p.DT) && p.mb <= kWave * M && used * kWavesPerWG <= kLdsPerCU) {
            p.solo = 1; p.coop = 0;
            p.lk_M = M; p.lk_ns = 1; p.lk_NT = NT; p.lk_padb = kWave * M - p.mb;
            p.lk_off_y = 0; p.lk_off_gy = o_gy; p.lk_off_krows = o_kr; p.lk_off_dump = o_dump; p.lk_off_gyp = o_gyp;
            p.y_lds = 1;
            p.lds_wave = used;
            p.lds_bytes = used * kWavesPerWG;
            int wgpc = (int)(kLdsPerCU / p.lds_bytes);
            if (wgpc > maxwg) wgpc = maxwg;
            const int64_t want = (p.npairs + kWavesPerWG - 1) / kWavesPerWG;
            const int64_t cap = (int64_t)kNumCU * wgpc;
            p.grid = (int)(want < cap ? want : cap);
            p.nslots = (int64_t)p.grid * kWavesPerWG;
            p.S = kLockS;
            p.nseg = NT / kLockS;
        }
    }

    // Tile mode: many pairs of at most 64 x 64 unrefined cells with 8 or 16 channels; the contractions over
    // the channels and over the rows / columns run as MFMA tiles, the sweep reads one number per cell from LDS.
    if (!p.lock && !lead_lag && p.BL == 0 && p.rs1 == 0 && p.rs2 == 0 && (p.DT == 8 || p.DT == 16) && p.mb > kWave / 2 &&
        p.mb <= kWave && p.nb > kWave / 2 && p.nb <= kWave && (!backward || p.uncompute) && !second_chance) {
        const int NT = (int)align_up((size_t)p.nb + kWave - 1, 8);
        size_t used = 0;
        auto lds_take = [&](size_t bytes) { size_t o = used; used = align_up(used + bytes, 256); return o; };
        lds_take((size_t)kTileCols * kTileStride * elem);
        // backward: compact checkpoints (two doubles per lane) every kTileCkChunks chunks of 8 macro-steps
        const int nck = backward ? (NT / kLockS - 1) / kTileCkChunks : 0;
        const size_t o_ck = nck ? lds_take((size_t)nck * 2 * kWave * elem) : 0;
        // backward: the pair's bottom row, node columns -kTileRowPad .. 64 and slack up to a multiple of eight
        const size_t o_kr = backward ? lds_take((size_t)(kTileRowPad + kWave + 8) * elem) : 0;
        p.tile = 1; p.solo = 0; p.coop = 0;
        p.lk_M = 1; p.lk_ns = 1; p.lk_NT = NT; p.lk_padb = kWave - p.mb;
        p.lk_off_y = 0; p.lk_off_gy = 0; p.lk_off_krows = o_kr; p.lk_off_dump = 0; p.lk_off_ck = o_ck;
        p.y_lds = 0;
        p.lds_wave = used;
        p.lds_bytes = used * kWavesPerWG;   // one workgroup per compute unit
        const int64_t want = (p.npairs + kWavesPerWG - 1) / kWavesPerWG;
        p.grid = (int)(want < kNumCU ? want : kNumCU);
        p.nslots = (int64_t)p.grid * kWavesPerWG;
        p.S = kLockS;
        p.nseg = NT / kLockS;
    }

    // Symmetric Gram matrix: k(x, y) = k(y, x) bit for bit, so the solo and tile kernels solve the pairs n <= m
    // only, write both entries of K, and use the sum of the two upstream gradients.  Eq. (1) is symmetric under
    // a swap of the paths together with their dyadic orders, so this holds for equal orders only; with unequal
    // orders K(X, X) is not a symmetric matrix and all N^2 pairs are solved over the shared increment buffer.
    if (symmetric && gram && nx == ny && lam1 == lam2 && (p.solo || p.tile)) {
        p.tri = 1;
        p.npairs = nx * (nx + 1) / 2;
        const int64_t want = (p.npairs + kWavesPerWG - 1) / kWavesPerWG;
        if (want < p.grid) p.grid = (int)want;
        p.nslots = (int64_t)p.grid * kWavesPerWG;
    }

    // Quad mode: forward calls for Gram matrices (the four pairs of a wavefront share the y path) on the shapes of the
    // tile kernels and on those of the solo kernels whose blocks hold all of the refinement.  The sequence is the Gram
    // matrix row by row (y-major) in groups of four x paths; a symmetric Gram matrix has the pairs n <= m of row m
    // only.  Two workgroups of four waves per compute unit.
    if ((p.tile || p.solo) && !backward && gram && !lead_lag && p.rs1 == 0 && p.rs2 == 0) {
        const int lanes = kWave / kQuadPairs;
        const int M = p.mb <= 4 * lanes ? 4 : 8;
        const size_t ycopy = align_up((size_t)(p.nb + 1) * quad_y_stride(p.DT) * elem, 256);   // the y copy and a row of zeros
        if (M <= quad_max_rows(p.BL, p.DT) && p.mb <= M * lanes && ycopy * kWavesPerWG <= kLdsPerCU) {
            p.tile = 0; p.solo = 0; p.quad = 1;
            if (p.tri) {
                const int64_t J = nx / kQuadPairs, e = nx % kQuadPairs;
                p.nquads = 2 * J * (J + 1) + e * (J + 1);
            } else {
                p.nquads = ny * ((nx + kQuadPairs - 1) / kQuadPairs);
            }
            p.lk_M = M; p.lk_ns = 1; p.lk_NT = p.nb + lanes - 1; p.lk_padb = M * lanes - p.mb;
            p.y_lds = 1;
            p.lds_wave = ycopy;
            p.lds_bytes = p.lds_wave * kWavesPerWG;
            const int64_t want = (p.nquads + kWavesPerWG - 1) / kWavesPerWG;
            const int64_t cap = (int64_t)kNumCU * (2 * p.lds_bytes <= kLdsPerCU ? 2 : 1);
            p.grid = (int)(want < cap ? want : cap);
            p.nslots = (int64_t)p.grid * kWavesPerWG;
        }
    }

    // Band mode: few pairs of long paths.  The strips of a pair are spread over workgroups (bands of kBandStrips
    // strips) that all run at once; chosen when that fills more of the chip than one workgroup per pair does.
    if (!p.lock && !p.tile && !p.solo && (!backward || p.uncompute) && p.DT >= 2 && p.DT <= 8 && p.ns > kBandMinStrips &&
        !second_chance) {
        const int nbands = (p.ns + kBandStrips - 1) / kBandStrips;
        if (p.npairs * nbands <= kNumCU) {
            const int NT = (int)align_up((size_t)p.nb + kWave - 1, 8);
            size_t used = 0;
            auto lds_take = [&](size_t bytes) { size_t o = used; used = align_up(used + bytes, 256); return o; };
            const size_t ybytes = (size_t)kBandYRing * p.DP * elem;
            p.bd_off_y = lds_take(ybytes);
            p.bd_off_gy = backward ? lds_take(ybytes) : 0;
            // forward: hand-over rings; backward: adjoint rings, forward-value rings, checkpoint staging
            p.bd_off_rings = lds_take(((size_t)(kBandStrips + 1) * kBandRing * C +
                                       (backward ? (size_t)kBandStrips * kBandRing * C +
                                                       (size_t)kBandStrips * 2 * (R + 1 + C) * kWave : 0)) * elem);
            p.band = 1; p.coop = 0; p.bd_nbands = nbands;
            p.lk_M = 1; p.lk_ns = p.ns; p.lk_NT = NT; p.lk_padb = p.ns * kWave - p.mb;
            p.y_lds = 1;
            p.lds_wave = 0;
            p.lds_bytes = used;
            p.grid = (int)(p.npairs * nbands);
            p.nslots = p.npairs;
            p.S = kLockS;
            p.nseg = NT / kLockS;
            p.nflags = (int)(2 * p.npairs * nbands);
        }
    }

    // Workspace layout (all offsets 256-byte aligned).
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes, 256); return o; };
    // first, so that their place does not depend on the rest of the layout: the error flag, the progress counters
    // of band mode directly behind it (cleared with it), and behind those the counter of drifted pairs
    p.off_err = take(256);
    p.off_flags = take((size_t)p.nflags * sizeof(int) + 4);
    p.off_badcnt = p.off_flags + (size_t)p.nflags * sizeof(int);
    if (!second_chance) {
        p.off_dxT = take((size_t)nx * p.xstride * elem);
        p.off_dyT = symmetric ? p.off_dxT : take((size_t)ny * p.ystride * elem);
    }
    p.rows_slot = (int64_t)p.ns * p.rowlen;
    p.off_rows = take((size_t)p.nslots * p.rows_slot * elem);
    if (backward) {
        if (!second_chance) {
            p.off_gdxT = take((size_t)nx * p.xstride * elem);
            p.off_gdyT = symmetric ? p.off_gdxT : take((size_t)ny * p.ystride * elem);
        }
        p.adj_slot = (p.band && p.bd_nbands > 4 ? p.bd_nbands : 4) * (int64_t)p.rowlen;   // two rows of 2C values per block column; band mode: one row per band
        p.off_adj = take((size_t)p.nslots * p.adj_slot * elem);
        // lane state kept per checkpoint: right edge, bottom edge, bottom-left corner
        const bool lean = p.lock || p.solo || p.tile || p.band;
        const int NVC = lean ? p.lk_M * R + C + 2 : R + C + 2;
        p.ckpt_slot = p.tile ? 0 : (int64_t)(lean ? p.lk_ns : p.ns) * (p.nseg + 1) * NVC * kWave;
        p.keep_solo = (keep && p.solo) ? 1 : 0;
        p.off_ckpt = take((size_t)(p.keep_solo ? p.npairs : p.nslots) * p.ckpt_slot * elem);
        if (p.keep_solo) {
            p.keep_len = (int64_t)kWave * C + (int64_t)p.lk_NT * C + 2;   // the bottom row as the kernel holds it in LDS
            p.off_keep = take((size_t)p.npairs * p.keep_len * elem);
            p.off_keep_tag = take(256);
        }
        if (p.lock) p.off_keep = take((size_t)p.npairs * (p.lk_ns + 1) * p.lk_rowlen * elem);
        else if (p.band) p.off_keep = take((size_t)p.kcount * elem);   // band mode: the kernel values of the kept sweep
        if (p.lock || p.band) p.off_keep_tag = take(256);   // which call's forward sweep the workspace holds
    }
    if (io_elem != elem) {
        p.off_kio = take((size_t)p.kcount * elem);
        if (backward) p.off_gkio = take((size_t)p.kcount * elem);
    }
    if (backward && p.uncompute && !second_chance) p.off_badlist = take((size_t)p.kcount * sizeof(long long));
    p.total = off;
    p.valid = true;
    return p;
}

}  // namespace sk

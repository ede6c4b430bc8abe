// Host-side launch plan for batched truncated signatures by Horner's scheme (paper Section 2.3): pure arithmetic,
// no HIP calls, so that the workspace query, the description and the launch agree by construction.
//
// How the update of Section 2.3 is spread over lanes.  One step of Horner's algorithm updates every level k by
//     A_k[w c] += G_k[w] z[c],   G_k[v c'] = G_k[v] z[c'] / (k - |v|) + A_{|v|+1}[v c'],   G_k[empty] = 1,
// for words w of length k - 1 (the nesting of Section 2.3 read word by word: G_k[w] = B_k[w] + A_{k-1}[w]).  The value
// at a word depends only on values at its prefixes, so the entries of the signature whose words start with a given
// prefix u form a closed system.  A lane owns a prefix u of Q letters, a block of S consecutive next letters, and
// every word that continues them up to M further letters: S (D^(M+1) - 1)/(D - 1) numbers, kept in registers for all
// steps of the path; it also carries the Q entries at the prefixes of u (every lane under the same prefix carries the
// same copies).  A step needs no communication between lanes.  Lanes of one wave belong to one path, so the
// increment z of a step is the same for the whole wave and is fetched by scalar loads.
#pragma once
#include <cstddef>
#include <cstdint>

namespace sg {

constexpr int kWave = 64;
constexpr int kWavesPerWG = 4;
constexpr int kXcds = 8;
constexpr int kQMax = 8;            // longest carried prefix
constexpr int kQExact = 4;          // prefix lengths with code of their own
constexpr int kLongPrefixMaxD = 9;   // channel counts whose variants also exist for prefixes longer than kQExact
constexpr int64_t kSimds = 1024;       // 256 compute units of 4 SIMDs
constexpr int kMinPiece = 32;          // fewest segments a piece of a path is cut down to
constexpr int kMaxPieces = 1024;
constexpr int kSharedMaxQ = 2;         // waves that hold several paths: longest prefix and most channels with such kernels
constexpr int kSharedMaxD = 9;

// (channels, owned depth M, letter block S), per channel count in order of falling register use.
#define SG_VARIANTS(X)                                                                                     \
    X(2, 5, 1) X(2, 4, 1) X(2, 3, 1) X(2, 2, 1) X(2, 1, 1)                                                 \
    X(3, 3, 1) X(3, 2, 1) X(3, 1, 1)                                                                       \
    X(4, 3, 1) X(4, 2, 1) X(4, 1, 1)                                                                       \
    X(5, 2, 1) X(5, 1, 1) X(6, 2, 1) X(6, 1, 1) X(7, 2, 1) X(7, 1, 1) X(8, 2, 1) X(8, 1, 1) X(9, 2, 1) X(9, 1, 1) \
    X(10, 1, 5) X(11, 1, 4) X(12, 1, 4) X(13, 1, 4) X(14, 1, 4) X(15, 1, 4) X(16, 1, 4) X(17, 1, 4)

// Variants of the backward kernels: a lane also holds the adjoints of its entries, so the subtrees are smaller.
#define SG_BWD_VARIANTS(X)                                                                                 \
    X(2, 4, 1) X(2, 3, 1) X(2, 2, 1) X(2, 1, 1)                                                            \
    X(3, 3, 1) X(3, 2, 1) X(3, 1, 1)                                                                       \
    X(4, 2, 2) X(4, 2, 1) X(4, 1, 1)                                                                       \
    X(5, 2, 1) X(5, 1, 1) X(6, 2, 1) X(6, 1, 3) X(6, 1, 1) X(7, 1, 4) X(7, 1, 1) X(8, 1, 4) X(8, 1, 1)     \
    X(9, 1, 3) X(9, 1, 1)                                                                                  \
    X(10, 1, 2) X(11, 1, 2) X(12, 1, 2) X(13, 1, 2) X(14, 1, 2) X(15, 1, 2) X(16, 1, 2) X(17, 1, 2)
constexpr int kBwdLongPrefixMaxD = 5;   // as kLongPrefixMaxD, for the backward variants
constexpr int kBwdMaxRuntimeD = 1024;   // run-time channel count kernel, backward: per-channel sums of a wave live in LDS

struct Variant { int D, M, S; };
#define SG_ROW(D, M, S) {D, M, S},
constexpr Variant kVariants[] = {SG_VARIANTS(SG_ROW)};
constexpr Variant kBwdVariants[] = {SG_BWD_VARIANTS(SG_ROW)};
#undef SG_ROW

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct Plan {
    bool valid = false;
    const char* why = "";
    int64_t B = 0, L = 0;
    int d = 0;            // channels of the caller's paths
    int D = 0;            // channels after the transformations
    int N = 0;
    int64_t n = 0;        // segments after the transformations
    int64_t np = 0;       // increment rows stored per piece: its segments, then zero rows up to an odd count
    int P = 1;            // pieces per path (forward only): the signatures of the pieces are multiplied afterwards
    int64_t Lc = 0;       // segments per piece
    int64_t VB = 0;       // pieces in the batch: B * P, each one a path of its own to the Horner kernel
    int DT = 0;           // kernel template channel count (0: run-time channel count, M = 0, S = 1)
    int M = 0, S = 1, Q = 0, NB = 1;
    int64_t LP = 0;       // lanes per path: D^Q * NB
    int64_t WP = 0;       // waves per path
    int PW = 1;           // paths per wave (forward): short paths side by side in one wave
    int64_t waves = 0;
    int64_t grid = 0;
    int Dpad = 0;         // doubles per stored increment row
    int64_t sig_len = 0;  // entries per path, level 0 included
    int io_elem = 8;
    size_t off_dz = 0, off_out = 0, total = 0;
    size_t off_t0 = 0, off_t1 = 0;   // signatures of the pieces and of their pairwise products (P > 1)
    // backward
    bool backward = false;
    size_t lds_wave = 0;      // doubles of LDS per wave
    size_t lds_bytes = 0;
    size_t off_gz = 0, off_sig = 0, off_gout = 0;
};

// entries of levels 0..N over D channels; 0 if that does not fit in 2^40
inline int64_t sig_length(int64_t D, int N)
{
    if (D < 1 || N < 0) return 0;
    const int64_t lim = (int64_t)1 << 40;
    int64_t tot = 0, p = 1;
    for (int k = 0; k <= N; ++k) {
        tot += p;
        if (tot > lim) return 0;
        if (k < N) {
            if (p > lim / D) return 0;
            p *= D;
        }
    }
    return tot;
}

// force_M >= 0 / force_S > 0 pick the variant with that owned depth / letter block (diagnostics and tests);
// -1 / 0 = the estimate below decides
// backward: the plan of signature_bwd (have_sig: the caller passes the signatures, else they are computed into the
// workspace first, with the forward plan for the same arguments)
inline Plan make_plan(int64_t B, int64_t L, int64_t d, int N, bool time_aug, bool lead_lag, bool io_double,
                      int force_M = -1, bool backward = false, bool have_sig = false, int force_S = 0,
                      int force_P = 0,   // force_P: 0 = the plan decides, else the number of pieces (a power of two)
                      int force_W = 0)   // force_W: 1 = a wave never holds more than one path
{
    Plan p;
    p.backward = backward;
    p.B = B; p.L = L; p.d = (int)d; p.N = N;
    p.io_elem = io_double ? 8 : 4;
    const int64_t D = (lead_lag ? 2 * d : d) + (time_aug ? 1 : 0);
    p.D = (int)D;
    p.n = L < 1 ? 0 : (lead_lag ? 2 * (L - 1) : L - 1);
    p.Lc = p.n;
    p.np = p.n == 0 ? 0 : (p.n | 1);
    p.VB = B;
    p.sig_len = sig_length(D, N);
    if (p.sig_len == 0) { p.why = "the signature has more than 2^40 entries per path"; return p; }
    if (B > 0 && p.sig_len > ((int64_t)1 << 46) / B) { p.why = "the batch of signatures has more than 2^46 entries"; return p; }
    if (B > 0 && p.np * (D + 1) > ((int64_t)1 << 44) / B) { p.why = "the batch of increments has more than 2^44 entries"; return p; }

    auto lanes = [&](int M, int S, int64_t& LP, int& Q, int& NB) -> bool {
        Q = N - M - 1;
        if (Q < 0 || Q > kQMax) return false;
        if (Q > kQExact && M > 0 && D > (backward ? kBwdLongPrefixMaxD : kLongPrefixMaxD)) return false;
        NB = (int)((D + S - 1) / S);
        LP = NB;
        for (int i = 0; i < Q; ++i) {
            if (LP > ((int64_t)1 << 40) / D) return false;
            LP *= D;
        }
        return true;
    };
    auto choose = [&](int64_t Bsel) -> bool {
        // The variant with the least estimated time.  A lane executes about `instr` vector instructions per step: the
        // multiply-adds of its owned levels and their chains, the chains over the carried prefix for each owned level,
        // the updates of the carried entries, and a fixed part for loads and loop control.  A SIMD issues one such
        // instruction per 4 clocks when it has several waves and per about 5 clocks when it has a single one, and the
        // waves of the launch are spread over kSimds SIMDs.
        bool have = false;
        double best = 0.0;
        const Variant* list = backward ? kBwdVariants : kVariants;
        const size_t nlist = backward ? sizeof(kBwdVariants) / sizeof(Variant) : sizeof(kVariants) / sizeof(Variant);
        for (size_t vi = 0; vi < nlist; ++vi) {
            const Variant& v = list[vi];
            if (v.D != D || (force_M >= 0 && v.M != force_M) || (force_S > 0 && v.S != force_S)) continue;
            int64_t LP; int Q, NB;
            if (!lanes(v.M, v.S, LP, Q, NB)) continue;
            // lane groups of at most half a wave can share a wave (forward kernels for few channels and letters)
            const int pw = (LP <= kWave / 2 && Q <= kSharedMaxQ && D <= kSharedMaxD && force_W != 1) ? (int)(kWave / LP) : 1;
            const int64_t waves = pw > 1 ? (Bsel + pw - 1) / pw : Bsel * ((LP + kWave - 1) / kWave);
            double owned = 0.0, lvl = v.S, sum = 0.0;
            for (int m = 0; m <= v.M; ++m) {
                sum += lvl;        // nodes of levels 0..m
                owned += sum;      // the update of owned level m touches all of them once
                lvl *= (double)D;
            }
            // several paths per wave: the increments are loaded per lane; backward, a lane per path and channel reads the
            // LDS rows of its path
            const double instr = owned + (v.M + 1) * (2.0 * Q + 1.0) + (double)Q * Q + 12.0 + (pw > 1 ? (double)D : 0.0) +
                                 (pw > 1 && backward ? (double)LP : 0.0);
            const double rounds = (double)((waves + kSimds - 1) / kSimds);
            const double cost = rounds * instr * (waves <= kSimds ? 5.0 : 4.0);
            if (!have || cost < best) {
                best = cost;
                p.DT = v.D; p.M = v.M; p.S = v.S; p.Q = Q; p.NB = NB; p.LP = LP; p.PW = pw;
                have = true;
            }
        }
        if (!have && force_M > 0) { p.why = "no kernel with the requested subtree depth for this number of channels and level"; return false; }
        if (!have) {
            int64_t LP; int Q, NB;
            if (!lanes(0, 1, LP, Q, NB)) { p.why = "truncation level too high for this number of channels (a lane carries at most 8 prefix letters)"; return false; }
            p.DT = 0; p.M = 0; p.S = 1; p.Q = Q; p.NB = NB; p.LP = LP;
            p.PW = (!backward && LP <= kWave / 2 && Q <= kSharedMaxQ && force_W != 1) ? (int)(kWave / LP) : 1;
        }
        p.WP = (p.LP + kWave - 1) / kWave;
        return true;
    };
    if (!choose(B)) return p;
    // Few long paths leave most SIMDs without a wave: cut every path into P pieces of Lc segments, let the Horner
    // kernel treat the pieces as paths, and multiply the signatures of the pieces pairwise afterwards (Chen's identity,
    // Proposition 2.2).  Backward: the same products, then their adjoints pair by pair back down to the pieces, then
    // the backward kernel on the pieces.
    if (p.n > 0) {
        int P = 1;
        if (force_P > 0) {
            P = force_P;
        } else if (B > 0 && p.n >= 2 * kMinPiece && p.sig_len < ((int64_t)1 << 31)) {
            // backward, the products and their adjoints cost several launches: only when the chip is mostly empty
            const int64_t w1 = p.PW > 1 ? (B + p.PW - 1) / p.PW : B * p.WP;
            const int64_t few = backward ? kSimds / 2 : kSimds, want = backward ? kSimds : 2 * kSimds;
            if (w1 < few)
                while (P < kMaxPieces && w1 * P < want && p.n / (2 * P) >= kMinPiece) P *= 2;
        }
        if (P > 1) {
            if ((P & (P - 1)) != 0 || P > kMaxPieces) { p.why = "the number of pieces must be a power of two up to 1024"; return p; }
            if (p.sig_len >= ((int64_t)1 << 31)) { p.why = "paths are cut into pieces only for signatures of fewer than 2^31 entries"; return p; }
            if (B > 0 && (p.sig_len > ((int64_t)1 << 44) / (B * P))) { p.why = "too many pieces for this signature size"; return p; }
            p.P = P;
            p.Lc = (p.n + P - 1) / P;
            if (lead_lag) p.Lc += p.Lc & 1;      // a piece starts with a move of the lead half
            p.np = p.Lc | 1;
            p.VB = B * P;
            if (!choose(p.VB)) return p;
        }
    }
    p.waves = p.PW > 1 ? (p.VB + p.PW - 1) / p.PW : p.VB * p.WP;
    p.grid = (p.waves + kWavesPerWG - 1) / kWavesPerWG;
    if (p.grid > 0x7fffffffLL) { p.why = "too many workgroups"; return p; }
    p.Dpad = (int)align_up((size_t)D, 2);
    size_t off = 0;
    p.off_dz = off;
    off = align_up(off + (size_t)p.VB * (size_t)p.np * p.Dpad * sizeof(double), 256);
    p.off_out = off;
    if (!backward) {
        if (!io_double) off = align_up(off + (size_t)B * (size_t)p.sig_len * sizeof(double), 256);
        if (p.P > 1) {
            p.off_t0 = off;
            off = align_up(off + (size_t)p.VB * (size_t)p.sig_len * sizeof(double), 256);
            p.off_t1 = off;
            off = align_up(off + (size_t)(p.VB / 2) * (size_t)p.sig_len * sizeof(double), 256);
        }
    } else {
        if (p.DT == 0 && D > kBwdMaxRuntimeD) { p.why = "backward: more than 1024 channels"; return p; }
        const bool uniform = p.DT > 0 && p.M > 0;
        p.lds_wave = (size_t)p.Dpad + (uniform ? (size_t)kWave * (size_t)(D | 1) : 0);
        p.lds_bytes = (size_t)kWavesPerWG * p.lds_wave * sizeof(double);
        p.off_gz = off;      // dF/dz, one row per stored increment row
        off = align_up(off + (size_t)p.VB * (size_t)p.np * p.Dpad * sizeof(double), 256);
        p.off_sig = off;     // signatures in double: computed here, or converted from a float caller's
        if (p.P == 1 && (!have_sig || !io_double)) off = align_up(off + (size_t)B * (size_t)p.sig_len * sizeof(double), 256);
        p.off_gout = off;    // float callers: the upstream gradient in double
        if (!io_double) off = align_up(off + (size_t)B * (size_t)p.sig_len * sizeof(double), 256);
        if (p.P > 1) {
            // signatures of the pieces and of the products of 2, 4, ... neighbouring pieces (levels 0 .. log2 P - 1 of
            // the product tree, P + P/2 + ... + 2 signatures per path), and the adjoints of the same
            const size_t tree = (size_t)(2 * p.VB - 2 * B) * (size_t)p.sig_len * sizeof(double);
            p.off_t0 = off;
            off = align_up(off + tree, 256);
            p.off_t1 = off;
            off = align_up(off + tree, 256);
        }
    }
    p.total = off < 256 ? 256 : off;
    p.valid = true;
    return p;
}

}  // namespace sg

/*
 * signature.h - C ABI for batched truncated signatures on MI355X (gfx950); part of libsigkernel.
 *
 * What is computed (paper Section 2): for a piecewise-linear path x of L points in R^d the levels 0..N of its
 * signature (Definition 2.1), S(x) = exp(z_1) (x) exp(z_2) (x) ... (x) exp(z_{L-1}) with z_l = x[l+1] - x[l]
 * (Proposition 2.1 for a segment, Chen's identity, Proposition 2.2, for the concatenation), evaluated by Horner's
 * scheme of Section 2.3 (Algorithm "Horner's Algorithm for Truncated Signatures"): per segment and level k,
 *     A_k <- (B_k + A_{k-1}) (x) z + A_k,   B_k = ((z/k + A_1) (x) z/(k-1) + A_2) (x) ... (x) z/2.
 *
 * Layout of a result: levels 0..N one after the other (level 0 is the number 1), level k in row-major order of
 * its word (i_1, ..., i_k), i_k fastest: signature_length(...) = (D^(N+1) - 1)/(D - 1) entries per path, D the number
 * of channels after the transformations of `flags` (d, 2d, d + 1 or 2d + 1).
 *
 * Conventions are those of sigkernel.h: device pointers to dense row-major arrays owned by the caller, element
 * type `dt` for every array of the call (the arithmetic is in double for both), caller-owned 256-byte aligned
 * workspace of at least signature_workspace_bytes(...) bytes, calls only enqueue work on `stream`, return value SK_OK
 * or a negative SK_ERR_* code with a message in sigkernel_last_error(), nothing enqueued on error.  B = 0 is a
 * successful no-op; a path of one point has the signature (1, 0, ..., 0).
 * flags: SK_FLAG_TIME_AUG and SK_FLAG_LEAD_LAG as in sigkernel.h (Section 4, applied on the fly: the transformed
 * paths are never formed, only their increments), and the diagnostics SK_SIG_DEPTH(m), SK_SIG_BLOCK(s), SK_SIG_PIECES(q), SK_SIG_ONE_PATH_PER_WAVE below; other bits are an error.
 * Limits: N >= 1; at most 2^40 entries per path and 2^46 per call; a lane carries the entries at up to 8 prefix
 * letters, which admits every N <= 9 (N <= 14 for two channels); beyond that SK_ERR_SHAPE.
 */
#ifndef SIGKERNEL_SIGNATURE_H
#define SIGKERNEL_SIGNATURE_H

#include "sigkernel.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Diagnostics, for the entry points of this header only: a lane keeps the entries of a subtree of words in registers,
 * a block of s consecutive letters after its prefix and every continuation by up to m more letters.  SK_SIG_DEPTH(m),
 * m = 0..5, and SK_SIG_BLOCK(s), s = 1..15, or-ed into `flags` force m and s instead of the library's own choice
 * (SK_ERR_SHAPE if no such kernel exists for the shape).  Results do not depend on them beyond rounding order. */
#define SK_SIG_DEPTH(m) (((m) + 1) << 8)
#define SK_SIG_BLOCK(s) ((s) << 12)
/* signature_fwd cuts each path of a small batch of long paths into 2^q pieces, runs the pieces as paths of their own
 * and multiplies their signatures afterwards (Chen's identity, Proposition 2.2).  SK_SIG_PIECES(q), q = 0..10, forces
 * 2^q pieces (q = 0: never cut) instead of the library's own choice. */
#define SK_SIG_PIECES(q) (((q) + 1) << 16)
/* signature_fwd lets a wave work on several short paths side by side when a path needs at most half a wave's lanes;
 * this flag keeps every wave to one path. */
#define SK_SIG_ONE_PATH_PER_WAVE 0x200000
#define SK_SIG_DEPTH_MASK 0x3fff00

/* Entries per path of the result for paths of d channels, level 0 included; 0 for invalid arguments or when the
 * count does not fit.  Pure host arithmetic. */
int64_t signature_length(int64_t d, int N, int flags);

/* Bytes of device scratch for signature_fwd with the same arguments (increments of the transformed paths, and a
 * double copy of the result for float callers).  Pure host arithmetic; 0 for invalid arguments. */
size_t signature_workspace_bytes(int64_t B, int64_t L, int64_t d, int N, int flags, sk_dtype dt);

/* x[B,L,d] -> out[B, signature_length(d, N, flags)]  (Section 2.3). */
int signature_fwd(const void* x, void* out, int64_t B, int64_t L, int64_t d, int N, int flags, sk_dtype dt, void* ws,
                  size_t ws_bytes, void* stream);

/*
 * Gradient with respect to the path points (Section 2.4): given grad_out[B, signature_length(d, N, flags)] = dF/dS for
 * the signatures S = signature_fwd(x), writes grad_x[B,L,d] = dF/dx.  sig is the output of signature_fwd for the same
 * x, N and flags, or NULL to have it computed into the workspace first.  As Section 2.4 describes, the path is walked
 * backwards, the signature before each segment is recovered from the one after it by multiplying with the tensor
 * exponential of the negated increment (Horner's step again), and the adjoint is taken through that one step; no
 * intermediate signature is stored.  Level 0 of grad_out has no effect.  Gradient entries are sums formed by
 * floating-point atomics: reproducible to rounding, not bit for bit.
 * have_sig != 0 in the workspace query if sig will not be NULL.
 */
size_t signature_bwd_workspace_bytes(int64_t B, int64_t L, int64_t d, int N, int flags, sk_dtype dt, int have_sig);
int signature_bwd(const void* x, const void* sig, const void* grad_out, void* grad_x, int64_t B, int64_t L, int64_t d,
                  int N, int flags, sk_dtype dt, void* ws, size_t ws_bytes, void* stream);

/* Diagnostics (no passage of the paper): human-readable launch plan for these arguments, as sigkernel_describe. */
int signature_bwd_describe(int64_t B, int64_t L, int64_t d, int N, int flags, sk_dtype dt, char* out, size_t out_bytes);
int signature_describe(int64_t B, int64_t L, int64_t d, int N, int flags, sk_dtype dt, char* out, size_t out_bytes);

#ifdef __cplusplus
}
#endif
#endif /* SIGKERNEL_SIGNATURE_H */

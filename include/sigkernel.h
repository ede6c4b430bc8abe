/*
 * sigkernel.h - C ABI of the MI355X (gfx950) signature-kernel library.
 *
 * What is computed (paper Section 3): for piecewise-linear paths x (L1 points in R^d) and y (L2 points)
 * the signature kernel k(x,y) = <S(x), S(y)> is the value at the far corner of the solution of the
 * Goursat PDE d2k/dsdt = <x'(s), y'(t)> k, k(0,.) = k(.,0) = 1 (Section 3.1), discretised by the explicit
 * scheme Eq. (1)
 *     k[i+1,j+1] = (k[i+1,j] + k[i,j+1]) A(p) - k[i,j] B(p),  A = 1 + p/2 + p^2/12,  B = 1 - p^2/12,
 * on the dyadically refined grid of 2^lam1 (L1-1) by 2^lam2 (L2-1) cells, with
 *     p = 2^-(lam1+lam2) <x[a+1]-x[a], y[b+1]-y[b]>,  a = i >> lam1,  b = j >> lam2
 * (refinement applied on the fly, Section 3.2 item (3); lam1 != lam2 allowed, item (1)).
 * The backward entry points return the exact gradients of that discrete scheme with respect to the
 * path points (Section 3.4: the adjoint recurrence for dF/dk[i,j], the local derivative giving
 * dF/dDelta, and the linear map from dF/dDelta to dF/dx and dF/dy).
 *
 * Conventions for every entry point
 *  - All data pointers are DEVICE pointers to dense row-major arrays owned by the caller; a path batch
 *    is [count, L, d] with d fastest.  Element type is given by `dt` (float or double) for every array
 *    of the call.  Outputs are overwritten, never accumulated into.
 *  - `ws` is caller-owned device scratch of at least sigkernel_workspace_bytes(...) bytes for the same
 *    arguments, 256-byte aligned; its contents are undefined afterwards.  The library allocates and frees
 *    nothing.
 *  - `stream` is a hipStream_t (NULL = the default stream).  Calls only enqueue work: no host
 *    synchronisation, results are complete when the stream reaches the end of the call's work.
 *    Two calls that share a workspace must be ordered (same stream).
 *    The work of a call is kernel launches and, in one launch mode, device-to-device copies: no allocation, no
 *    memset.  A call can therefore be recorded into a HIP graph (stream capture) and replayed, provided the same
 *    call has been made once before outside a capture (the first launch of a kernel sets its attributes) and event
 *    timing is off.
 *  - Return value: SK_OK (0) or a negative error code.  Arguments are checked before anything is enqueued, so
 *    nothing is enqueued for SK_ERR_NULL .. SK_ERR_WORKSPACE; after SK_ERR_HIP (a launch was refused by the
 *    runtime) the launches made before the failing one stay enqueued and the outputs are undefined.  Errors never
 *    throw or exit.  sigkernel_last_error() gives a thread-local message for the last non-zero return.
 *  - Empty batches (B = 0, N*M = 0) are a successful no-op.  A path with a single point (L = 1) has no
 *    increments: k = 1 and all gradients are 0.
 *  - flags: SK_FLAG_TIME_AUG appends the channel t_i = i/(L-1) to both paths on the fly (Section 4);
 *    gradients are returned for the original d channels only.  SK_FLAG_LEAD_LAG applies the lead-lag transform
 *    of Section 4 to both paths on the fly: a path of L points in R^d is treated as the path of 2L - 1 points in
 *    R^2d with lead_i = x[k] for i in {2k - 1, 2k} and lag_i = x[k] for i in {2k, 2k + 1} (lead channels first);
 *    neither the transformed paths nor their increments are formed (the sweep runs on the grid of the original
 *    increments with one more level of refinement, whose off-diagonal quadrants carry no increment product), and
 *    the gradients come back with respect to the original points.  With both flags the time channel is that of
 *    the transformed path, t_i = i/(2L - 2).  Dyadic orders then refine the 2 (L - 1) steps of the transformed path.
 */
#ifndef SIGKERNEL_H
#define SIGKERNEL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { SK_F32 = 0, SK_F64 = 1 } sk_dtype;

enum {
    SK_FLAG_TIME_AUG = 1,   /* append the channel t_i = i/(L-1) to both paths on the fly (Section 4) */
    SK_FLAG_BWD_REPLAY = 2, /* backward: replay forward segments instead of inverting Eq. (1); see sigkernel_bwd */
    SK_FLAG_LEAD_LAG = 8,   /* lead-lag transform of both paths on the fly (Section 4) */
    SK_FLAG_KEEP_FORWARD = 16, /* forward calls: leave the forward sweep in the workspace for the backward call
                                  (Section 3.4: the backward pass works on the forward pass's grid); see sigkernel_bwd */
    SK_FLAG_HAVE_FORWARD = 32, /* backward calls: the workspace holds the forward sweep a forward call kept */
    SK_FLAG_SHORT_WAITS = 4 /* diagnostic: a workgroup that waits for another one's progress gives up after a single
                               poll.  Exercises the path a wait that runs out takes: every kernel still ends normally
                               and the results of the call are NaN.  Only launches whose workgroups wait for each
                               other are affected (a few pairs of very long paths). */
};

enum {
    SK_OK = 0,
    SK_ERR_NULL = -1,      /* a required pointer is NULL */
    SK_ERR_SHAPE = -2,     /* L < 1, d < 1, negative batch, or (L-1) << lam does not fit in 31 bits */
    SK_ERR_DYADIC = -3,    /* lam1 or lam2 negative or above 20 */
    SK_ERR_DTYPE = -4,     /* dt is neither SK_F32 nor SK_F64; unknown flag bits */
    SK_ERR_WORKSPACE = -5, /* ws is NULL, misaligned or smaller than the query says */
    SK_ERR_HIP = -6        /* a HIP runtime call failed (message has the HIP error string) */
};

/* Operations for the workspace query. */
enum { SK_OP_FWD = 0, SK_OP_BWD = 1, SK_OP_GRAM = 2, SK_OP_GRAM_BWD = 3 };

/*
 * Bytes of device scratch the operation `op` needs.  Pure host arithmetic, no GPU required.
 * B_or_N is B for SK_OP_FWD / SK_OP_BWD (M ignored) and N for the Gram operations.  Returns 0 for
 * invalid arguments or empty batches.
 */
size_t sigkernel_workspace_bytes(int op, int64_t B_or_N, int64_t M, int64_t L1, int64_t L2, int64_t d,
                                 int lam1, int lam2, int flags, sk_dtype dt);

/*
 * Forward over a batch of pairs (Algorithm "CPU Algorithm for Signature Kernels", Eq. (1)):
 *   x[B,L1,d], y[B,L2,d]  ->  k[B],  k[b] = k(x[b], y[b]).
 */
int sigkernel_fwd(const void* x, const void* y, void* k, int64_t B, int64_t L1, int64_t L2, int64_t d,
                  int lam1, int lam2, int flags, sk_dtype dt, void* ws, size_t ws_bytes, void* stream);

/*
 * Backward over a batch of pairs (Section 3.4 and Algorithm "CPU Algorithm for Backpropagation through
 * Signature Kernels"): given grad_k[B] = dF/dk[b], writes
 *   grad_x[B,L1,d] = dF/dx,  grad_y[B,L2,d] = dF/dy   (either may be NULL = not wanted)
 * and, if k_out != NULL, k_out[B] = k(x[b], y[b]) (the forward values are recomputed inside).
 * By default the reverse sweep recovers the forward values it needs by inverting Eq. (1) between exact
 * checkpoints eight block steps apart (32 in one launch mode), and checks the recovered state against every
 * checkpoint and, at the left end of the grid, against the boundary value 1.  Increment inner products of order one
 * make the inverse recurrence ill-conditioned (it divides by B(p)): where the recovered state differs from the exact
 * one by more than 1e-11 of the largest forward value met along the row, the pair is left out of the gradient sums
 * and solved once more, in the same call, by the variant that replays forward segments, which has no such limit.
 * The gradients are therefore the exact ones of the scheme for any input (Section 3.4); such pairs only cost more
 * time (a few launch modes cannot tell which pair drifted and then solve every pair of the call again).
 * SK_FLAG_BWD_REPLAY selects the replaying variant for the whole call from the start: the choice for data sets
 * whose increments are large throughout.  sigkernel_describe says where in the workspace the call counts the
 * pairs it solved twice.
 *
 * A forward sweep that was kept (sigkernel_fwd then sigkernel_bwd; sigkernel_gram without, then with grad_K).
 * A training step makes the forward call and then the backward call on the same paths; the backward call then need
 * not sweep forward again.
 *  - The forward call with SK_FLAG_KEEP_FORWARD takes the workspace of the backward call and leaves the checkpoints
 *    of its sweep there.  That workspace is asked for with the flags: sigkernel_workspace_bytes for SK_OP_FWD /
 *    SK_OP_GRAM with SK_FLAG_KEEP_FORWARD, or for SK_OP_BWD / SK_OP_GRAM_BWD with SK_FLAG_HAVE_FORWARD (the same
 *    number).  It can be much larger than without the flags: launch modes that keep checkpoints per wavefront then
 *    keep them per pair.
 *  - The backward call with SK_FLAG_HAVE_FORWARD, the same workspace, the same arrays x and y, shapes, lam and other
 *    flags, and no other call on that workspace in between, runs the reverse sweep from them.  It leaves them as they
 *    are: it may be repeated, say with another grad_k.
 *  - The caller vouches for all of that.  What the library checks: a kept sweep is signed with a hash of the call's
 *    pointers x and y, shapes, lam, transformation flags and dtype; a backward call that sweeps forward itself in
 *    that workspace erases the signature (where it lays the workspace out in the same way); and a backward call
 *    whose own hash differs from the signature it finds returns NaN gradients.  Paths changed in place between the
 *    two calls, or another forward call on that workspace, are not noticed.
 *  - Launch modes without this form ignore both flags (the forward call runs as usual, the backward call sweeps
 *    forward itself), so results never depend on the flags; sigkernel_describe names the kernels either way.
 */
int sigkernel_bwd(const void* x, const void* y, const void* grad_k, void* grad_x, void* grad_y, void* k_out,
                  int64_t B, int64_t L1, int64_t L2, int64_t d, int lam1, int lam2, int flags, sk_dtype dt,
                  void* ws, size_t ws_bytes, void* stream);

/*
 * sigkernel_bwd for callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc) and have no workspace to hand in: the same operation, arguments and results as
 * sigkernel_bwd, with the scratch taken from an array of SK_STATIC_SCRATCH_BYTES bytes that is part of the library
 * (one copy per GPU, held until the process ends).  The call allocates and frees nothing.
 *  - Shapes whose sigkernel_workspace_bytes(SK_OP_BWD, ...) exceeds SK_STATIC_SCRATCH_BYTES are refused with
 *    SK_ERR_WORKSPACE (configuration-2-sized batches fit: 128 pairs of 256 points at dyadic order 1).
 *  - SK_FLAG_KEEP_FORWARD / SK_FLAG_HAVE_FORWARD are refused (SK_ERR_DTYPE): the scratch belongs to no caller.
 *  - Every call on a GPU uses that GPU's one array: calls that overlap on one GPU (two streams, two threads) race.
 *    Calls on one stream are ordered and safe; each call clears what it needs cleared.
 *  - The first call on a device looks the array's address up (hipGetSymbolAddress); make that call, like the first
 *    call of any kernel, outside a stream capture.
 */
#define SK_STATIC_SCRATCH_BYTES (64u << 20)
int sigkernel_bwd_static(const void* x, const void* y, const void* grad_k, void* grad_x, void* grad_y, void* k_out,
                         int64_t B, int64_t L1, int64_t L2, int64_t d, int lam1, int lam2, int flags, sk_dtype dt,
                         void* stream);

/*
 * Gram matrix (the N x M product set of Eq. (1) solves): X[N,L1,d], Y[M,L2,d] -> K[N,M] = k(X[n], Y[m]).
 * If grad_K[N,M] = dF/dK is not NULL, also
 *   grad_X[n] = sum_m grad_K[n,m] dk(X[n],Y[m])/dX[n],   grad_Y[m] = sum_n grad_K[n,m] dk(X[n],Y[m])/dY[m]
 * (either may be NULL).  K may be NULL when grad_K is given.  Y == X (same pointer, N == M, L1 == L2)
 * selects the symmetric case K(X,X): grad_X then receives the total derivative (both argument slots)
 * and grad_Y is ignored.
 */
int sigkernel_gram(const void* X, const void* Y, void* K, const void* grad_K, void* grad_X, void* grad_Y,
                   int64_t N, int64_t M, int64_t L1, int64_t L2, int64_t d, int lam1, int lam2, int flags,
                   sk_dtype dt, void* ws, size_t ws_bytes, void* stream);

/*
 * Squared maximum mean discrepancy between two sets of paths under the signature kernel, the kind of training
 * loss for generative models that the paper's abstract and Section 1 give as the motivation for differentiable
 * signature kernels (the gradients are the exact ones of Section 3.4):
 *   loss = mean_{n,n'} k(X[n], X[n']) - 2 mean_{n,m} k(X[n], Y[m]) + mean_{m,m'} k(Y[m], Y[m'])
 * (the biased estimate, diagonals included), X[N,L1,d], Y[M,L2,d], N, M >= 1.  loss is a device pointer to one
 * element.  If grad_X / grad_Y are not NULL they receive d loss / dX [N,L1,d] and d loss / dY [M,L2,d].
 * Three Gram computations (two of them symmetric: half of their pairs are solved) with constant upstream
 * weights that are generated on the device, then one reduction.  Same conventions as the other entry points;
 * the workspace size comes from sigkernel_mmd2_workspace_bytes (with_grads != 0 if any gradient is wanted).
 * SK_FLAG_KEEP_FORWARD and SK_FLAG_HAVE_FORWARD do not apply here (one call computes everything) and are refused.
 */
size_t sigkernel_mmd2_workspace_bytes(int64_t N, int64_t M, int64_t L1, int64_t L2, int64_t d, int lam1, int lam2,
                                      int flags, sk_dtype dt, int with_grads);
int sigkernel_mmd2(const void* X, const void* Y, void* loss, void* grad_X, void* grad_Y, int64_t N, int64_t M,
                   int64_t L1, int64_t L2, int64_t d, int lam1, int lam2, int flags, sk_dtype dt, void* ws,
                   size_t ws_bytes, void* stream);

/*
 * Benchmark support (no passage of the paper): while enabled, every sweep-kernel launch made by the
 * entry points above is bracketed by a HIP event pair recorded on the caller's stream.
 * sigkernel_event_timing(enable): 0 switches it off, any other value switches it on and is kept as a tag
 * with every launch recorded from then on (a benchmark that times several kinds of call tags them apart).
 * sigkernel_event_timing_read waits for the recorded launches to finish, returns the summed elapsed
 * milliseconds and the launch counts of the forward and the backward sweep kernels since the last
 * read (any pointer may be NULL), and releases the events; sigkernel_event_timing_read_tag does the same
 * for the launches recorded under one tag and leaves the others (tag 0: all of them).
 * Not for use under stream capture.
 */
int sigkernel_event_timing(int enable);
int sigkernel_event_timing_read_tag(int tag, double* fwd_ms, int* fwd_launches, double* bwd_ms, int* bwd_launches);
int sigkernel_event_timing_read(double* fwd_ms, int* fwd_launches, double* bwd_ms, int* bwd_launches);

/*
 * Diagnostics (no passage of the paper): writes a NUL-terminated, human-readable description of the launch
 * the library would make for this operation and shape into out (host memory, out_bytes >= 1; truncated if
 * too small): the launch mode, the name of the sweep kernel as a profiler reports it, grid and workgroup
 * size, LDS bytes per workgroup and the workspace size; kept_sweep_half (1: the launch is the forward half of
 * the backward pass, kept for the backward call; 2: its reverse half; 0: neither); lead_lag_form (none, or
 * checkerboard: the grid of the caller's increments swept with one more level of refinement whose off-diagonal
 * quadrants carry no increment product); second_launch_lds_bytes (backward calls: LDS per workgroup of the launch
 * that solves drifted pairs once more).  Same arguments as sigkernel_workspace_bytes.
 * Pure host arithmetic: no GPU call.  Returns SK_OK or a negative error code.
 */
int sigkernel_describe(int op, int64_t B_or_N, int64_t M, int64_t L1, int64_t L2, int64_t d, int lam1, int lam2,
                       int flags, sk_dtype dt, char* out, size_t out_bytes);

/* Thread-local, NUL-terminated message describing the last non-zero return on this thread. */
const char* sigkernel_last_error(void);

/* Library version string. */
const char* sigkernel_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SIGKERNEL_H */

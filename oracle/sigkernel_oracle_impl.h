/*
 * TEST INFRASTRUCTURE - not part of the product path.
 *
 * Plain CPU oracle for the signature kernel of two piecewise-linear paths and its exact discrete
 * gradients (paper Section 3: the Goursat PDE, the finite-difference scheme Eq. (1), Algorithm
 * "CPU Algorithm for Signature Kernels", the two adjoint relations of Section 3.4 and Algorithm
 * "CPU Algorithm for Backpropagation through Signature Kernels").
 *
 * This header is the body of the oracle for ONE scalar type. sigkernel_oracle.c includes it twice:
 * REAL = double (suffix _f64) and REAL = long double (suffix _f80, used only to arbitrate rounding).
 * Everything is the definition written out: full grids, row-major double loops, no blocking, no fusion,
 * no reordering.  Compile with -ffp-contract=off so that every operation rounds where it is written.
 *
 * Notation (paper Section 3.1): path x has L1 points in R^d, y has L2 points; lambda1, lambda2 are
 * the dyadic orders; the refined grid has m = 2^lambda1 (L1-1) by n = 2^lambda2 (L2-1) cells and
 * (m+1) x (n+1) nodes; Delta[a,b] = <x[a+1]-x[a], y[b+1]-y[b]>.
 *
 * Readings of the paper taken here (each is listed in the design document of this repository):
 *  - A(p) = 1 + p/2 + p^2/12 and B(p) = 1 - p^2/12 as in Eq. (1); the forward listing drops the 1/12.
 *  - a path of L points has L-1 increments, so the grid has 2^lambda (L-1) cells per side.
 *  - on the refined grid every segment is cut into 2^lambda equal pieces, hence the increment inner
 *    product of a refined cell is p = 2^-(lambda1+lambda2) Delta[i >> lambda1, j >> lambda2].
 *  - the y index of the lookup shifts by lambda2 (the forward listing prints lambda1 twice).
 *  - time augmentation appends the channel t_i = i/(L-1) as the last channel (Section 4).
 */

#define CAT_(a, b) a##b
#define CAT(a, b) CAT_(a, b)
#define FN(name) CAT(name, SUFFIX)

/* Section 4 (time augmentation) + first line of both listings: the (optionally augmented) path and
 * its increments.  out has (L-1) rows of de = d + (time_aug ? 1 : 0) entries. */
static void FN(increments)(const REAL* x, long L, long d, int time_aug, REAL* out)
{
    long de = d + (time_aug ? 1 : 0);
    REAL* path = (REAL*)malloc(sizeof(REAL) * (size_t)(L > 0 ? L : 1) * (size_t)de);
    for (long i = 0; i < L; ++i) {
        for (long c = 0; c < d; ++c) path[i * de + c] = x[i * d + c];
        if (time_aug) path[i * de + d] = (L > 1) ? (REAL)i / (REAL)(L - 1) : (REAL)0;
    }
    for (long a = 0; a + 1 < L; ++a)
        for (long c = 0; c < de; ++c) out[a * de + c] = path[(a + 1) * de + c] - path[a * de + c];
    free(path);
}

/* Eq. (1), third line: Delta = dx dy^T, one inner product per coarse cell. */
static void FN(delta_from_increments)(const REAL* dx, const REAL* dy, long r, long q, long de, REAL* Delta)
{
    for (long a = 0; a < r; ++a)
        for (long b = 0; b < q; ++b) {
            REAL s = 0;
            for (long c = 0; c < de; ++c) s += dx[a * de + c] * dy[b * de + c];
            Delta[a * q + b] = s;
        }
}

static REAL FN(coefA)(REAL p) { return (REAL)1 + p / (REAL)2 + p * p / (REAL)12; }
static REAL FN(coefB)(REAL p) { return (REAL)1 - p * p / (REAL)12; }

/* Refined-cell inner product: dyadic refinement applied on the fly (Section 3.2, choice (3)). */
static REAL FN(cell_p)(const REAL* Delta, long q, int lam1, int lam2, REAL sc, long i, long j)
{
    return sc * Delta[(i >> lam1) * q + (j >> lam2)];
}

/* Eq. (1) over the whole refined grid.  Delta is r x q (coarse); grid is (m+1) x (n+1), row-major,
 * m = r << lam1, n = q << lam2.  Boundary condition k(0,.) = k(.,0) = 1. */
static void FN(solve_grid)(const REAL* Delta, long r, long q, int lam1, int lam2, REAL* grid)
{
    long m = r << lam1, n = q << lam2;
    REAL sc = (REAL)1 / (REAL)((long)1 << (lam1 + lam2));
    for (long j = 0; j <= n; ++j) grid[j] = 1;
    for (long i = 0; i <= m; ++i) grid[i * (n + 1)] = 1;
    for (long i = 0; i < m; ++i)
        for (long j = 0; j < n; ++j) {
            REAL p = FN(cell_p)(Delta, q, lam1, lam2, sc, i, j);
            grid[(i + 1) * (n + 1) + (j + 1)] =
                (grid[(i + 1) * (n + 1) + j] + grid[i * (n + 1) + (j + 1)]) * FN(coefA)(p)
                - grid[i * (n + 1) + j] * FN(coefB)(p);
        }
}

/* The two adjoint relations of Section 3.4 on a refined grid.  gk = dF/dk[m,n].  Output G = dF/dDelta
 * (r x q, overwritten).  g holds dF/dk at the nodes; it lives on an (m+2) x (n+2) array so that the
 * "zero outside the grid" convention of the paper needs no branches. */
static void FN(adjoint_grid)(const REAL* Delta, long r, long q, int lam1, int lam2, const REAL* grid,
                             REAL gk, REAL* G)
{
    long m = r << lam1, n = q << lam2;
    REAL sc = (REAL)1 / (REAL)((long)1 << (lam1 + lam2));
    long w = n + 2;
    REAL* g = (REAL*)calloc((size_t)(m + 2) * (size_t)w, sizeof(REAL));
    for (long t = 0; t < r * q; ++t) G[t] = 0;
    if (m == 0 || n == 0) { free(g); return; }
    for (long i = m; i >= 1; --i)
        for (long j = n; j >= 1; --j) {
            if (i == m && j == n) {
                g[i * w + j] = gk;
            } else {
                /* node (i,j) feeds node (i+1,j) through cell (i,j-1), node (i,j+1) through cell (i-1,j)
                 * and node (i+1,j+1) through cell (i,j); a term is present only if its target exists. */
                REAL s = 0;
                if (i < m) s += g[(i + 1) * w + j] * FN(coefA)(FN(cell_p)(Delta, q, lam1, lam2, sc, i, j - 1));
                if (j < n) s += g[i * w + (j + 1)] * FN(coefA)(FN(cell_p)(Delta, q, lam1, lam2, sc, i - 1, j));
                if (i < m && j < n)
                    s -= g[(i + 1) * w + (j + 1)] * FN(coefB)(FN(cell_p)(Delta, q, lam1, lam2, sc, i, j));
                g[i * w + j] = s;
            }
            /* second relation: derivative of the cell whose output node is (i,j), chained through
             * p = sc * Delta and summed over the refined cells of one coarse cell. */
            REAL p = FN(cell_p)(Delta, q, lam1, lam2, sc, i - 1, j - 1);
            REAL kl = grid[i * (n + 1) + (j - 1)];
            REAL ku = grid[(i - 1) * (n + 1) + j];
            REAL kd = grid[(i - 1) * (n + 1) + (j - 1)];
            G[((i - 1) >> lam1) * q + ((j - 1) >> lam2)] +=
                sc * g[i * w + j] * ((kl + ku) * ((REAL)1 / (REAL)2 + p / (REAL)6) + kd * p / (REAL)6);
        }
    free(g);
}

/* Linear map from dF/dDelta to dF/dx and dF/dy (Section 3.4: "a linear transformation"):
 * dF/d(dx)[a,c] = sum_b G[a,b] dy[b,c]; dF/d(dy)[b,c] = sum_a G[a,b] dx[a,c]; since dx[a] = x[a+1]-x[a],
 * dF/dx[i] = dF/d(dx)[i-1] - dF/d(dx)[i] with out-of-range terms zero.  The time channel is dropped.
 * gx, gy are ACCUMULATED into with weight 1 (caller zeroes them). */
static void FN(map_to_paths)(const REAL* G, const REAL* dx, const REAL* dy, long L1, long L2, long d, long de,
                             REAL* gx, REAL* gy)
{
    long r = L1 - 1, q = L2 - 1;
    if (gx) {
        REAL* gdx = (REAL*)calloc((size_t)(r > 0 ? r : 1) * (size_t)de, sizeof(REAL));
        for (long a = 0; a < r; ++a)
            for (long c = 0; c < de; ++c) {
                REAL s = 0;
                for (long b = 0; b < q; ++b) s += G[a * q + b] * dy[b * de + c];
                gdx[a * de + c] = s;
            }
        for (long i = 0; i < L1; ++i)
            for (long c = 0; c < d; ++c) {
                REAL hi = (i >= 1) ? gdx[(i - 1) * de + c] : (REAL)0;
                REAL lo = (i < r) ? gdx[i * de + c] : (REAL)0;
                gx[i * d + c] += hi - lo;
            }
        free(gdx);
    }
    if (gy) {
        REAL* gdy = (REAL*)calloc((size_t)(q > 0 ? q : 1) * (size_t)de, sizeof(REAL));
        for (long b = 0; b < q; ++b)
            for (long c = 0; c < de; ++c) {
                REAL s = 0;
                for (long a = 0; a < r; ++a) s += G[a * q + b] * dx[a * de + c];
                gdy[b * de + c] = s;
            }
        for (long j = 0; j < L2; ++j)
            for (long c = 0; c < d; ++c) {
                REAL hi = (j >= 1) ? gdy[(j - 1) * de + c] : (REAL)0;
                REAL lo = (j < q) ? gdy[j * de + c] : (REAL)0;
                gy[j * d + c] += hi - lo;
            }
        free(gdy);
    }
}

/* One pair, everything: k, optionally dF/dDelta (Gout, r x q), optionally gx/gy accumulated with the
 * pair's weight gk folded in (the adjoint is linear in gk).  grid_out, if given, receives the grid. */
static REAL FN(pair)(const REAL* x, const REAL* y, long L1, long L2, long d, int lam1, int lam2, int time_aug,
                     int want_grad, REAL gk, REAL* gx, REAL* gy, REAL* Gout, REAL* grid_out)
{
    long de = d + (time_aug ? 1 : 0);
    long r = L1 - 1, q = L2 - 1;
    if (r <= 0 || q <= 0) return 1; /* no increments: the signature is trivial, k = 1, zero gradients */
    long m = r << lam1, n = q << lam2;
    REAL* dx = (REAL*)malloc(sizeof(REAL) * (size_t)r * (size_t)de);
    REAL* dy = (REAL*)malloc(sizeof(REAL) * (size_t)q * (size_t)de);
    REAL* Delta = (REAL*)malloc(sizeof(REAL) * (size_t)r * (size_t)q);
    REAL* grid = (REAL*)malloc(sizeof(REAL) * (size_t)(m + 1) * (size_t)(n + 1));
    FN(increments)(x, L1, d, time_aug, dx);
    FN(increments)(y, L2, d, time_aug, dy);
    FN(delta_from_increments)(dx, dy, r, q, de, Delta);
    FN(solve_grid)(Delta, r, q, lam1, lam2, grid);
    REAL k = grid[m * (n + 1) + n];
    if (grid_out) memcpy(grid_out, grid, sizeof(REAL) * (size_t)(m + 1) * (size_t)(n + 1));
    if (want_grad) {
        REAL* G = (REAL*)malloc(sizeof(REAL) * (size_t)r * (size_t)q);
        FN(adjoint_grid)(Delta, r, q, lam1, lam2, grid, gk, G);
        if (Gout) memcpy(Gout, G, sizeof(REAL) * (size_t)r * (size_t)q);
        FN(map_to_paths)(G, dx, dy, L1, L2, d, de, gx, gy);
        free(G);
    }
    free(dx); free(dy); free(Delta); free(grid);
    return k;
}

/* ---- exported entry points (host pointers, dense row-major, caller owns everything) ---- */

/* Kernel from a given coarse Delta (r x q): used by tests to difference with respect to Delta. */
REAL FN(osk_kernel_from_delta)(const REAL* Delta, long r, long q, int lam1, int lam2)
{
    if (r <= 0 || q <= 0) return 1;
    long m = r << lam1, n = q << lam2;
    REAL* grid = (REAL*)malloc(sizeof(REAL) * (size_t)(m + 1) * (size_t)(n + 1));
    FN(solve_grid)(Delta, r, q, lam1, lam2, grid);
    REAL k = grid[m * (n + 1) + n];
    free(grid);
    return k;
}

/* One pair with all intermediate results exposed: Delta_out (r x q), grid_out ((m+1) x (n+1)),
 * G_out = dk/dDelta for gk = 1 (r x q); any may be NULL. Returns k. */
REAL FN(osk_pair_debug)(const REAL* x, const REAL* y, long L1, long L2, long d, int lam1, int lam2, int flags,
                        REAL* Delta_out, REAL* grid_out, REAL* G_out)
{
    int ta = flags & 1;
    if (Delta_out && L1 > 1 && L2 > 1) {
        long de = d + ta, r = L1 - 1, q = L2 - 1;
        REAL* dx = (REAL*)malloc(sizeof(REAL) * (size_t)r * (size_t)de);
        REAL* dy = (REAL*)malloc(sizeof(REAL) * (size_t)q * (size_t)de);
        FN(increments)(x, L1, d, ta, dx);
        FN(increments)(y, L2, d, ta, dy);
        FN(delta_from_increments)(dx, dy, r, q, de, Delta_out);
        free(dx); free(dy);
    }
    return FN(pair)(x, y, L1, L2, d, lam1, lam2, ta, G_out != NULL, (REAL)1, NULL, NULL, G_out, grid_out);
}

/* Batch of pairs, forward: x[B,L1,d], y[B,L2,d] -> k[B]. */
int FN(osk_fwd)(const REAL* x, const REAL* y, REAL* k, long B, long L1, long L2, long d, int lam1, int lam2,
                int flags)
{
    int ta = flags & 1;
#pragma omp parallel for schedule(dynamic, 1)
    for (long b = 0; b < B; ++b)
        k[b] = FN(pair)(x + b * L1 * d, y + b * L2 * d, L1, L2, d, lam1, lam2, ta, 0, (REAL)0, NULL, NULL, NULL,
                        NULL);
    return 0;
}

/* Batch of pairs, backward: grad_k[B] -> grad_x[B,L1,d], grad_y[B,L2,d] (either may be NULL), k_out[B]
 * optional.  Outputs are overwritten. */
int FN(osk_bwd)(const REAL* x, const REAL* y, const REAL* grad_k, REAL* grad_x, REAL* grad_y, REAL* k_out,
                long B, long L1, long L2, long d, int lam1, int lam2, int flags)
{
    int ta = flags & 1;
#pragma omp parallel for schedule(dynamic, 1)
    for (long b = 0; b < B; ++b) {
        REAL* gx = grad_x ? grad_x + b * L1 * d : NULL;
        REAL* gy = grad_y ? grad_y + b * L2 * d : NULL;
        if (gx) for (long t = 0; t < L1 * d; ++t) gx[t] = 0;
        if (gy) for (long t = 0; t < L2 * d; ++t) gy[t] = 0;
        REAL k = FN(pair)(x + b * L1 * d, y + b * L2 * d, L1, L2, d, lam1, lam2, ta, 1, grad_k[b], gx, gy, NULL,
                          NULL);
        if (k_out) k_out[b] = k;
    }
    return 0;
}

/* Gram matrix K[N,M] = k(X[n], Y[m]); if grad_K != NULL also
 * grad_X[n] = sum_m grad_K[n,m] dk(X[n],Y[m])/dX[n], grad_Y[m] = sum_n grad_K[n,m] dk(X[n],Y[m])/dY[m].
 * If Y == X (same pointer) both contributions are summed into grad_X (total derivative) and grad_Y is
 * not touched.  Rows are distributed over threads; each thread keeps a private grad_Y and the
 * privates are summed in thread order at the end. */
int FN(osk_gram)(const REAL* X, const REAL* Y, REAL* K, const REAL* grad_K, REAL* grad_X, REAL* grad_Y, long N,
                 long M, long L1, long L2, long d, int lam1, int lam2, int flags)
{
    int ta = flags & 1;
    int sym = (X == Y);
    if (!grad_K) {
#pragma omp parallel for schedule(dynamic, 1)
        for (long nm = 0; nm < N * M; ++nm) {
            long n_ = nm / M, m_ = nm % M;
            K[nm] = FN(pair)(X + n_ * L1 * d, Y + m_ * L2 * d, L1, L2, d, lam1, lam2, ta, 0, (REAL)0, NULL, NULL,
                             NULL, NULL);
        }
        return 0;
    }
    int nthreads = 1;
#ifdef _OPENMP
    nthreads = omp_get_max_threads();
#endif
    size_t ysz = (size_t)M * (size_t)L2 * (size_t)d;
    REAL* priv = (REAL*)calloc((size_t)nthreads * (ysz > 0 ? ysz : 1), sizeof(REAL));
    if (grad_X) for (long t = 0; t < N * L1 * d; ++t) grad_X[t] = 0;
#pragma omp parallel
    {
        int tid = 0;
#ifdef _OPENMP
        tid = omp_get_thread_num();
#endif
        REAL* mygy = priv + (size_t)tid * ysz;
#pragma omp for schedule(static)
        for (long n_ = 0; n_ < N; ++n_) {
            for (long m_ = 0; m_ < M; ++m_) {
                REAL* gx = grad_X ? grad_X + n_ * L1 * d : NULL;
                REAL* gy = (sym ? (grad_X != NULL) : (grad_Y != NULL)) ? mygy + m_ * L2 * d : NULL;
                REAL k = FN(pair)(X + n_ * L1 * d, Y + m_ * L2 * d, L1, L2, d, lam1, lam2, ta, 1,
                                  grad_K[n_ * M + m_], gx, gy, NULL, NULL);
                if (K) K[n_ * M + m_] = k;
            }
        }
    }
    REAL* dst = sym ? grad_X : grad_Y;
    if (dst) {
        if (!sym) for (size_t t = 0; t < ysz; ++t) dst[t] = 0;
        for (int th = 0; th < nthreads; ++th)
            for (size_t t = 0; t < ysz; ++t) dst[t] += priv[(size_t)th * ysz + t];
    }
    free(priv);
    return 0;
}

#undef FN
#undef CAT
#undef CAT_

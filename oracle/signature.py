"""TEST INFRASTRUCTURE - not part of the product path.

CPU oracle for batched truncated signatures (paper Section 2), in float64 numpy.  Only ``tests/``,
``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of ``bench.py`` may import this module.  It shares no code
with the HIP path.

The truncated signature of a piecewise-linear path has a plain definition (the iterated integrals of Definition 2.1
up to level N), and Section 2.1 gives the two facts that evaluate it exactly: the signature of one linear segment is
the tensor exponential of its increment (Proposition 2.1), and the signature of a concatenation is the tensor product
of the signatures (Chen's identity, Proposition 2.2).  This module writes those two facts out, segment by segment,
with full truncated tensor products: no Horner nesting, no in-place updates, no reordering.  The direct algorithm
and Horner's algorithm of Sections 2.2 and 2.3 reach the same numbers up to rounding order.

Layout of a result: the levels 0..N flattened one after the other (level 0 is the single number 1), each level in
row-major order of its word (i_1, ..., i_k), i_k fastest: (d^(N+1) - 1)/(d - 1) numbers per path.

Path transformations (Section 4) are applied by forming the transformed path explicitly before anything else.
"""
import numpy as np

FLAG_TIME_AUG = 1
FLAG_LEAD_LAG = 8


def sig_length(d, N):
    """Number of entries of a signature truncated at level N over d channels, level 0 included."""
    return sum(d ** k for k in range(N + 1))


def time_augment(x):
    """x[..., L, d] -> [..., L, d + 1]: the channel t_i = i/(L - 1) appended (Section 4; the points are taken as
    equally spaced on [0, 1]; a path of one point gets t = 0)."""
    x = np.asarray(x, dtype=np.float64)
    L = x.shape[-2]
    t = np.arange(L, dtype=np.float64) / max(L - 1, 1)
    t = np.broadcast_to(t.reshape((1,) * (x.ndim - 2) + (L, 1)), x.shape[:-1] + (1,))
    return np.concatenate([x, t], axis=-1)


def lead_lag(x):
    """Section 4: a path of L points in R^d becomes the path of 2L - 1 points in R^2d with
    lead_i = x[k] for i in {2k - 1, 2k} and lag_i = x[k] for i in {2k, 2k + 1}, lead channels first."""
    x = np.asarray(x, dtype=np.float64)
    L, d = x.shape[-2], x.shape[-1]
    out = np.empty(x.shape[:-2] + (2 * L - 1, 2 * d), dtype=np.float64)
    for i in range(2 * L - 1):
        out[..., i, :d] = x[..., (i + 1) // 2, :]
        out[..., i, d:] = x[..., i // 2, :]
    return out


def transform(x, flags):
    """Lead-lag first, then the time channel of the transformed path."""
    if flags & FLAG_LEAD_LAG:
        x = lead_lag(x)
    if flags & FLAG_TIME_AUG:
        x = time_augment(x)
    return np.asarray(x, dtype=np.float64)


def segment_levels(z, N):
    """Proposition 2.1: levels 0..N of exp(z) = sum_k z^(tensor k)/k! for the increment z of one linear segment."""
    levels = [np.ones(())]
    for k in range(1, N + 1):
        levels.append(np.multiply.outer(levels[k - 1], z) / k)
    return levels


def tensor_product(A, B, N):
    """Truncated product in the tensor algebra: level n of A (x) B is sum_{i + j = n} A_i (x) B_j."""
    return [sum(np.multiply.outer(A[i], B[n - i]) for i in range(n + 1)) for n in range(N + 1)]


def levels_of_path(path, N):
    """Levels 0..N of the signature of the piecewise-linear path through path[L, d] (Chen's identity, Proposition 2.2,
    applied segment after segment; a path of one point has the signature (1, 0, 0, ...))."""
    path = np.asarray(path, dtype=np.float64)
    L, d = path.shape
    S = segment_levels(np.zeros(d), N)
    for a in range(L - 1):
        S = tensor_product(S, segment_levels(path[a + 1] - path[a], N), N)
    return S


def flatten(levels):
    return np.concatenate([np.asarray(lv, dtype=np.float64).reshape(-1) for lv in levels])


def signature(x, N, flags=0):
    """x[B, L, d] -> [B, sig_length(d', N)], d' the number of channels after the transformations of `flags`."""
    x = np.asarray(x, dtype=np.float64)
    assert x.ndim == 3 and N >= 1
    xt = transform(x, flags)
    out = np.empty((x.shape[0], sig_length(xt.shape[-1], N)), dtype=np.float64)
    for b in range(x.shape[0]):
        out[b] = flatten(levels_of_path(xt[b], N))
    return out


# ---------------------------------------------------------------- gradients (Section 2.4)
# The gradient of F = <grad_out, S(x)> with respect to the points of x, by the chain rule through the same products
# the forward function performs, every intermediate signature kept (no time reversal, no deconstruction: those are
# ways to save memory that reach the same numbers).
def unflatten(flat, d, N):
    out, off = [], 0
    for k in range(N + 1):
        out.append(np.asarray(flat[off:off + d ** k], dtype=np.float64).reshape((d,) * k))
        off += d ** k
    return out


def lead_lag_pullback(g):
    """Chain rule through lead_lag: a point of the path is copied into the lead half of the transformed points
    2k - 1, 2k and into the lag half of 2k, 2k + 1.  g[..., 2L - 1, 2d] -> [..., L, d]."""
    g = np.asarray(g, dtype=np.float64)
    L, d = (g.shape[-2] + 1) // 2, g.shape[-1] // 2
    out = np.zeros(g.shape[:-2] + (L, d), dtype=np.float64)
    for i in range(2 * L - 1):
        out[..., (i + 1) // 2, :] += g[..., i, :d]
        out[..., i // 2, :] += g[..., i, d:]
    return out


def path_backward(path, grad_levels, N):
    """d <grad, S(path)> / d path for one path[L, D] (no transformations); grad_levels[k] has shape (D,)*k."""
    path = np.asarray(path, dtype=np.float64)
    L, D = path.shape
    S = [segment_levels(np.zeros(D), N)]
    for a in range(L - 1):
        S.append(tensor_product(S[a], segment_levels(path[a + 1] - path[a], N), N))
    G = [np.array(g, dtype=np.float64) for g in grad_levels]
    gz = np.zeros((max(L - 1, 0), D))
    for a in range(L - 2, -1, -1):
        z = path[a + 1] - path[a]
        E = segment_levels(z, N)
        P = S[a]                                   # signature before this segment: S[a + 1] = P (x) E
        # level n of the product is sum_i P_i (x) E_{n-i}: the adjoint of E_j collects P_i against G_{i+j} over the
        # first i indices, the adjoint of P_i collects G_{i+j} against E_j over the last j indices
        Ebar = [sum(np.tensordot(P[i], G[i + j], axes=i) for i in range(N - j + 1)) for j in range(N + 1)]
        Gprev = [sum(np.tensordot(G[i + j], E[j], axes=j) for j in range(N - i + 1)) for i in range(N + 1)]
        # E_j = E_{j-1} (x) z / j
        zbar = np.zeros(D)
        for j in range(N, 0, -1):
            zbar += np.tensordot(E[j - 1], Ebar[j], axes=j - 1) / j
            Ebar[j - 1] = Ebar[j - 1] + np.tensordot(Ebar[j], z, axes=([j - 1], [0])) / j
        gz[a] = zbar
        G = Gprev
    gp = np.zeros((L, D))
    for a in range(L - 1):                         # z_a = path[a + 1] - path[a]
        gp[a + 1] += gz[a]
        gp[a] -= gz[a]
    return gp


def signature_backward(x, grad_out, N, flags=0):
    """x[B, L, d], grad_out[B, sig_length(d', N)] -> d <grad_out, signature(x)> / dx  [B, L, d]."""
    x = np.asarray(x, dtype=np.float64)
    grad_out = np.asarray(grad_out, dtype=np.float64)
    B, L, d = x.shape
    xt = transform(x, flags)
    D = xt.shape[-1]
    assert grad_out.shape == (B, sig_length(D, N))
    out = np.empty_like(x)
    for b in range(B):
        g = path_backward(xt[b], unflatten(grad_out[b], D, N), N)
        if flags & FLAG_TIME_AUG:
            g = g[:, :-1]                          # the time channel does not depend on the path
        if flags & FLAG_LEAD_LAG:
            g = lead_lag_pullback(g)
        out[b] = g
    return out

"""Pins of the truncated-signature oracle (oracle/signature.py) to facts it does not compute itself: the iterated
integrals of Definition 2.1 evaluated by exact polynomial integration, closed forms for straight and axis-parallel
paths, the shuffle identities, the shoelace area of a polygon, and invariances.  No GPU needed."""
import itertools
import math

import numpy as np
import pytest
from numpy.polynomial import polynomial as npoly

from oracle import signature as osig


def level(flat, d, k):
    off = sum(d ** j for j in range(k))
    return flat[off:off + d ** k].reshape((d,) * k) if k > 0 else flat[0]


def iterated_integrals(path, N):
    """Definition 2.1 taken literally for a piecewise-linear path: I_w(t) = int_0^t I_{w minus last letter}(s) dx^{last}(s),
    I_empty = 1.  On each segment every I_w is a polynomial in the local time; numpy integrates it exactly."""
    path = np.asarray(path, dtype=np.float64)
    L, d = path.shape
    words = [w for k in range(N + 1) for w in itertools.product(range(d), repeat=k)]
    start = {w: (1.0 if len(w) == 0 else 0.0) for w in words}
    for a in range(L - 1):
        z = path[a + 1] - path[a]
        poly = {(): np.array([1.0])}
        for w in words[1:]:
            integ = npoly.polyint(poly[w[:-1]])               # integral from 0 of the shorter word's polynomial
            poly[w] = npoly.polyadd(np.array([start[w]]), z[w[-1]] * integ)
        start = {w: float(npoly.polyval(1.0, poly[w])) for w in words}
    return start


@pytest.mark.parametrize("L,d,N,seed", [(2, 2, 4, 1), (4, 2, 5, 2), (5, 3, 4, 3), (7, 4, 3, 4), (3, 1, 6, 5)])
def test_s1_signature_is_the_iterated_integrals(L, d, N, seed):
    rng = np.random.default_rng(seed)
    x = np.cumsum(rng.normal(0, 0.8, size=(L, d)), axis=0)
    flat = osig.signature(x[None], N)[0]
    assert flat.shape == (osig.sig_length(d, N),)
    I = iterated_integrals(x, N)
    for k in range(N + 1):
        lv = level(flat, d, k)
        for w in itertools.product(range(d), repeat=k):
            got = lv[w] if k > 0 else lv
            assert abs(got - I[w]) < 1e-12 * max(1.0, abs(I[w])), (w, got, I[w])


def test_s2_straight_line_closed_form():
    # A straight path from 0 to v, in any number of collinear pieces: S^(i1..ik) = v_i1 ... v_ik / k!
    v = np.array([0.7, -1.3, 0.4])
    for cuts in ([0.0, 1.0], [0.0, 0.25, 0.6, 1.0], [0.0, 0.5, 0.5, 1.0]):
        x = np.outer(np.array(cuts), v)
        flat = osig.signature(x[None], 5)[0]
        for k in range(1, 6):
            lv = level(flat, 3, k)
            for w in itertools.product(range(3), repeat=k):
                assert abs(lv[w] - np.prod(v[list(w)]) / math.factorial(k)) < 1e-14


def test_s2_axis_parallel_path_closed_form():
    # a along axis 0, then b along axis 1, then c along axis 2: the only words with a non-zero integral are
    # 0^p 1^q 2^r (letters in the order the axes are travelled), with value a^p b^q c^r / (p! q! r!).
    a, b, c = 1.5, -0.8, 0.6
    x = np.array([[0, 0, 0], [a, 0, 0], [a, b, 0], [a, b, c]], dtype=np.float64)
    N = 5
    flat = osig.signature(x[None], N)[0]
    for k in range(1, N + 1):
        lv = level(flat, 3, k)
        for w in itertools.product(range(3), repeat=k):
            if list(w) == sorted(w):
                p, q, r = w.count(0), w.count(1), w.count(2)
                want = a ** p * b ** q * c ** r / (math.factorial(p) * math.factorial(q) * math.factorial(r))
            else:
                want = 0.0
            assert abs(lv[w] - want) < 1e-14, (w, lv[w], want)


def test_s3_shuffle_identities_and_total_increment():
    rng = np.random.default_rng(7)
    d = 3
    x = np.cumsum(rng.normal(0, 0.6, size=(9, d)), axis=0)
    flat = osig.signature(x[None], 3)[0]
    S1, S2, S3 = level(flat, d, 1), level(flat, d, 2), level(flat, d, 3)
    assert flat[0] == 1.0
    assert np.allclose(S1, x[-1] - x[0], atol=1e-14)
    for i, j in itertools.product(range(d), repeat=2):
        assert abs(S1[i] * S1[j] - (S2[i, j] + S2[j, i])) < 1e-13
    for i, j, k in itertools.product(range(d), repeat=3):
        assert abs(S1[i] * S2[j, k] - (S3[i, j, k] + S3[j, i, k] + S3[j, k, i])) < 1e-13


def test_s3_levy_area_of_a_closed_polygon_is_the_shoelace_area():
    rng = np.random.default_rng(8)
    pts = rng.normal(0, 1.0, size=(7, 2))
    x = np.concatenate([pts, pts[:1]], axis=0)
    S2 = level(osig.signature(x[None], 2)[0], 2, 2)
    shoelace = 0.5 * sum(x[i, 0] * x[i + 1, 1] - x[i + 1, 0] * x[i, 1] for i in range(len(x) - 1))
    assert abs(0.5 * (S2[0, 1] - S2[1, 0]) - shoelace) < 1e-13
    assert abs(S2[0, 1] + S2[1, 0]) < 1e-13          # closed path: the symmetric part vanishes


def test_s4_invariances():
    rng = np.random.default_rng(9)
    x = np.cumsum(rng.normal(0, 0.5, size=(6, 2)), axis=0)
    N = 4
    base = osig.signature(x[None], N)[0]
    # translation
    assert np.allclose(osig.signature((x + np.array([3.0, -2.0]))[None], N)[0], base, atol=1e-13)
    # a point inserted on a segment, and a repeated point
    mid = np.insert(x, 3, 0.3 * x[2] + 0.7 * x[3], axis=0)
    assert np.allclose(osig.signature(mid[None], N)[0], base, atol=1e-13)
    rep = np.insert(x, 2, x[2], axis=0)
    assert np.allclose(osig.signature(rep[None], N)[0], base, atol=1e-13)
    # scaling the path by c scales level k by c^k
    sc = osig.signature((2.0 * x)[None], N)[0]
    for k in range(N + 1):
        assert np.allclose(level(sc, 2, k), 2.0 ** k * level(base, 2, k), atol=1e-12)
    # the reversed path has the reversed words with sign (-1)^k  (the antipode)
    rev = osig.signature(x[::-1][None], N)[0]
    for k in range(1, N + 1):
        want = (-1) ** k * np.transpose(level(base, 2, k), axes=tuple(range(k - 1, -1, -1)))
        assert np.allclose(level(rev, 2, k), want, atol=1e-13)
    # batch entries are independent, one-point paths give (1, 0, ...)
    two = osig.signature(np.stack([x, 2.0 * x]), N)
    assert np.array_equal(two[0], base) and np.array_equal(two[1], sc)
    one = osig.signature(np.zeros((2, 1, 3)), 3)
    assert one.shape == (2, 40) and np.array_equal(one[:, 0], [1.0, 1.0]) and not one[:, 1:].any()


def test_s5_time_augmentation_and_lead_lag_flags():
    rng = np.random.default_rng(10)
    L, d = 6, 2
    x = np.cumsum(rng.normal(0, 0.7, size=(L, d)), axis=0)
    # time channel: total increment 1, and int x dt + int t dx = x_T - x_0 (integration by parts)
    flat = osig.signature(x[None], 2, flags=osig.FLAG_TIME_AUG)[0]
    S1, S2 = level(flat, 3, 1), level(flat, 3, 2)
    assert abs(S1[2] - 1.0) < 1e-15 and abs(S2[2, 2] - 0.5) < 1e-15
    for c in range(d):
        assert abs(S2[c, 2] + S2[2, c] - (x[-1, c] - x[0, c])) < 1e-14
        # int_0^1 (x_t - x_0) dt by the trapezoid rule, exact for a piecewise-linear path on the equally spaced grid
        trap = sum(0.5 * ((x[i, c] - x[0, c]) + (x[i + 1, c] - x[0, c])) / (L - 1) for i in range(L - 1))
        assert abs(S2[c, 2] - trap) < 1e-14
    # lead-lag: the second level picks up the quadratic variation, S^(lead_c, lag_c) - S^(lag_c, lead_c) = sum dx_c^2
    flat = osig.signature(x[None], 2, flags=osig.FLAG_LEAD_LAG)[0]
    S1, S2 = level(flat, 2 * d, 1), level(flat, 2 * d, 2)
    dx = np.diff(x, axis=0)
    for c in range(d):
        assert abs((S2[c, d + c] - S2[d + c, c]) - np.sum(dx[:, c] ** 2)) < 1e-13
    assert np.allclose(S1[:d], x[-1] - x[0]) and np.allclose(S1[d:], x[-1] - x[0])
    # both flags: the time channel is that of the transformed path (last channel, total increment 1)
    flat = osig.signature(x[None], 2, flags=osig.FLAG_LEAD_LAG | osig.FLAG_TIME_AUG)[0]
    assert flat.shape == (1 + 5 + 25,) and abs(level(flat, 5, 1)[4] - 1.0) < 1e-15
    xt = osig.transform(x, osig.FLAG_LEAD_LAG | osig.FLAG_TIME_AUG)
    assert xt.shape == (2 * L - 1, 5) and np.allclose(np.diff(xt[:, 4]), 1.0 / (2 * L - 2))


# ---------------------------------------------------------------- gradients (Section 2.4)
def fd_gradient(x, g, N, flags, h=1e-6):
    """Central differences of F = <g, signature(x)> (forward function only)."""
    out = np.zeros_like(x)
    for idx in np.ndindex(*x.shape):
        xp, xm = x.copy(), x.copy()
        xp[idx] += h
        xm[idx] -= h
        out[idx] = (np.sum(g * osig.signature(xp[None], N, flags)[0]) - np.sum(g * osig.signature(xm[None], N, flags)[0])) / (2 * h)
    return out


@pytest.mark.parametrize("L,d,N,flags", [(4, 2, 4, 0), (5, 3, 3, 0), (2, 2, 5, 0), (4, 2, 3, osig.FLAG_TIME_AUG),
                                         (4, 2, 3, osig.FLAG_LEAD_LAG), (3, 2, 2, osig.FLAG_LEAD_LAG | osig.FLAG_TIME_AUG)])
def test_s6_gradient_vs_central_differences(L, d, N, flags):
    rng = np.random.default_rng(60 + L + d + N + flags)
    x = np.cumsum(rng.normal(0, 0.6, size=(L, d)), axis=0)
    n = osig.sig_length(osig.transform(x, flags).shape[-1], N)
    g = rng.normal(0, 1.0, size=n)
    got = osig.signature_backward(x[None], g[None], N, flags)[0]
    ref = fd_gradient(x, g, N, flags)
    assert np.max(np.abs(got - ref)) < 2e-8 * max(1.0, np.max(np.abs(ref)))


def test_s6_gradient_closed_forms_and_invariants():
    rng = np.random.default_rng(66)
    L, d, N = 6, 2, 3
    x = np.cumsum(rng.normal(0, 0.7, size=(L, d)), axis=0)
    n = osig.sig_length(d, N)
    # level 1 is the total increment: its gradient is -1 at the first point and +1 at the last one
    for c in range(d):
        g = np.zeros(n)
        g[1 + c] = 1.0
        gx = osig.signature_backward(x[None], g[None], N)[0]
        want = np.zeros((L, d))
        want[0, c], want[-1, c] = -1.0, 1.0
        assert np.allclose(gx, want, atol=1e-14)
    # the Levy area (S^01 - S^10)/2 = 1/2 sum_i (x_i^0 x_{i+1}^1 - x_{i+1}^0 x_i^1) - 1/2 (x_0^0 x_L^1 - x_L^0 x_0^1)
    # (shoelace of the polygon closed by the chord), differentiated by hand
    g = np.zeros(n)
    g[1 + d + 1], g[1 + d + d] = 0.5, -0.5
    gx = osig.signature_backward(x[None], g[None], N)[0]
    want = np.zeros((L, d))
    for i in range(L):
        nxt = x[i + 1] if i + 1 < L else None
        prv = x[i - 1] if i > 0 else None
        if nxt is not None:
            want[i, 0] += 0.5 * nxt[1]
            want[i, 1] -= 0.5 * nxt[0]
        if prv is not None:
            want[i, 1] += 0.5 * prv[0]
            want[i, 0] -= 0.5 * prv[1]
    want[0, 0] -= 0.5 * x[-1, 1]
    want[0, 1] += 0.5 * x[-1, 0]
    want[-1, 1] -= 0.5 * x[0, 0]
    want[-1, 0] += 0.5 * x[0, 1]
    assert np.allclose(gx, want, atol=1e-13)
    # translation invariance: the gradients of the points sum to zero; level 0 has no gradient; linear in grad_out
    g1, g2 = rng.normal(size=n), rng.normal(size=n)
    a = osig.signature_backward(x[None], g1[None], N)[0]
    b = osig.signature_backward(x[None], g2[None], N)[0]
    assert np.max(np.abs(a.sum(axis=0))) < 1e-12
    assert np.allclose(osig.signature_backward(x[None], (2.0 * g1 - 3.0 * g2)[None], N)[0], 2.0 * a - 3.0 * b, atol=1e-12)
    g0 = np.zeros(n)
    g0[0] = 5.0
    assert not osig.signature_backward(x[None], g0[None], N)[0].any()
    # batch entries are independent; one-point paths have zero gradient
    both = osig.signature_backward(np.stack([x, 2.0 * x]), np.stack([g1, g2]), N)
    assert np.array_equal(both[0], a)
    assert not osig.signature_backward(np.zeros((2, 1, 3)), np.ones((2, 40)), 3).any()

"""GPU parity of the gradient of truncated signatures (signature_bwd through the C ABI) against the CPU oracle
(oracle/signature.py: chain rule with every intermediate signature kept), on the same seeded inputs.

Tolerance: fp64 1e-10, fp32 1e-4, in the sense max|gpu - ref| <= tol * max(1, max|ref|) per gradient tensor (entries
cross zero, so they are compared against the tensor's scale).  fp32 runs compute in double from the fp32-rounded
inputs and are compared with the oracle on those inputs.
"""
import os
import re

import numpy as np
import pytest
import torch

from oracle import signature as osig
from paper_2509_10613_amd import binding as sk
from paper_2509_10613_amd import workloads

pytestmark = pytest.mark.gpu

TOL = {torch.float64: 1e-10, torch.float32: 1e-4}


def dev(a, dtype=torch.float64):
    return torch.tensor(np.asarray(a), dtype=dtype, device="cuda")


def host(t):
    return t.detach().cpu().numpy().astype(np.float64)


def paths(seed, B, L, d, scale=0.4):
    rng = np.random.default_rng(seed)
    return np.cumsum(rng.normal(0, scale, size=(B, L, d)), axis=1)


def check(X, N, flags=0, dtype=torch.float64, give_sig=False, seed=3):
    B, L, d = X.shape
    tflags = flags & (sk.SK_FLAG_TIME_AUG | sk.SK_FLAG_LEAD_LAG)
    n = sk.signature_length(d, N, tflags)
    G = np.random.default_rng(seed).normal(0, 1.0, size=(B, n))
    x, g = dev(X, dtype), dev(G, dtype)
    print("signature_bwd B=%d L=%d d=%d N=%d flags=%d %s sig=%s: %s" % (
        B, L, d, N, flags, dtype, give_sig,
        sk.signature_bwd_describe(B, L, d, N, flags, sk.SK_F64 if dtype == torch.float64 else sk.SK_F32)), flush=True)
    sig = sk.signature_fwd(x, N, tflags) if give_sig else None
    got = host(sk.signature_bwd(x, g, N, flags, sig=sig))
    torch.cuda.synchronize()
    ref = osig.signature_backward(host(x), host(g), N, tflags)
    assert got.shape == ref.shape and np.all(np.isfinite(got))
    scale = max(1.0, np.max(np.abs(ref))) if ref.size else 1.0
    err = (np.max(np.abs(got - ref)) if ref.size else 0.0) / scale
    print("  max err / scale %.3e (scale %.3g, tol %.0e)" % (err, scale, TOL[dtype]), flush=True)
    assert err <= TOL[dtype]
    return got


def bwd_variants():
    hdr = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2509_10613_amd", "csrc", "sg_plan.h")
    text = open(hdr).read()
    body = text[text.index("#define SG_BWD_VARIANTS(X)"):text.index("constexpr int kBwdLongPrefixMaxD")]
    return [tuple(int(v) for v in m) for m in re.findall(r"X\((\d+), (\d+), (\d+)\)", body)]


@pytest.mark.parametrize("D,M,S", bwd_variants())
def test_every_backward_kernel_variant(D, M, S):
    for Q in (0, 1, 2, 3, 4, 6):
        N = M + 1 + Q
        if D ** N > (400000 if Q > 4 else 40000) or (Q > 4 and D > 5):
            continue
        L = 5 if D ** N < 5000 else 3
        force = sk.SK_SIG_DEPTH(M) | sk.SK_SIG_BLOCK(S)
        desc = sk.signature_bwd_describe(2, L, D, N, force, sk.SK_F64)
        assert "horner_bwd_kernel<%d, %d, %d, %d, " % (D, M, S, Q if Q <= 4 else 8) in desc, desc
        check(paths(2000 * D + 10 * M + Q, 2, L, D, 0.5), N, flags=force)
        if "paths_per_wave=1 " not in desc:     # the kernel whose waves hold one path each, too
            check(paths(2000 * D + 10 * M + Q, 2, L, D, 0.5), N, flags=force | sk.SK_SIG_ONE_PATH_PER_WAVE)


def test_backward_run_time_channel_kernel():
    for d, N in ((1, 4), (2, 4), (3, 3), (7, 3), (18, 2), (40, 2), (70, 1)):
        desc = sk.signature_bwd_describe(2, 6, d, N, sk.SK_SIG_DEPTH(0), sk.SK_F64)
        assert "horner_bwd_kernel<0, 0, 1," in desc, desc
        check(paths(88 + d, 2, 6, d), N, flags=sk.SK_SIG_DEPTH(0))


@pytest.mark.parametrize("B,L,d,N", [(3, 12, 2, 5), (2, 9, 3, 4), (2, 10, 4, 4), (2, 8, 5, 3), (2, 7, 8, 3), (1, 6, 16, 3),
                                     (3, 4, 2, 1), (2, 16, 6, 3), (130, 7, 3, 5)])
def test_backward_library_choice_and_given_signatures(B, L, d, N):
    a = check(paths(300 + d + N, B, L, d), N)
    b = check(paths(300 + d + N, B, L, d), N, give_sig=True)
    assert np.max(np.abs(a - b)) <= 1e-12 * max(1.0, np.max(np.abs(a)))


def test_backward_several_short_paths_share_a_wave():
    for (B, L, d, N) in ((50, 9, 2, 3), (7, 8, 2, 2), (64, 6, 3, 3), (13, 7, 3, 2), (33, 6, 4, 3), (9, 5, 5, 2), (21, 5, 8, 2),
                         (300, 6, 2, 4), (40, 6, 9, 2)):
        desc = sk.signature_bwd_describe(B, L, d, N, 0, sk.SK_F64)
        assert int(desc.split("paths_per_wave=")[1].split(" ")[0]) > 1, desc
        a = check(paths(700 + B + d, B, L, d), N)
        b = check(paths(700 + B + d, B, L, d), N, flags=sk.SK_SIG_ONE_PATH_PER_WAVE, give_sig=True)
        assert np.max(np.abs(a - b)) <= 1e-12 * max(1.0, np.max(np.abs(a)))
    check(paths(722, 11, 9, 2), 3, flags=sk.SK_FLAG_TIME_AUG)
    check(paths(723, 11, 9, 1), 3, flags=sk.SK_FLAG_LEAD_LAG | sk.SK_FLAG_TIME_AUG, dtype=torch.float32)
    check(paths(724, 3000, 10, 3, 0.3), 4)


@pytest.mark.parametrize("flags", [sk.SK_FLAG_TIME_AUG, sk.SK_FLAG_LEAD_LAG, sk.SK_FLAG_TIME_AUG | sk.SK_FLAG_LEAD_LAG])
def test_backward_with_path_transformations(flags):
    check(paths(21, 3, 9, 2), 4, flags)
    check(paths(22, 2, 6, 4), 3, flags, give_sig=True)
    check(paths(23, 2, 5, 8), 2, flags)


def test_backward_paths_cut_into_pieces():
    # forced: 2 .. 16 pieces per path, lengths that do not divide, pieces left empty, short and long sums in the
    # adjoints of the pair products (few and many channels, low and high levels); then the library's own choice
    for q, (B, L, d, N) in ((1, (3, 12, 2, 4)), (2, (2, 11, 3, 3)), (3, (2, 9, 3, 3)), (3, (2, 5, 4, 3)), (2, (2, 30, 5, 4)),
                            (1, (2, 10, 16, 3)), (4, (1, 70, 2, 6)), (2, (2, 2, 3, 3)), (2, (2, 14, 2, 9)), (1, (2, 9, 6, 5)),
                            (3, (2, 20, 1, 5)), (2, (3, 9, 20, 2))):
        desc = sk.signature_bwd_describe(B, L, d, N, sk.SK_SIG_PIECES(q), sk.SK_F64)
        assert "pieces_per_path=%d " % (1 << q) in desc, desc
        a = check(paths(800 + 10 * q + d, B, L, d), N, flags=sk.SK_SIG_PIECES(q))
        b = check(paths(800 + 10 * q + d, B, L, d), N, flags=sk.SK_SIG_PIECES(0))
        assert np.max(np.abs(a - b)) <= 1e-11 * max(1.0, np.max(np.abs(a)))
    check(paths(821, 2, 13, 2), 4, flags=sk.SK_SIG_PIECES(2) | sk.SK_FLAG_TIME_AUG | sk.SK_FLAG_LEAD_LAG)
    check(paths(822, 2, 13, 3), 3, flags=sk.SK_SIG_PIECES(2) | sk.SK_FLAG_LEAD_LAG, dtype=torch.float32)
    check(paths(823, 2, 13, 3), 3, flags=sk.SK_SIG_PIECES(1), give_sig=True)      # the given signatures are not needed
    for (B, L, d, N) in ((2, 400, 3, 3), (1, 1500, 2, 5), (3, 257, 5, 3)):
        desc = sk.signature_bwd_describe(B, L, d, N, 0, sk.SK_F64)
        assert int(desc.split("pieces_per_path=")[1].split(" ")[0]) > 1, desc
        check(paths(830 + d, B, L, d, 0.1), N)


def test_backward_float32():
    check(paths(31, 3, 12, 3), 4, dtype=torch.float32)
    check(paths(32, 2, 8, 16), 3, dtype=torch.float32, give_sig=True)
    check(paths(33, 2, 8, 2), 3, flags=sk.SK_FLAG_TIME_AUG | sk.SK_FLAG_LEAD_LAG, dtype=torch.float32)


def test_backward_degenerate_shapes_and_errors():
    got = check(paths(41, 3, 1, 3), 4)           # one point: no gradient
    assert not got.any()
    check(paths(42, 2, 2, 3), 5)                 # one segment
    out = sk.signature_bwd(torch.empty((0, 5, 3), dtype=torch.float64, device="cuda"),
                           torch.empty((0, 40), dtype=torch.float64, device="cuda"), 3)
    assert out.shape == (0, 5, 3)
    got = check(np.ones((2, 6, 4)), 3)           # a constant path still has a gradient (level 1: -g, 0, ..., +g)
    x = dev(paths(51, 2, 5, 3))
    g = dev(np.ones((2, 40)))
    with pytest.raises(sk.SigKernelError):
        sk.signature_bwd(x, g, 3, flags=2)
    with pytest.raises(sk.SigKernelError):
        sk.signature_bwd(x, g, 3, ws=torch.empty((256,), dtype=torch.uint8, device="cuda")[:16])
    check(paths(53, 2, 5, 3), 3)


@pytest.mark.parametrize("name", ["s1", "s2", "s3"])
def test_backward_benchmark_shapes_sampled(name):
    # full size of the Table 1 shapes: the oracle computes two paths; every path is checked for translation
    # invariance (the gradients of its points sum to zero) and against the closed form for the first level
    (B, L, d, N), X = workloads.make_signature(name)
    n = sk.signature_length(d, N, 0)
    rng = np.random.default_rng(9)
    G = rng.normal(0, 1.0, size=(B, n))
    x, g = dev(X), dev(G)
    print(name, sk.signature_bwd_describe(B, L, d, N, 0, sk.SK_F64), flush=True)
    got = host(sk.signature_bwd(x, g, N))
    torch.cuda.synchronize()
    assert got.shape == X.shape and np.all(np.isfinite(got))
    for b in (0, B - 1):
        ref = osig.signature_backward(X[b:b + 1], G[b:b + 1], N)[0]
        scale = max(1.0, np.max(np.abs(ref)))
        err = np.max(np.abs(got[b] - ref)) / scale
        print("  path %d: max err / scale %.3e (scale %.3g)" % (b, err, scale), flush=True)
        assert err <= 1e-10
    assert np.max(np.abs(got.sum(axis=1))) <= 1e-9 * max(1.0, np.max(np.abs(got)))
    # only level 1 upstream: gradient is -g at the first point, +g at the last, zero in between
    G1 = np.zeros((B, n))
    G1[:, 1:1 + d] = rng.normal(size=(B, d))
    got1 = host(sk.signature_bwd(x, dev(G1), N))
    assert np.max(np.abs(got1[:, 0] + G1[:, 1:1 + d])) <= 1e-10 and np.max(np.abs(got1[:, -1] - G1[:, 1:1 + d])) <= 1e-10
    assert np.max(np.abs(got1[:, 1:-1])) <= 1e-10


def test_autograd_wrapper_gives_the_oracle_gradient():
    from paper_2509_10613_amd import autograd as ag
    X = paths(71, 3, 7, 3)
    N = 4
    x = dev(X).requires_grad_(True)
    S = ag.signature(x, N)
    w = dev(np.random.default_rng(72).normal(size=S.shape))
    loss = (S * w).sum() + (S[:, 1:4] ** 2).sum()
    loss.backward()
    Sh = osig.signature(X, N)
    assert np.max(np.abs(host(S) - Sh)) <= 1e-10 * max(1.0, np.max(np.abs(Sh)))
    gout = host(w).copy()
    gout[:, 1:4] += 2.0 * Sh[:, 1:4]
    ref = osig.signature_backward(X, gout, N)
    assert np.max(np.abs(host(x.grad) - ref)) <= 1e-10 * max(1.0, np.max(np.abs(ref)))


@pytest.mark.parametrize("B,L,d,N", [(200000, 5, 2, 2), (3, 6001, 3, 3), (40000, 17, 3, 3), (6, 300, 6, 6), (2, 1500, 2, 9)])
def test_large_shapes_sampled_forward_and_backward(B, L, d, N):
    # sizes that stress the index arithmetic (many paths, long paths, many entries); the oracle computes three of
    # the paths, every path is checked for the level-1 identity and for translation invariance of the gradient
    rng = np.random.default_rng(B + L)
    X = np.cumsum(rng.normal(0, 1.0 / np.sqrt(L), size=(B, L, d)), axis=1)
    n = sk.signature_length(d, N, 0)
    G = rng.normal(0, 1.0, size=(B, n))
    x, g = dev(X), dev(G)
    print(sk.signature_describe(B, L, d, N, 0, sk.SK_F64), flush=True)
    print(sk.signature_bwd_describe(B, L, d, N, 0, sk.SK_F64), flush=True)
    S = sk.signature_fwd(x, N)
    gx = host(sk.signature_bwd(x, g, N, sig=S))
    S = host(S)
    torch.cuda.synchronize()
    assert np.all(np.isfinite(S)) and np.all(np.isfinite(gx))
    for b in (0, B // 2, B - 1):
        ref = osig.signature(X[b:b + 1], N)[0]
        assert np.max(np.abs(S[b] - ref) / np.maximum(1.0, np.abs(ref))) <= 1e-10
        gref = osig.signature_backward(X[b:b + 1], G[b:b + 1], N)[0]
        assert np.max(np.abs(gx[b] - gref)) <= 1e-10 * max(1.0, np.max(np.abs(gref)))
    assert np.max(np.abs(S[:, 1:1 + d] - (X[:, -1] - X[:, 0]))) <= 1e-11
    assert np.max(np.abs(gx.sum(axis=1))) <= 1e-9 * max(1.0, np.max(np.abs(gx)))


def test_time_grids_of_the_callers_own():
    # a general time grid is an ordinary channel: the wrappers append it; values and gradients against the oracle on
    # the paths with that channel, and the uniform grid reproduces the library's flag
    import oracle
    from paper_2509_10613_amd import autograd as ag
    rng = np.random.default_rng(91)
    B, L, d, N = 3, 9, 2, 3
    X, Y = paths(92, B, L, d), paths(93, B, L + 2, d)
    tx = np.sort(rng.uniform(0, 1, size=L))
    ty = np.sort(rng.uniform(0, 2, size=(B, L + 2)), axis=1)
    Xt = np.concatenate([X, np.broadcast_to(tx, (B, L))[..., None]], axis=-1)
    Yt = np.concatenate([Y, ty[..., None]], axis=-1)
    x, y = dev(X).requires_grad_(True), dev(Y).requires_grad_(True)
    k = ag.sig_kernel(x, y, 1, 1, times_x=dev(tx), times_y=dev(ty))
    w = rng.normal(size=B)
    (k * dev(w)).sum().backward()
    kr, gxr, gyr = oracle.bwd(Xt, Yt, w, 1, 1, 0)
    assert np.max(np.abs(host(k) - kr) / np.maximum(1.0, np.abs(kr))) <= 1e-10
    assert np.max(np.abs(host(x.grad) - gxr[..., :d])) <= 1e-10 * max(1.0, np.max(np.abs(gxr)))
    assert np.max(np.abs(host(y.grad) - gyr[..., :d])) <= 1e-10 * max(1.0, np.max(np.abs(gyr)))
    xs = dev(X).requires_grad_(True)
    S = ag.signature(xs, N, times=dev(tx))
    ws = rng.normal(size=tuple(S.shape))
    (S * dev(ws)).sum().backward()
    Sr = osig.signature(Xt, N)
    assert np.max(np.abs(host(S) - Sr) / np.maximum(1.0, np.abs(Sr))) <= 1e-10
    gr = osig.signature_backward(Xt, ws, N)[..., :d]
    assert np.max(np.abs(host(xs.grad) - gr)) <= 1e-10 * max(1.0, np.max(np.abs(gr)))
    uni = np.arange(L) / (L - 1)
    a = host(ag.signature(dev(X), N, times=dev(uni)))
    b = host(ag.signature(dev(X), N, flags=sk.SK_FLAG_TIME_AUG))
    assert np.max(np.abs(a - b)) <= 1e-13


def _random_signature_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    while len(cases) < n:
        d = int(rng.integers(1, 21))
        N = int(rng.integers(1, 8))
        flags = int(rng.choice([0, sk.SK_FLAG_TIME_AUG, sk.SK_FLAG_LEAD_LAG, sk.SK_FLAG_TIME_AUG | sk.SK_FLAG_LEAD_LAG]))
        D = (2 * d if flags & sk.SK_FLAG_LEAD_LAG else d) + (1 if flags & sk.SK_FLAG_TIME_AUG else 0)
        if D ** N > 60000:
            continue
        B = int(rng.choice([1, 2, 3, 5, 17, 64, 200]))
        L = int(rng.choice([1, 2, 3, 4, 7, 16, 33, 70, 130]))
        if B * L * D ** N > 1500000:
            continue
        dtype = torch.float32 if rng.random() < 0.2 else torch.float64
        cases.append((B, L, d, N, flags, dtype, bool(rng.random() < 0.5), int(rng.integers(1, 1 << 30))))
    return cases


@pytest.mark.parametrize("chunk", range(6))
def test_random_signature_shapes(chunk):
    # batch sizes, lengths, channel counts, depths, transformations and element types from a seeded generator: whichever
    # kernel variant, prefix length, piece count and lane grouping the plan picks, the numbers are the oracle's
    for B, L, d, N, flags, dtype, give, seed in _random_signature_cases(12, 5200 + chunk):
        X = paths(seed, B, L, d, 0.6 / max(1.0, L) ** 0.5)
        check(X, N, flags, dtype, give_sig=give, seed=seed % 1000)

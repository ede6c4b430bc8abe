"""GPU parity of the truncated-signature path (signature_fwd through the C ABI) against the CPU oracle
(oracle/signature.py), entry by entry on the same seeded inputs.

Tolerance: fp64 1e-10, fp32 1e-5, in the sense |gpu - ref| <= tol * max(1, |ref|) per entry.  fp32 runs compute in
double from the fp32-rounded inputs and round the result once, and are compared with the oracle on those inputs.
"""
import numpy as np
import pytest
import torch

from oracle import signature as osig
from paper_2509_10613_amd import binding as sk
from paper_2509_10613_amd import workloads

pytestmark = pytest.mark.gpu

TOL = {torch.float64: 1e-10, torch.float32: 1e-5}


def dev(a, dtype=torch.float64):
    return torch.tensor(np.asarray(a), dtype=dtype, device="cuda")


def host(t):
    return t.detach().cpu().numpy().astype(np.float64)


def paths(seed, B, L, d, scale=0.4):
    rng = np.random.default_rng(seed)
    return np.cumsum(rng.normal(0, scale, size=(B, L, d)), axis=1)


def check(X, N, flags=0, dtype=torch.float64, what=""):
    x = dev(X, dtype)
    B, L, d = X.shape
    print("signature_fwd B=%d L=%d d=%d N=%d flags=%d %s: %s" % (B, L, d, N, flags, dtype,
          sk.signature_describe(B, L, d, N, flags, sk.SK_F64 if dtype == torch.float64 else sk.SK_F32)), flush=True)
    got = host(sk.signature_fwd(x, N, flags))
    torch.cuda.synchronize()
    ref = osig.signature(host(x), N, flags)
    assert got.shape == ref.shape
    assert np.all(np.isfinite(got))
    err = np.abs(got - ref) / np.maximum(1.0, np.abs(ref))
    print("  max scaled err %.3e (tol %.0e)" % (err.max() if err.size else 0.0, TOL[dtype]), flush=True)
    assert (err.max() if err.size else 0.0) <= TOL[dtype], what
    return got


# every channel count with a kernel of its own (2..17), the run-time channel count kernel (1, 18, 20), prefix lengths
# 0..4 and the longer ones, letter blocks that do not divide the channel count (11, 13, 14, 15, 17), lanes per path
# that do not fill a wave, several waves per path with a ragged last one
@pytest.mark.parametrize("B,L,d,N", [
    (3, 9, 2, 1), (3, 9, 2, 2), (2, 12, 2, 6), (2, 7, 2, 9), (1, 6, 2, 12),
    (3, 8, 3, 3), (2, 8, 3, 4), (2, 6, 3, 7),
    (3, 10, 4, 2), (2, 9, 4, 4), (2, 6, 4, 6),
    (2, 9, 5, 3), (2, 7, 5, 5), (1, 5, 5, 7),
    (2, 8, 6, 3), (1, 6, 6, 5), (2, 8, 7, 3), (1, 5, 7, 5), (2, 8, 8, 3), (1, 6, 8, 5), (2, 6, 9, 3), (1, 5, 9, 4),
    (2, 6, 10, 2), (1, 5, 10, 4), (2, 6, 11, 3), (2, 6, 12, 3), (2, 6, 13, 3), (2, 5, 14, 3), (2, 5, 15, 3),
    (2, 7, 16, 2), (2, 6, 16, 3), (1, 5, 16, 4), (2, 5, 17, 3),
    (4, 11, 1, 5), (2, 6, 18, 2), (2, 5, 20, 3), (1, 4, 12, 1),
])
def test_signature_matches_the_oracle(B, L, d, N):
    check(paths(100 * d + N, B, L, d), N)


def kernel_variants():
    """(channels, owned depth, letter block) of every kernel variant, read from the plan header."""
    import os
    import re
    hdr = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2509_10613_amd", "csrc", "sg_plan.h")
    text = open(hdr).read()
    body = text[text.index("#define SG_VARIANTS(X)"):text.index("#define SG_BWD_VARIANTS(X)")]
    return [tuple(int(v) for v in m) for m in re.findall(r"X\((\d+), (\d+), (\d+)\)", body)]


@pytest.mark.parametrize("D,M,S", kernel_variants())
def test_every_kernel_variant(D, M, S):
    # each register-resident subtree depth, forced through the diagnostic flag, with prefixes of 0, 1, 2 letters,
    # and (where the result stays small) 3, 4 and 6 letters
    for Q in (0, 1, 2, 3, 4, 6):
        N = M + 1 + Q
        if D ** N > 300000 or (Q > 4 and D > 9):
            continue
        L = 5 if D ** N < 20000 else 3
        desc = sk.signature_describe(2, L, D, N, sk.SK_SIG_DEPTH(M), sk.SK_F64)
        assert "horner_kernel<%d, %d, %d, %d, " % (D, M, S, Q if Q <= 4 else 8) in desc, desc
        check(paths(1000 * D + 10 * M + Q, 2, L, D, 0.5), N, flags=sk.SK_SIG_DEPTH(M))
        if "paths_per_wave=1 " not in desc:     # the kernel whose waves hold one path each, too
            check(paths(1000 * D + 10 * M + Q, 2, L, D, 0.5), N, flags=sk.SK_SIG_DEPTH(M) | sk.SK_SIG_ONE_PATH_PER_WAVE)


def test_run_time_channel_kernel_for_any_channel_count():
    for d, N in ((2, 5), (3, 4), (7, 3), (16, 2), (23, 2), (40, 2)):
        desc = sk.signature_describe(2, 6, d, N, sk.SK_SIG_DEPTH(0), sk.SK_F64)
        assert "horner_kernel<0, 0, 1," in desc, desc
        check(paths(77 + d, 2, 6, d), N, flags=sk.SK_SIG_DEPTH(0))


def test_several_short_paths_share_a_wave():
    # lane groups of at most half a wave sit side by side in one wave: batch sizes that do and do not fill the last
    # wave, every prefix length with such kernels, the run-time channel count kernel, with pieces, flags, float32
    for (B, L, d, N) in ((50, 9, 2, 3), (7, 8, 2, 2), (64, 6, 3, 3), (13, 7, 3, 2), (33, 6, 4, 3), (9, 5, 5, 2), (21, 5, 8, 2),
                         (10, 6, 9, 1), (5, 6, 20, 1), (40, 5, 1, 3), (300, 6, 2, 4)):
        desc = sk.signature_describe(B, L, d, N, 0, sk.SK_F64)
        pw = int(desc.split("paths_per_wave=")[1].split(" ")[0])
        assert pw > 1, desc
        got = check(paths(600 + B + d, B, L, d), N)
        one = host(sk.signature_fwd(dev(paths(600 + B + d, B, L, d)), N, sk.SK_SIG_ONE_PATH_PER_WAVE))
        assert np.max(np.abs(got - one) / np.maximum(1.0, np.abs(one))) <= 1e-13
    assert "paths_per_wave=1 " in sk.signature_describe(50, 9, 2, 3, sk.SK_SIG_ONE_PATH_PER_WAVE, sk.SK_F64)
    check(paths(621, 5, 40, 2), 3, flags=sk.SK_SIG_PIECES(2))
    check(paths(622, 11, 9, 2), 3, flags=sk.SK_FLAG_TIME_AUG)
    check(paths(623, 11, 9, 1), 3, flags=sk.SK_FLAG_LEAD_LAG | sk.SK_FLAG_TIME_AUG, dtype=torch.float32)
    # many short paths, the case this is for
    check(paths(624, 5000, 12, 3, 0.3), 4)


def test_paths_cut_into_pieces():
    # forced: 2, 4 and 8 pieces per path, piece lengths that do not divide the path, pieces left empty, with flags and
    # in float32; the library's own choice for a few long paths
    for q, (B, L, d, N) in ((1, (3, 12, 2, 4)), (2, (2, 11, 3, 3)), (3, (2, 9, 3, 3)), (3, (2, 5, 4, 3)), (2, (2, 30, 5, 4)),
                            (1, (2, 10, 16, 3)), (4, (1, 70, 2, 6)), (2, (2, 2, 3, 3))):
        desc = sk.signature_describe(B, L, d, N, sk.SK_SIG_PIECES(q), sk.SK_F64)
        assert "pieces_per_path=%d " % (1 << q) in desc, desc
        check(paths(500 + 10 * q + d, B, L, d), N, flags=sk.SK_SIG_PIECES(q))
    check(paths(521, 2, 13, 2), 4, flags=sk.SK_SIG_PIECES(2) | sk.SK_FLAG_TIME_AUG | sk.SK_FLAG_LEAD_LAG)
    check(paths(522, 2, 13, 3), 3, flags=sk.SK_SIG_PIECES(2) | sk.SK_FLAG_LEAD_LAG, dtype=torch.float32)
    assert "pieces_per_path=1 " in sk.signature_describe(2, 400, 3, 3, sk.SK_SIG_PIECES(0), sk.SK_F64)
    for (B, L, d, N) in ((2, 400, 3, 3), (1, 1500, 2, 5), (3, 257, 5, 3)):
        desc = sk.signature_describe(B, L, d, N, 0, sk.SK_F64)
        assert int(desc.split("pieces_per_path=")[1].split(" ")[0]) > 1, desc
        check(paths(530 + d, B, L, d, 0.1), N)


def test_signature_batches_beyond_one_wave_per_simd():
    # many paths: the launch has more waves than the chip has SIMDs, and picks the deepest register-resident subtree
    check(paths(7, 2100, 6, 3, 0.5), 4)
    check(paths(8, 700, 5, 8, 0.5), 3)


@pytest.mark.parametrize("flags", [sk.SK_FLAG_TIME_AUG, sk.SK_FLAG_LEAD_LAG, sk.SK_FLAG_TIME_AUG | sk.SK_FLAG_LEAD_LAG])
def test_signature_with_path_transformations(flags):
    check(paths(21, 3, 9, 2), 4, flags)
    check(paths(22, 2, 6, 4), 3, flags)
    check(paths(23, 2, 5, 8), 2, flags)


def test_signature_float32():
    check(paths(31, 3, 12, 3), 4, dtype=torch.float32)
    check(paths(32, 2, 8, 16), 3, dtype=torch.float32)
    check(paths(33, 2, 8, 2), 3, flags=sk.SK_FLAG_TIME_AUG | sk.SK_FLAG_LEAD_LAG, dtype=torch.float32)


def test_signature_degenerate_shapes():
    # a path of one point: (1, 0, ..., 0); two points: the tensor exponential of the one increment
    got = check(paths(41, 3, 1, 3), 4)
    assert np.array_equal(got[:, 0], np.ones(3)) and not got[:, 1:].any()
    check(paths(42, 2, 2, 3), 5)
    # empty batch: a successful no-op
    out = sk.signature_fwd(torch.empty((0, 5, 3), dtype=torch.float64, device="cuda"), 3)
    assert out.shape == (0, 40)
    # a constant path
    got = check(np.ones((2, 6, 4)), 3)
    assert not got[:, 1:].any()


def test_signature_argument_errors():
    x = dev(paths(51, 2, 5, 3))
    with pytest.raises(sk.SigKernelError):
        sk.signature_fwd(x, 0)
    with pytest.raises(sk.SigKernelError):
        sk.signature_fwd(x, 3, flags=2)
    with pytest.raises(sk.SigKernelError):
        sk.signature_fwd(x, 3, ws=torch.empty((256,), dtype=torch.uint8, device="cuda")[:16])
    with pytest.raises(sk.SigKernelError):
        sk.signature_fwd(dev(paths(52, 1, 4, 16)), 12)      # more than 2^40 entries
    # the failed calls leave a later good call intact
    check(paths(53, 2, 5, 3), 3)


@pytest.mark.parametrize("name", ["s1", "s2", "s3"])
def test_signature_benchmark_shapes_sampled(name):
    # the shapes of the paper's Table 1 in the launch configuration bench.py times; the oracle computes a sample of
    # the paths one by one, and two properties are checked for every path: level 1 is the total increment and the
    # symmetric part of level 2 is half its outer square (shuffle identity)
    (B, L, d, N), X = workloads.make_signature(name)
    x = dev(X)
    print(name, sk.signature_describe(B, L, d, N, 0, sk.SK_F64), flush=True)
    got = host(sk.signature_fwd(x, N))
    torch.cuda.synchronize()
    assert got.shape == (B, osig.sig_length(d, N)) and np.all(np.isfinite(got))
    whole = host(sk.signature_fwd(x, N, sk.SK_SIG_PIECES(0)))     # uncut paths: the same numbers up to rounding order
    assert np.max(np.abs(got - whole) / np.maximum(1.0, np.abs(whole))) <= 1e-12
    for b in (0, B // 2 + 1, B - 1):
        ref = osig.signature(X[b:b + 1], N)[0]
        err = np.abs(got[b] - ref) / np.maximum(1.0, np.abs(ref))
        print("  path %d: max scaled err %.3e" % (b, err.max()), flush=True)
        assert err.max() <= 1e-10
    S1 = got[:, 1:1 + d]
    S2 = got[:, 1 + d:1 + d + d * d].reshape(B, d, d)
    assert np.abs(S1 - (X[:, -1] - X[:, 0])).max() <= 1e-12
    assert np.abs(S2 + S2.transpose(0, 2, 1) - S1[:, :, None] * S1[:, None, :]).max() <= 1e-12
    assert np.array_equal(got[:, 0], np.ones(B))


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
        check(X, N, flags, dtype)

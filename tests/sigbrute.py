"""Truncated signatures by brute force (test helper, independent of both the oracle and the HIP path).

Paper Section 2.1: the signature of a linear segment with increment z is the tensor exponential
sum_k z^{(x)k}/k! (Proposition 2.1) and the signature of a concatenation is the tensor product of the
signatures (Chen's identity, Proposition 2.2).  The signature kernel is the inner product of the two
signatures (Section 3.1), here truncated at level N.
"""
import numpy as np


def segment_exp(z, N):
    levels = [np.array(1.0)]
    for k in range(1, N + 1):
        levels.append(np.multiply.outer(levels[-1], z) / k)
    return levels


def chen(A, B, N):
    out = []
    for n in range(N + 1):
        acc = 0
        for i in range(n + 1):
            acc = acc + np.multiply.outer(A[i], B[n - i])
        out.append(acc)
    return out


def signature(path, N):
    path = np.asarray(path, dtype=np.float64)
    d = path.shape[1]
    S = segment_exp(np.zeros(d), N)
    for a in range(path.shape[0] - 1):
        S = chen(S, segment_exp(path[a + 1] - path[a], N), N)
    return S


def truncated_kernel(x, y, N):
    Sx, Sy = signature(x, N), signature(y, N)
    return float(sum(np.sum(a * b) for a, b in zip(Sx, Sy)))

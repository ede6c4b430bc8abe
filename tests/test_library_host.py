"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the header
declares, validates arguments and answers the workspace query."""
import ctypes as C
import os
import re

import pytest

from paper_2509_10613_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2509_10613_amd import build
        build.build()
    return binding.load()


def test_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "sigkernel.h")).read()
    declared = set(re.findall(r"\b(sigkernel_[a-z_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None
    assert b"gfx950" in lib.sigkernel_version()


def test_argument_validation_needs_no_gpu(lib):
    f = lib.sigkernel_fwd
    one = C.c_void_p(256)
    # bad dtype, bad flags, bad dyadic order, bad shape: all rejected before any GPU work
    assert f(one, one, one, 4, 8, 8, 2, 0, 0, 0, 7, one, 1 << 20, None) == -4
    assert f(one, one, one, 4, 8, 8, 2, 0, 0, 4, 1, one, 1 << 20, None) == -4
    assert f(one, one, one, 4, 8, 8, 2, -1, 0, 0, 1, one, 1 << 20, None) == -3
    assert f(one, one, one, 4, 8, 8, 2, 0, 21, 0, 1, one, 1 << 20, None) == -3
    assert f(one, one, one, 4, 0, 8, 2, 0, 0, 0, 1, one, 1 << 20, None) == -2
    assert f(one, one, one, 4, 8, 8, 0, 0, 0, 0, 1, one, 1 << 20, None) == -2
    assert f(one, one, one, -1, 8, 8, 2, 0, 0, 0, 1, one, 1 << 20, None) == -2
    assert f(one, one, one, 4, 1 << 20, 8, 2, 12, 0, 0, 1, one, 1 << 20, None) == -2
    assert b"2^29" in lib.sigkernel_last_error()
    assert f(None, one, one, 4, 8, 8, 2, 0, 0, 0, 1, one, 1 << 20, None) == -1
    # empty batch: successful no-op
    assert f(None, None, None, 0, 8, 8, 2, 0, 0, 0, 1, None, 0, None) == 0


def test_workspace_query(lib):
    q = binding.sigkernel_workspace_bytes
    f64 = binding.SK_F64
    a = q(binding.SK_OP_FWD, 128, 0, 256, 256, 5, 1, 1, 1, f64)
    b = q(binding.SK_OP_BWD, 128, 0, 256, 256, 5, 1, 1, 1, f64)
    assert 0 < a < b < (1 << 31)
    assert a % 256 == 0 and b % 256 == 0
    assert q(binding.SK_OP_FWD, 0, 0, 256, 256, 5, 1, 1, 0, f64) == 0
    assert q(binding.SK_OP_FWD, 4, 0, 1, 256, 5, 1, 1, 0, f64) == 0      # L = 1: nothing to sweep
    assert q(9, 4, 0, 8, 8, 2, 0, 0, 0, f64) == 0
    assert q(binding.SK_OP_GRAM_BWD, 1024, 1024, 64, 64, 16, 0, 0, 0, f64) < (8 << 30)
    assert q(binding.SK_OP_BWD, 32, 0, 2048, 2048, 8, 2, 2, 0, f64) < (8 << 30)
    # float callers stage k and grad_k in double: a little more scratch than double callers, same order
    f32 = q(binding.SK_OP_BWD, 16, 0, 64, 64, 3, 1, 1, 0, binding.SK_F32)
    f64b = q(binding.SK_OP_BWD, 16, 0, 64, 64, 3, 1, 1, 0, f64)
    assert f64b <= f32 <= f64b + 4096

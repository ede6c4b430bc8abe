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
    header = open(os.path.join(ROOT, "include", "sigkernel.h")).read() + open(os.path.join(ROOT, "include", "signature.h")).read()
    declared = set(re.findall(r"\b((?:sigkernel|signature)_[a-z0-9_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None
    assert b"gfx950" in lib.sigkernel_version()


def test_mmd2_takes_no_kept_sweep(lib):
    q = lib.sigkernel_mmd2_workspace_bytes
    assert q(8, 8, 16, 16, 3, 0, 0, 0, binding.SK_F64, 1) > 0
    assert q(8, 8, 16, 16, 3, 0, 0, binding.SK_FLAG_KEEP_FORWARD, binding.SK_F64, 1) == 0
    one = C.c_void_p(256)
    assert lib.sigkernel_mmd2(one, one, one, one, one, 8, 8, 16, 16, 3, 0, 0, binding.SK_FLAG_HAVE_FORWARD, binding.SK_F64,
                              one, 1 << 30, None) == -4


def test_argument_validation_needs_no_gpu(lib):
    f = lib.sigkernel_fwd
    one = C.c_void_p(256)
    # bad dtype, bad flags, bad dyadic order, bad shape: all rejected before any GPU work
    assert f(one, one, one, 4, 8, 8, 2, 0, 0, 0, 7, one, 1 << 20, None) == -4
    assert f(one, one, one, 4, 8, 8, 2, 0, 0, 64, 1, one, 1 << 20, None) == -4
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


def _plan(op, *shape):
    text = binding.sigkernel_describe(op, *shape)
    kernel = text.split("kernel=", 1)[1].split(" grid=", 1)[0]
    rest = text.replace("kernel=" + kernel + " ", "")
    d = dict(kv.split("=", 1) for kv in rest.split(" ") if "=" in kv)
    d["kernel"] = kernel
    return d


def test_launch_plan_of_the_five_configurations(lib):
    f64, f32 = binding.SK_F64, binding.SK_F32
    # c2 (128 pairs, L = 256, order 1): the chip is under-filled -> one workgroup per pair in lock step,
    # two strips of 128 block rows, eight waves, everything resident at once, caller's arrays used directly
    p = _plan(binding.SK_OP_BWD, 128, 0, 256, 256, 5, 1, 1, 1, f64)
    assert p["mode"] == "lock-step" and p["kernel"] == "lock_bwd_kernel<1, 5, 2, 0, 0>"
    assert (p["grid"], p["threads"], p["strips"], p["rows_per_lane"], p["fused"]) == ("128", "512", "2", "2", "1")
    assert int(p["lds_bytes"]) <= 160 * 1024
    p = _plan(binding.SK_OP_FWD, 128, 0, 256, 256, 5, 1, 1, 1, f64)
    assert p["kernel"] == "lock_fwd_kernel<1, 5, 2, 0>" and p["fused"] == "1"
    assert _plan(binding.SK_OP_FWD, 128, 0, 256, 256, 5, 1, 1, 1, f32)["fused"] == "0"   # float callers are converted
    # a forward sweep kept for the backward call: the two halves of the backward kernel as launches of their own, in
    # the backward call's workspace; launch modes without that form ignore the flags
    KEEP, HAVE = binding.SK_FLAG_KEEP_FORWARD, binding.SK_FLAG_HAVE_FORWARD
    p1 = _plan(binding.SK_OP_FWD, 128, 0, 256, 256, 5, 1, 1, 1 | KEEP, f64)
    p2 = _plan(binding.SK_OP_BWD, 128, 0, 256, 256, 5, 1, 1, 1 | HAVE, f64)
    assert p1["kernel"] == "lock_bwd_kernel<1, 5, 2, 1, 0>" and p2["kernel"] == "lock_bwd_kernel<1, 5, 2, 2, 0>"
    q = lib.sigkernel_workspace_bytes
    assert q(binding.SK_OP_FWD, 128, 0, 256, 256, 5, 1, 1, 1 | KEEP, f64) == q(binding.SK_OP_BWD, 128, 0, 256, 256, 5, 1, 1, 1, f64)
    assert int(p1["workspace_bytes"]) == q(binding.SK_OP_BWD, 128, 0, 256, 256, 5, 1, 1, 1, f64)
    assert q(binding.SK_OP_FWD, 128, 0, 256, 256, 5, 1, 1, 1, f64) < q(binding.SK_OP_FWD, 128, 0, 256, 256, 5, 1, 1, 1 | KEEP, f64)
    # many pairs, and Gram matrices, in solo mode: checkpoints and bottom rows per pair instead of per wave
    assert _plan(binding.SK_OP_FWD, 5000, 0, 6, 5, 2, 1, 1, KEEP, f64)["kernel"] == "solo_bwd_kernel<1, 2, 1, 1, 0, 2>"
    p1 = _plan(binding.SK_OP_GRAM, 256, 256, 128, 128, 3, 1, 1, KEEP, f64)
    p2 = _plan(binding.SK_OP_GRAM_BWD, 256, 256, 128, 128, 3, 1, 1, HAVE, f64)
    assert p1["kernel"] == "solo_bwd_kernel<1, 3, 2, 1, 0, 2>" and p2["kernel"] == "solo_bwd_kernel<1, 3, 2, 2, 0, 2>"
    assert p1["workspace_bytes"] == p2["workspace_bytes"]
    assert int(p1["workspace_bytes"]) == q(binding.SK_OP_GRAM, 256, 256, 128, 128, 3, 1, 1, KEEP, f64) \
        == q(binding.SK_OP_GRAM_BWD, 256, 256, 128, 128, 3, 1, 1, HAVE, f64)
    assert 6 << 30 < int(p1["workspace_bytes"]) < 8 << 30          # 65536 pairs x 26 checkpoints of 8 x 64 doubles
    assert q(binding.SK_OP_GRAM_BWD, 256, 256, 128, 128, 3, 1, 1, 0, f64) < 1 << 30
    # tile mode keeps its checkpoints in LDS: no such form (the forward call takes the quad kernel as without the flag)
    assert _plan(binding.SK_OP_GRAM, 1024, 1024, 64, 64, 16, 0, 0, KEEP, f64)["kernel"] == "quad_fwd_kernel<0, 16, 4>"
    assert _plan(binding.SK_OP_BWD, 128, 0, 256, 256, 5, 1, 1, 1 | HAVE, f32)["kernel"] == "lock_bwd_kernel<1, 5, 2, 0, 0>"
    # c1: tiny, one strip: stencil, coefficient and auxiliary wave
    p = _plan(binding.SK_OP_FWD, 8, 0, 32, 32, 2, 0, 0, 0, f64)
    assert p["mode"] == "lock-step" and p["threads"] == "192" and p["strips"] == "1"
    # c3 (Gram matrix with 65536 pairs of short paths): one wave per pair fills the chip, and a pair is a single
    # strip (127 block rows at two per lane)
    p = _plan(binding.SK_OP_GRAM_BWD, 256, 256, 128, 128, 3, 1, 1, 0, f64)
    assert p["mode"] == "solo" and p["kernel"] == "solo_bwd_kernel<1, 3, 2, 0, 0, 2>" and p["strips"] == "1"
    # c5 (1048576 pairs, 63 x 63 unrefined cells, 16 channels).  Forward: quad mode, four pairs of a Gram row per
    # wave (16 lanes with four grid rows each per pair), two workgroups per compute unit; a pair batch of that shape
    # has no shared y path and takes the tile kernel.  Backward: the channel contraction dominates -> tile mode,
    # increment Gram matrix of a pair in LDS, contractions on the matrix cores, one workgroup per compute unit
    p = _plan(binding.SK_OP_GRAM, 1024, 1024, 64, 64, 16, 0, 0, 0, f64)
    assert p["mode"] == "quad" and p["kernel"] == "quad_fwd_kernel<0, 16, 4>" and p["grid"] == "512" and p["rows_per_lane"] == "4"
    p = _plan(binding.SK_OP_FWD, 100000, 0, 64, 64, 16, 0, 0, 0, f64)
    assert p["mode"] == "tile" and p["kernel"] == "tile_fwd_kernel<4>" and p["grid"] == "256"
    p = _plan(binding.SK_OP_GRAM_BWD, 1024, 1024, 64, 64, 16, 0, 0, 0, f64)
    assert p["mode"] == "tile" and p["kernel"] == "tile_bwd_kernel<4, true>" and int(p["lds_bytes"]) <= 160 * 1024
    assert _plan(binding.SK_OP_GRAM_BWD, 1024, 1024, 64, 64, 7, 0, 0, 1, f64)["kernel"] == "tile_bwd_kernel<2, true>"
    # 64 columns leave no zero column behind the zero column: the sweeps move one column per LDS instruction
    assert _plan(binding.SK_OP_GRAM_BWD, 1024, 1024, 64, 65, 16, 0, 0, 0, f64)["kernel"] == "tile_bwd_kernel<4, false>"
    # the same shape with few channels, with dyadic refinement, or with very short paths stays with the solo kernels
    assert _plan(binding.SK_OP_GRAM_BWD, 1024, 1024, 64, 64, 3, 0, 0, 0, f64)["mode"] == "solo"
    assert _plan(binding.SK_OP_GRAM_BWD, 1024, 1024, 64, 64, 16, 1, 1, 0, f64)["mode"] == "solo"
    assert _plan(binding.SK_OP_GRAM_BWD, 1024, 1024, 30, 64, 16, 0, 0, 0, f64)["mode"] == "solo"
    # ... whose forward Gram calls take the quad kernel where its lanes can hold the rows' increments (four or eight
    # block rows per lane, blocks of at most 2 x 2 cells that hold all of the refinement)
    assert _plan(binding.SK_OP_GRAM, 1024, 1024, 64, 64, 3, 0, 0, 0, f64)["kernel"] == "quad_fwd_kernel<0, 3, 4>"
    assert _plan(binding.SK_OP_GRAM, 1024, 1024, 30, 64, 16, 0, 0, 0, f64)["kernel"] == "quad_fwd_kernel<0, 16, 4>"
    assert _plan(binding.SK_OP_GRAM, 256, 256, 128, 128, 3, 1, 1, 0, f64)["kernel"] == "quad_fwd_kernel<1, 3, 8>"   # c3
    assert _plan(binding.SK_OP_GRAM, 1024, 1024, 64, 64, 16, 1, 1, 0, f64)["mode"] == "solo"    # 16 channels, 126 block rows
    assert _plan(binding.SK_OP_GRAM, 256, 256, 128, 128, 3, 2, 2, 0, f64)["mode"] == "solo"     # blocks of 4 x 4 cells
    assert _plan(binding.SK_OP_GRAM, 256, 256, 100, 128, 3, 2, 1, 0, f64)["mode"] != "quad"     # refinement above the blocks
    assert _plan(binding.SK_OP_FWD, 5000, 0, 128, 128, 3, 1, 1, 0, f64)["mode"] == "solo"       # no shared y path
    # many pairs of longer paths (more than 128 block rows): strips chained through global rows
    p = _plan(binding.SK_OP_BWD, 4096, 0, 300, 300, 4, 0, 0, 0, f64)
    assert p["mode"] == "wave-per-pair" and p["kernel"].startswith("sweep_bwdu_kernel<0, 4,") and p["strips"] == "5"
    # more than 16 channels: runtime channel loop, y increments in global memory
    p = _plan(binding.SK_OP_FWD, 4096, 0, 40, 40, 20, 1, 1, 0, f64)
    assert p["mode"] == "wave-per-pair" and p["kernel"] == "sweep_fwd_kernel<1, 0, false>"
    # c4 (32 pairs, 2047 block rows = 32 strips each): bands of four strips on different compute units, eight
    # bands per pair, all 256 workgroups resident at once; four strip waves and a data-moving wave each
    p = _plan(binding.SK_OP_BWD, 32, 0, 2048, 2048, 8, 2, 2, 0, f64)
    assert p["mode"] == "band" and p["kernel"] == "band_fwd_kernel<2, 8, true, 0>+band_rev_kernel<2, 8, 0>" and p["grid"] == "256"
    assert p["threads"] == "320" and p["strips"] == "32" and int(p["lds_bytes"]) <= 160 * 1024
    p = _plan(binding.SK_OP_FWD, 32, 0, 2048, 2048, 8, 2, 2, 0, f64)
    assert p["mode"] == "band" and p["kernel"] == "band_fwd_kernel<2, 8, false, 0>" and p["grid"] == "256"
    # more long pairs than the chip has room for bands: one workgroup per pair, its strips in rounds
    p = _plan(binding.SK_OP_BWD, 64, 0, 2048, 2048, 8, 2, 2, 0, f64)
    assert p["mode"] == "cooperative" and p["grid"] == "64"
    # 16 channels have no band kernel
    assert _plan(binding.SK_OP_FWD, 8, 0, 2048, 2048, 16, 2, 2, 0, f64)["mode"] == "cooperative"
    # the replay variant of the backward pass never runs in lock step
    p = _plan(binding.SK_OP_BWD, 128, 0, 256, 256, 5, 1, 1, 1 | binding.SK_FLAG_BWD_REPLAY, f64)
    assert p["mode"] == "cooperative" and p["kernel"].startswith("sweep_bwd_coop_kernel")


def test_launch_plan_stays_inside_the_hardware_limits(lib):
    f64 = binding.SK_F64
    for op in (binding.SK_OP_FWD, binding.SK_OP_BWD):
        for B in (1, 7, 128, 256, 300, 1024, 5000):
            for L in (2, 9, 65, 129, 300, 700, 3000):
                for d in (1, 3, 5, 8, 16, 20):
                    for lam in (0, 1, 2, 3):
                        if ((L - 1) << lam) >= (1 << 14):
                            continue
                        for flags in (0, binding.SK_FLAG_LEAD_LAG | 1, binding.SK_FLAG_BWD_REPLAY):
                            if flags & binding.SK_FLAG_LEAD_LAG and ((2 * L - 2) << lam) >= (1 << 14):
                                continue
                            p = _plan(op, B, 0, L, max(2, L // 2), d, lam, lam, flags, f64)
                            assert int(p["lds_bytes"]) <= 160 * 1024, p
                            # the launch that solves drifted pairs once more (the replay kernel)
                            assert int(p["second_launch_lds_bytes"]) <= 160 * 1024, p
                        p = _plan(op, B, 0, L, max(2, L // 2), d, lam, lam, 0, f64)
                        assert 64 <= int(p["threads"]) <= 1024 and int(p["threads"]) % 64 == 0, p
                        assert 1 <= int(p["grid"]), p
                        if p["mode"] == "lock-step":
                            assert int(p["grid"]) == B and int(p["strips"]) <= (4 if op == binding.SK_OP_FWD else 2), p
                            assert d <= 16, p
    buf = C.create_string_buffer(8)
    assert lib.sigkernel_describe(binding.SK_OP_FWD, 4, 0, 8, 8, 2, 0, 0, 0, f64, buf, 8) == 0
    assert len(buf.value) == 7                                  # truncated, still NUL-terminated
    assert lib.sigkernel_describe(99, 4, 0, 8, 8, 2, 0, 0, 0, f64, buf, 8) == -2
    assert lib.sigkernel_describe(binding.SK_OP_FWD, 4, 0, 8, 8, 2, 0, 0, 0, f64, None, 8) == -1


# ---------------------------------------------------------------- truncated signatures (include/signature.h)
def test_signature_host_side(lib):
    one = C.c_void_p(256)
    assert lib.signature_length(4, 6, 0) == 5461 and lib.signature_length(16, 4, 0) == 69905
    assert lib.signature_length(2, 3, binding.SK_FLAG_TIME_AUG | binding.SK_FLAG_LEAD_LAG) == 1 + 5 + 25 + 125
    assert lib.signature_length(1, 7, 0) == 8
    assert lib.signature_length(16, 12, 0) == 0 and lib.signature_length(0, 3, 0) == 0 and lib.signature_length(3, 0, 0) == 0
    f = lib.signature_fwd
    assert f(one, one, 4, 8, 3, 3, 0, 7, one, 1 << 20, None) == -4       # dtype
    assert f(one, one, 4, 8, 3, 3, 2, 1, one, 1 << 20, None) == -4       # a flag of the kernel entry points
    assert f(one, one, 4, 8, 3, 0, 0, 1, one, 1 << 20, None) == -2       # N < 1
    assert f(one, one, 4, 0, 3, 3, 0, 1, one, 1 << 20, None) == -2       # L < 1
    assert f(one, one, -1, 8, 3, 3, 0, 1, one, 1 << 20, None) == -2
    assert f(one, one, 4, 8, 16, 12, 0, 1, one, 1 << 20, None) == -2     # more than 2^40 entries per path
    assert b"2^40" in lib.sigkernel_last_error()
    assert f(None, one, 4, 8, 3, 3, 0, 1, one, 1 << 20, None) == -1
    assert f(one, one, 4, 8, 3, 3, 0, 1, one, 16, None) == -5
    assert f(one, one, 4, 8, 3, 3, 0, 1, C.c_void_p(264), 1 << 20, None) == -5
    assert f(None, None, 0, 8, 3, 3, 0, 1, None, 0, None) == 0           # empty batch
    # workspace: increments of the (transformed) paths in double, rows padded to an even count, plus the double
    # staging of the result for float callers
    assert binding.signature_workspace_bytes(128, 1024, 16, 4, 0, binding.SK_F64) >= 128 * 1023 * 16 * 8
    assert binding.signature_workspace_bytes(128, 1024, 16, 4, 0, binding.SK_F64) < 128 * 1023 * 16 * 8 + 512
    w32 = binding.signature_workspace_bytes(10, 20, 3, 3, binding.SK_FLAG_LEAD_LAG, binding.SK_F32)
    assert w32 >= 10 * 38 * 6 * 8 + 10 * (1 + 6 + 36 + 216) * 8
    assert binding.signature_workspace_bytes(0, 20, 3, 3, 0, binding.SK_F64) == 0


def test_signature_launch_plans(lib):
    def plan(B, L, d, N, flags=0):
        text = binding.signature_describe(B, L, d, N, flags, binding.SK_F64)
        kern = re.search(r"kernel=(horner_kernel<[^>]*>)", text).group(1)
        vals = {k: int(v) for k, v in re.findall(r"(\w+)=(\d+)", text)}
        return kern, vals
    # the three shapes of Table 1: deepest subtree that still gives every SIMD a wave
    kern, v = plan(128, 256, 4, 6)     # too few waves for the chip as whole paths: cut into 4 pieces of 64 segments
    assert kern == "horner_kernel<4, 2, 1, 3, false, false>" and v["lanes_per_path"] == 256 and v["grid"] == 512
    assert v["pieces_per_path"] == 4 and v["segments_per_piece"] == 64
    kern, v = plan(128, 256, 4, 6, binding.SK_SIG_PIECES(0))
    assert kern == "horner_kernel<4, 2, 1, 3, false, false>" and v["grid"] == 128 and v["pieces_per_path"] == 1
    kern, v = plan(128, 512, 8, 5)
    assert kern == "horner_kernel<8, 2, 1, 2, false, false>" and v["lanes_per_path"] == 512 and v["grid"] == 256
    assert v["pieces_per_path"] == 1
    kern, v = plan(128, 1024, 16, 4)
    assert kern == "horner_kernel<16, 1, 4, 2, false, false>" and v["lanes_per_path"] == 1024 and v["grid"] == 512
    assert v["entries_per_path"] == 69905 and v["pieces_per_path"] == 1
    # the shape of the paper's figure (32 long paths): pieces of at least 32 segments
    kern, v = plan(32, 1024, 5, 4)
    assert v["pieces_per_path"] == 16 and v["segments_per_piece"] == 64
    # a large batch prefers the deepest subtree; channel counts without a kernel of their own, and one channel, take
    # the run-time kernel; the transformations change the channel count the plan sees
    assert plan(100000, 50, 3, 8)[0] == "horner_kernel<3, 3, 1, 4, false, false>"
    assert plan(4, 50, 20, 3)[0] == "horner_kernel<0, 0, 1, 2, false, false>"
    assert plan(4, 50, 1, 5)[0] == "horner_kernel<0, 0, 1, 4, false, false>"
    assert plan(4, 50, 2, 3, binding.SK_FLAG_TIME_AUG | binding.SK_FLAG_LEAD_LAG)[1]["channels"] == 5
    # lanes of a wave never span two paths, every lane's words fit the level count, the grid covers all waves
    for (B, L, d, N) in [(3, 9, 5, 4), (7, 5, 11, 3), (2, 4, 17, 4), (1, 3, 2, 14), (9, 9, 9, 9)]:
        kern, v = plan(B, L, d, N)
        D, M, S, QC = (int(t) for t in re.search(r"<(\d+), (\d+), (\d+), (\d+), \w+, \w+>", kern).groups())
        Q = v["prefix_letters"]
        assert Q == N - M - 1 and (QC == Q or (QC == 8 and 4 < Q <= 8))
        assert v["letter_blocks"] * S >= d and (v["letter_blocks"] - 1) * S < d
        assert v["lanes_per_path"] == d ** Q * v["letter_blocks"]
        assert v["waves_per_path"] * 64 >= v["lanes_per_path"] > (v["waves_per_path"] - 1) * 64
        assert v["grid"] * 4 >= B * v["waves_per_path"] > (v["grid"] - 1) * 4
    # levels beyond what a lane can carry are refused
    with pytest.raises(binding.SigKernelError):
        binding.signature_describe(1, 3, 3, 13, 0, binding.SK_F64)
    with pytest.raises(binding.SigKernelError):
        binding.signature_describe(1, 3, 16, 4, binding.SK_SIG_DEPTH(2), binding.SK_F64)


def test_signature_backward_host_side(lib):
    one = C.c_void_p(256)
    f = lib.signature_bwd
    assert f(one, None, one, one, 4, 8, 3, 3, 0, 7, one, 1 << 20, None) == -4
    assert f(one, None, one, one, 4, 8, 3, 0, 0, 1, one, 1 << 20, None) == -2
    assert f(one, None, None, one, 4, 8, 3, 3, 0, 1, one, 1 << 20, None) == -1
    assert f(one, None, one, one, 4, 8, 3, 3, 0, 1, one, 16, None) == -5
    assert f(None, None, None, None, 0, 8, 3, 3, 0, 1, None, 0, None) == 0
    # workspace: increments and their gradients (rows rounded up to an odd count), the signatures when the caller
    # does not pass them, double copies for float callers
    n = 1 + 3 + 9 + 27
    base = 2 * 4 * 7 * 4 * 8
    w0 = lib.signature_bwd_workspace_bytes(4, 8, 3, 3, 0, 1, 1)
    w1 = lib.signature_bwd_workspace_bytes(4, 8, 3, 3, 0, 1, 0)
    w2 = lib.signature_bwd_workspace_bytes(4, 8, 3, 3, 0, 0, 1)
    assert base <= w0 < base + 1024 and w1 >= w0 + 4 * n * 8 and w2 >= w0 + 2 * 4 * n * 8
    # launch plans: the backward variants hold entries and adjoints, so the subtrees are smaller than the forward's
    text = binding.signature_bwd_describe(128, 1024, 16, 4, 0, binding.SK_F64)
    assert "horner_bwd_kernel<16, 1, 2, 2, false, false>" in text and "lanes_per_path=2048" in text and "grid=1024" in text
    assert "horner_bwd_kernel<8, 1, 4, 3, false, false>" in binding.signature_bwd_describe(128, 512, 8, 5, 0, binding.SK_F64)
    assert "horner_bwd_kernel<0, 0, 1, 2, false, false>" in binding.signature_bwd_describe(4, 9, 20, 3, 0, binding.SK_F64)
    lds = int(re.search(r"lds_bytes=(\d+)", text).group(1))
    assert lds == 4 * (16 + 64 * 17) * 8
    # lead-lag paths take the kernels that leave out the half of the channels a segment does not move
    assert "horner_bwd_kernel<16, 1, 2, 2, false, true>" in binding.signature_bwd_describe(
        128, 512, 8, 4, binding.SK_FLAG_LEAD_LAG, binding.SK_F64)
    assert "horner_kernel<16, 1, 4, 2, false, true>" in binding.signature_describe(
        128, 512, 8, 4, binding.SK_FLAG_LEAD_LAG, binding.SK_F64)
    assert "horner_kernel<2, 3, 1, 2, true, false>" in binding.signature_describe(    # two channels: no such form
        128, 512, 1, 6, binding.SK_FLAG_LEAD_LAG, binding.SK_F64)
    with pytest.raises(binding.SigKernelError):
        binding.signature_bwd_describe(4, 9, 2000, 2, 0, binding.SK_F64)    # beyond the run-time kernel's channel limit

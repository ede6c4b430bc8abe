"""Compile the HIP library (libsigkernel.so, gfx950) in-tree with hipcc."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsigkernel.so")
SOURCES = ["sk_api.hip", "sk_kernels.hip", "sk_lockstep.hip", "sk_solo.hip", "sk_solo_one.hip", "sk_tile.hip", "sk_tile_bwd.hip", "sk_quad.hip", "sk_band.hip", "sg_horner.hip", "sg_horner_bwd.hip"]
HEADERS = ["sk_plan.h", "sk_kernels.h", "sk_dev.h", "sk_lane.h", "sk_solo_impl.h", "sk_tile.h", "sg_plan.h", "sg_kernels.h", "sg_dev.h"]
PUBLIC = ["sigkernel.h", "signature.h"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-munsafe-fp-atomics",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]
# Per source file.  The tile backward kernel moves every MFMA result on (to LDS, to atomics): with the results in
# vector registers instead of accumulation registers the copies between the two fall away (c5 backward: -1 %).
FILE_FLAGS = {"sk_tile_bwd.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"]}


def _stale(target, deps):
    return (not os.path.exists(target)) or any(os.path.getmtime(target) < os.path.getmtime(d) for d in deps)


def build(force: bool = False, verbose: bool = False, extra_flags=()) -> str:
    deps = [os.path.join(CSRC, f) for f in SOURCES + HEADERS] + [os.path.join(ROOT, "include", h) for h in PUBLIC]
    if not force and not _stale(LIB, deps):
        return LIB
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)

    hdrs = [os.path.join(CSRC, f) for f in HEADERS] + [os.path.join(ROOT, "include", h) for h in PUBLIC]

    def compile_one(src):
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        if not force and not extra_flags and not _stale(obj, [os.path.join(CSRC, src)] + hdrs):
            return obj   # this object is newer than its source and every header
        cmd = ["hipcc"] + FLAGS + FILE_FLAGS.get(src, []) + list(extra_flags) + ["-c", os.path.join(CSRC, src), "-o", obj]
        r = subprocess.run(cmd, capture_output=True, text=True)
        err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
        if r.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (src, err))
        if verbose and err.strip():
            print(err, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    cmd = ["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    return LIB


if __name__ == "__main__":
    print(build(force=True, verbose=True, extra_flags=[a for a in sys.argv[1:] if a.startswith("-D")]))

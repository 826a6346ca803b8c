"""Build liblg.so (the HIP kernels and their C ABI) for gfx950 with hipcc, in-tree."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OUT = os.path.join(HERE, "liblg.so")
OBJ_DIR = os.path.join(HERE, "_build")

SOURCES = ["status.hip", "memops.hip", "reduce.hip", "dwconv.hip", "gemm.hip", "gemm_t.hip", "gemm_direct.hip", "gemv.hip", "calib.hip"]

# Packed-fp32 VALU forms are disabled on purpose (device-side target feature).
HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               "-Wno-unused-command-line-argument",
               # the global->LDS transfers name m0 as clobbered so that the compiler keeps no value of its
               # own there across them; clang notes that m0 is a reserved register, which is the point
               "-Wno-inline-asm",
               "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


def _hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    return "hipcc"


def _compile(src, obj_dir=OBJ_DIR, extra_flags=()):
    obj = os.path.join(obj_dir, os.path.splitext(src)[0] + ".o")
    cmd = [_hipcc()] + HIPCC_FLAGS + list(extra_flags) + ["-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    # the host pass does not know the device-only feature flag; that notice is noise
    log = "\n".join(l for l in r.stdout.splitlines() if "not a recognized feature" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{log}")
    return obj, log


def build(verbose=False, out=OUT, obj_dir=OBJ_DIR, extra_flags=()):
    """Compile every source and link liblg.so; always recompiles.  `out`, `obj_dir` and `extra_flags`
    (more hipcc options, e.g. -D overrides of tuning constants) build a second copy elsewhere."""
    os.makedirs(obj_dir, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        results = list(ex.map(lambda src: _compile(src, obj_dir, extra_flags), SOURCES))
    for _, log in results:
        if verbose and log.strip():
            print(log)
    cmd = [_hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", out] + [o for o, _ in results]
    subprocess.run(cmd, check=True)
    return out


if __name__ == "__main__":
    print(build(verbose=True))
    sys.exit(0)

"""Compile libdsqconv.so (HIP, gfx950 only) in-tree with hipcc.

Every source is compiled to an object file of its own (side by side, one
hipcc process per file) and the objects are linked into the shared library.
"""
import glob
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libdsqconv.so")
OBJ_DIR = os.path.join(HERE, "_build")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    # no fused multiply-add may be formed inside the quantizer recipe
    "-ffp-contract=off",
    # device code must not use the packed fp32 ALU forms (v_pk_*_f32).  The
    # feature name belongs to the gfx950 pass only; hipcc's host (x86) pass
    # prints a note that it does not know it, which is expected and harmless.
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _newest_header():
    hdrs = glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(HERE, "..", "include", "*.h"))
    return max(os.path.getmtime(h) for h in hdrs)


def build_library(verbose=False, incremental=False, jobs=None):
    """Compiles every source (or, with incremental=True, those newer than their
    object file) and links libdsqconv.so."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    hdr_time = _newest_header()
    todo, objs = [], []
    for src in sources():
        obj = os.path.join(OBJ_DIR, os.path.basename(src)[:-4] + ".o")
        objs.append(obj)
        fresh = incremental and os.path.exists(obj) and \
            os.path.getmtime(obj) > max(os.path.getmtime(src), hdr_time)
        if not fresh:
            todo.append((src, obj))

    def compile_one(job):
        src, obj = job
        proc = subprocess.run([hipcc] + HIPCC_FLAGS + ["-c", src, "-o", obj + ".tmp"],
                              stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if proc.returncode == 0:
            os.replace(obj + ".tmp", obj)
        return src, proc.returncode, proc.stdout

    jobs = jobs or min(8, os.cpu_count() or 1)
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        results = list(pool.map(compile_one, todo))
    log = "".join(out for _, _, out in results)
    failed = [src for src, rc, _ in results if rc != 0]
    if failed:
        raise RuntimeError("hipcc failed on %s:\n%s" % (", ".join(failed), log))
    tmp = LIB + ".tmp.%d" % os.getpid()
    proc = subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp] + objs,
                          stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    log += proc.stdout
    if proc.returncode != 0:
        if os.path.exists(tmp):
            os.remove(tmp)
        raise RuntimeError("linking libdsqconv.so failed:\n" + log)
    if verbose and log.strip():
        print(log)
    os.replace(tmp, LIB)
    return LIB


def build_ceilings_probe():
    """The stand-alone micro-benchmark of the machine's ceilings (matrix
    instruction rates, LDS, vector L1, HBM): ceilings/ceilings_probe."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    src = os.path.join(HERE, "ceilings", "ceilings.hip")
    exe = os.path.join(HERE, "ceilings", "ceilings_probe")
    proc = subprocess.run([hipcc, "--offload-arch=gfx950", "-O3", "-Xclang", "-target-feature", "-Xclang",
                           "-packed-fp32-ops", src, "-o", exe],
                          stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed on ceilings.hip:\n" + proc.stdout)
    return exe


if __name__ == "__main__":
    import sys
    print(build_library(verbose="-q" not in sys.argv, incremental="-i" in sys.argv))
    if "-i" not in sys.argv:
        print(build_ceilings_probe())

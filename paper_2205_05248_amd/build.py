"""Build the C-ABI library libmarl_qnet.so for gfx950 with hipcc (in-tree).

Every source file is compiled to an object of its own (in parallel) and the objects are linked;
`python -m paper_2205_05248_amd.build --incremental` recompiles only the sources that are newer
than their object (any header change recompiles everything).
"""
import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libmarl_qnet.so")

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC",
    # keep the compiler from forming packed-fp32 vector instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def headers():
    return glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(HERE, "..", "include", "*.h"))


def _object_of(src):
    return os.path.join(OBJ, os.path.splitext(os.path.basename(src))[0] + ".o")


def build(verbose=True, incremental=False, jobs=8):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    newest_header = max(os.path.getmtime(p) for p in headers())
    todo = []
    for src in sources():
        obj = _object_of(src)
        fresh = (incremental and os.path.exists(obj) and os.path.getmtime(obj) > os.path.getmtime(src)
                 and os.path.getmtime(obj) > newest_header)
        if not fresh:
            todo.append(src)

    def compile_one(src):
        cmd = [hipcc] + HIPCC_FLAGS + ["-c", src, "-o", _object_of(src)]
        if verbose:
            print(" ".join(cmd), flush=True)
        done = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        # the host pass does not know the device-only feature flag and says so once per file
        out = "\n".join(l for l in done.stdout.splitlines() if "packed-fp32-ops" not in l)
        if out.strip() and (verbose or done.returncode):
            print(out, flush=True)
        if done.returncode:
            raise subprocess.CalledProcessError(done.returncode, cmd)

    with ThreadPoolExecutor(max_workers=max(1, jobs)) as pool:
        list(pool.map(compile_one, todo))
    known = {_object_of(s) for s in sources()}
    for stale in glob.glob(os.path.join(OBJ, "*.o")):
        if stale not in known:
            os.remove(stale)
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + sorted(known)
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


def needs_build():
    if not os.path.exists(LIB):
        return True
    t = os.path.getmtime(LIB)
    return any(os.path.getmtime(p) > t for p in sources() + headers())


if __name__ == "__main__":
    build(incremental="--incremental" in sys.argv[1:])
    sys.exit(0)

"""Builds libsmartmem.so (HIP kernels for gfx950 + the C-ABI host code) in-tree."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libsmartmem.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
COMMON = ["-O3", "-fPIC", "-std=c++17", "-Wall", "-Wno-unused-function"]
HIPFLAGS = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def sources():
    names = sorted(os.listdir(CSRC))
    return [n for n in names if n.endswith(".cpp")], [n for n in names if n.endswith(".hip")]


def _compile(args):
    r = subprocess.run(args, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("build failed: %s\n%s\n%s" % (" ".join(args), r.stdout, r.stderr))
    return r.stderr


def build(force=True, jobs=8, verbose=False):
    os.makedirs(OBJ, exist_ok=True)
    cpps, hips = sources()
    hdr_m = max(os.path.getmtime(os.path.join(d, f)) for d in (CSRC, os.path.join(HERE, "..", "include"))
                for f in os.listdir(d) if f.endswith(".h"))

    def newest_dep(obj, src):
        """mtime of the newest file the object was built from (the compiler's dependency file), else of any header"""
        dep = obj + ".d"
        if not os.path.exists(dep):
            return max(os.path.getmtime(src), hdr_m)
        words = open(dep).read().replace("\\\n", " ").split()[1:]
        try:
            return max(os.path.getmtime(w) for w in words if not w.startswith("/opt/") and not w.startswith("/usr/"))
        except OSError:
            return float("inf")
    cmds, objs = [], []
    for n in cpps + hips:
        src = os.path.join(CSRC, n)
        obj = os.path.join(OBJ, n + ".o")
        objs.append(obj)
        if not force and os.path.exists(obj) and os.path.getmtime(obj) > newest_dep(obj, src):
            continue
        if n.endswith(".hip"):
            cmds.append([HIPCC, "-x", "hip"] + COMMON + HIPFLAGS + ["-MD", "-MF", obj + ".d", "-c", src, "-o", obj])
        else:
            cmds.append([HIPCC, "-x", "c++", "-I/opt/rocm/include", "-D__HIP_PLATFORM_AMD__"] + COMMON + ["-MD", "-MF", obj + ".d", "-c", src, "-o", obj])
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        for w in ex.map(_compile, cmds):
            if verbose and w.strip():
                print(w, file=sys.stderr)
    _compile([HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB] + objs + ["-L/opt/rocm/lib", "-lamdhip64"])
    return LIB


if __name__ == "__main__":
    print(build(force="--incremental" not in sys.argv, verbose=True))

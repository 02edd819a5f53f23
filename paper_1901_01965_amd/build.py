"""Builds the HIP library in-tree: hipcc --offload-arch=gfx950 -> csrc/../lib/libwinograd_mi355x.so."""
import concurrent.futures
import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB_DIR = os.path.join(HERE, "lib")
OBJ_DIR = os.path.join(LIB_DIR, "obj")
LIB_PATH = os.path.join(LIB_DIR, "libwinograd_mi355x.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # keep matrix-core results in ordinary vector registers where they fit: the vector ALU reads
    # them right away (limb joins, output transform) and would otherwise pay one copy per register
    "-mllvm", "-amdgpu-mfma-vgpr-form=1",
    "-Wall", "-Wno-unused-function",
]


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _headers():
    return glob.glob(os.path.join(CSRC, "*.h")) + glob.glob(os.path.join(ROOT, "include", "*.h"))


def _run(cmd):
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in proc.stdout.splitlines() if "is not a recognized feature for this target" not in l)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed: %s\n%s" % (" ".join(cmd), out))
    return out


def build(verbose=False, incremental=False, jobs=None):
    """Compile every HIP source for gfx950 (one object per source, in parallel) and link them into one shared
    library.  Everything is recompiled unless `incremental` is set, in which case a source is skipped when its
    object is newer than it and than every header."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    newest_header = max(os.path.getmtime(h) for h in _headers())
    todo, objects = [], []
    for src in sources():
        obj = os.path.join(OBJ_DIR, os.path.basename(src)[:-4] + ".o")
        objects.append(obj)
        fresh = (incremental and os.path.exists(obj) and
                 os.path.getmtime(obj) > max(os.path.getmtime(src), newest_header))
        if not fresh:
            todo.append([hipcc] + HIPCC_FLAGS + ["-I", os.path.join(ROOT, "include"), "-I", CSRC, "-c", src, "-o", obj])
    jobs = jobs or min(8, int(os.environ.get("MAX_JOBS", "8")), max(1, len(todo)))
    with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as pool:
        for cmd, out in zip(todo, pool.map(_run, todo)):
            if verbose:
                print(" ".join(cmd))
                if out.strip():
                    print(out)
    out = _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB_PATH] + objects)
    if verbose and out.strip():
        print(out)
    return LIB_PATH


if __name__ == "__main__":
    import sys
    print(build(verbose=True, incremental="--incremental" in sys.argv))

"""Compile libknng.so (HIP, gfx950 only) in-tree with hipcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libknng.so")
SOURCES = ("knng_build.hip", "knng_brute.hip", "knng_recall.hip", "knng_merge.hip", "knng_optimize.hip", "knng_search.hip")
HEADERS = ("knng_device.h", "knng_host.h", "knng_join_wave.h", os.path.join("..", "..", "include", "knng.h"))
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function"]
# per-source flags.  knng_brute.hip: accumulators of the matrix instructions in ordinary vector
# registers; with the accumulator-register form the compiler moves all sixteen in and out around
# every slab of k_brute_mfma, and the read back waits for the matrix pipe to drain.
EXTRA_FLAGS = {"knng_brute.hip": ["-mllvm", "-amdgpu-mfma-vgpr-form"]}


def up_to_date() -> bool:
    if not os.path.exists(LIB):
        return False
    t = os.path.getmtime(LIB)
    deps = [os.path.join(CSRC, f) for f in SOURCES + HEADERS] + [os.path.abspath(__file__)]
    return all(os.path.getmtime(p) <= t for p in deps)


def build(force: bool = True, verbose: bool = False, defines=(), lib: str = LIB) -> str:
    """Compile every HIP source and link the shared library; returns its path.

    `defines` ("NAME=value" strings) and `lib` build a variant of the library somewhere else
    (tuning experiments); the default builds libknng.so in-tree."""
    if not force and lib == LIB and not defines and up_to_date():
        return LIB
    objdir = CSRC if lib == LIB else os.path.dirname(os.path.abspath(lib))
    tag = "" if lib == LIB else os.path.splitext(os.path.basename(lib))[0] + "_"
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(objdir, tag + src.replace(".hip", ".o"))
        cmd = [HIPCC, *FLAGS, *EXTRA_FLAGS.get(src, []), *("-D" + d for d in defines), "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd))
        procs.append((cmd, subprocess.Popen(cmd, stderr=subprocess.PIPE, text=True)))
        objs.append(obj)
    for cmd, p in procs:
        err = p.communicate()[1]
        err = "\n".join(l for l in err.splitlines() if "packed-fp32-ops" not in l)   # the host pass does not know the feature
        if err:
            print(err)
        if p.returncode != 0:
            raise RuntimeError("hipcc failed: " + " ".join(cmd))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs]
    subprocess.run(cmd, check=True)
    return lib


if __name__ == "__main__":
    print(build(force=True, verbose=True))

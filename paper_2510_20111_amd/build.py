"""Build step of libhzp: one hipcc invocation for gfx950 (cross-compiles without a GPU)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SOURCES = ["planner.cpp", "api.cpp", "scheduler.cpp", "kernels.hip"]
LIB = os.path.join(HERE, "libhzp.so")


def build(verbose=False):
    """Compile csrc/ into paper_2510_20111_amd/libhzp.so.  Always recompiles."""
    cmd = ["hipcc", "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
           # packed fp32 instructions stay off (see the hipcc flag of the same name)
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wall", "-Wno-unused-command-line-argument", "-pthread",
           "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(HERE, "csrc")]
    cmd += [os.path.join(HERE, "csrc", s) for s in SOURCES]
    cmd += ["-o", LIB]
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))

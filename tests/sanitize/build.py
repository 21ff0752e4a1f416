"""Host-only sanitizer build (test infrastructure): the library's planner, entry-point argument
checks and scheduler host code, and the C oracle, compiled with -fsanitize=address,undefined.
The kernel launchers are replaced by stubs that refuse (launch_stubs.cpp): nothing here can reach a
GPU.  Output goes to _build/ at the repository root (not committed)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
OUT = os.path.join(ROOT, "_build")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]


def build():
    os.makedirs(OUT, exist_ok=True)
    csrc = os.path.join(ROOT, "paper_2510_20111_amd", "csrc")
    lib = os.path.join(OUT, "libhzp_san.so")
    cmd = ["g++", "-std=c++17", "-fPIC", "-shared", "-pthread", "-Wall"] + SAN + [
        "-I" + os.path.join(ROOT, "include"), "-I" + csrc, "-I/opt/rocm/include", "-D__HIP_PLATFORM_AMD__",
        os.path.join(csrc, "planner.cpp"), os.path.join(csrc, "api.cpp"), os.path.join(csrc, "scheduler.cpp"),
        os.path.join(HERE, "launch_stubs.cpp"), "-o", lib, "-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib"]
    subprocess.run(cmd, check=True)
    ora = os.path.join(OUT, "libhzp_oracle_san.so")
    cmd = ["gcc", "-fno-fast-math", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared"] + SAN + [
        os.path.join(ROOT, "oracle", "numeric.c"), "-o", ora, "-lm"]
    subprocess.run(cmd, check=True)
    return lib, ora


if __name__ == "__main__":
    print(build())

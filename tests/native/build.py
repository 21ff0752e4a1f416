"""Builds tests/native/selftest: a C++ program that drives libhzp.so with the HIP runtime alone and
checks it against the C oracle.  Test infrastructure; needs both libraries built first."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
EXE = os.path.join(HERE, "selftest")


def build():
    libdir = os.path.join(ROOT, "paper_2510_20111_amd")
    oradir = os.path.join(ROOT, "oracle")
    # host code only: the system C++ compiler with the HIP runtime's headers
    cmd = ["g++", "-O2", "-std=c++17", "-Wall", os.path.join(HERE, "selftest.cpp"), "-o", EXE,
           "-I" + os.path.join(ROOT, "include"), "-I/opt/rocm/include", "-D__HIP_PLATFORM_AMD__",
           "-L" + libdir, "-l:libhzp.so", "-L" + oradir, "-l:libhzp_oracle.so",
           "-Wl,-rpath,$ORIGIN/../../paper_2510_20111_amd", "-Wl,-rpath,$ORIGIN/../../oracle",
           "-Wl,-rpath,/opt/rocm/lib", "-L/opt/rocm/lib", "-lamdhip64"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("building the native self-test failed:\n" + res.stderr)
    return EXE


if __name__ == "__main__":
    print(build())

"""Builds tests/cpu_emul/libsttm_cpu.so: the library's own sources compiled with g++ against the CPU
stand-in for HIP in this folder (test infrastructure; the product is the hipcc build)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
CSRC = os.path.join(ROOT, "paper_2507_07990_amd", "csrc")
LIB = os.path.join(HERE, "libsttm_cpu.so")
SOURCES = ["sttm_api.hip", "sttm_spatial.hip", "sttm_temporal.hip", "sttm_reduce.hip"]


SANITIZE_EXE = os.path.join(HERE, "sanitize_run")


def build_sanitized(verbose: bool = False) -> str:
    """tests/cpu_emul/sanitize_main.cpp and the library's sources in one executable, under AddressSanitizer and
    UndefinedBehaviorSanitizer (any report ends the run with a non-zero status)."""
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-pthread", "-I", HERE, "-I", CSRC, "-Wno-unknown-pragmas", "-Wno-attributes",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"]
    for s in SOURCES:
        cmd += ["-x", "c++", os.path.join(CSRC, s)]
    cmd += ["-x", "c++", os.path.join(HERE, "emul.cpp"), "-x", "c++", os.path.join(HERE, "sanitize_main.cpp"),
            "-o", SANITIZE_EXE]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return SANITIZE_EXE


def build(verbose: bool = False) -> str:
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fPIC", "-shared", "-pthread", "-I", HERE, "-I", CSRC,
           "-Wno-unknown-pragmas", "-Wno-attributes"]
    for s in SOURCES:
        cmd += ["-x", "c++", os.path.join(CSRC, s)]
    cmd += ["-x", "c++", os.path.join(HERE, "emul.cpp"), "-o", LIB]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build_sanitized(verbose=True) if "--sanitize" in sys.argv else build(verbose=True))

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


def build(sanitize: bool = False, verbose: bool = False) -> str:
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fPIC", "-shared", "-pthread", "-I", HERE, "-I", CSRC,
           "-Wno-unknown-pragmas", "-Wno-attributes"]
    if sanitize:
        # AddressSanitizer only: with -fsanitize=undefined g++ 11 sends the conditional-pointer stores of the
        # pyramid kernel ("(is_dot ? pd : pn)[i] = v") to the wrong element without any report, so results of
        # such a build mean nothing.
        cmd += ["-fsanitize=address", "-fno-omit-frame-pointer"]
    for s in SOURCES:
        cmd += ["-x", "c++", os.path.join(CSRC, s)]
    cmd += ["-x", "c++", os.path.join(HERE, "emul.cpp"), "-o", LIB]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(sanitize="--asan" in sys.argv, verbose=True))

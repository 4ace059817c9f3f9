"""Compile the C part of the CPU oracle (test infrastructure) with gcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "bns_oracle.c")
LIB = os.path.join(HERE, "libbns_oracle.so")
LIB_SANITIZED = os.path.join(HERE, "libbns_oracle_asan.so")


def build(force: bool = True) -> str:
    if force or not os.path.exists(LIB) or os.path.getmtime(LIB) < os.path.getmtime(SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-Wall", "-o", LIB, SRC, "-lm"])
    return LIB


def build_sanitized() -> str:
    """The same source under AddressSanitizer and UndefinedBehaviorSanitizer (host code only); a
    process that loads it needs gcc's libasan preloaded (sanitizer_preload())."""
    subprocess.check_call(["gcc", "-O1", "-g", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall",
                           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                           "-fno-omit-frame-pointer", "-o", LIB_SANITIZED, SRC, "-lm"])
    return LIB_SANITIZED


def sanitizer_preload() -> str:
    return subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()


if __name__ == "__main__":
    print(build())

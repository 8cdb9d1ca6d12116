"""Builds the CPU oracle (test infrastructure) into oracle/libee_oracle.so with g++.

`python -m oracle.build --sanitize` builds oracle/libee_oracle_san.so with AddressSanitizer and
UndefinedBehaviorSanitizer instead (host code only); run the CPU pins against it with
    EE_ORACLE_LIB=oracle/libee_oracle_san.so LD_PRELOAD=$(g++ -print-file-name=libasan.so) \
        ASAN_OPTIONS=detect_leaks=0 python -m pytest tests -m "not gpu" -k oracle
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "libee_oracle.so")
LIB_SAN = os.path.join(HERE, "libee_oracle_san.so")


def build(force: bool = True, sanitize: bool = False) -> str:
    src = os.path.join(HERE, "ee_oracle.cpp")
    lib = LIB_SAN if sanitize else LIB
    if not force and os.path.exists(lib) and os.path.getmtime(lib) >= max(
            os.path.getmtime(src), os.path.getmtime(os.path.join(HERE, "ee_oracle.h"))):
        return lib
    cmd = ["g++", "-std=c++17", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-ffp-contract=off"]
    if sanitize:
        cmd += ["-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"]
    subprocess.check_call(cmd + [src, "-o", lib])
    return lib


if __name__ == "__main__":
    print(build(sanitize="--sanitize" in sys.argv[1:]))

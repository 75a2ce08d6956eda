"""Compile the fp64 CPU oracle (test infrastructure) into oracle/libchela_oracle.so with gcc.

build(sanitize=True) makes a second library, oracle/libchela_oracle_san.so, with AddressSanitizer and
UndefinedBehaviorSanitizer compiled in (-O1, frame pointers kept, undefined behaviour is fatal): the pin tests are run
against it as well, in a child process that preloads the sanitizer's runtime (tests/test_sanitizers.py)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "chela_oracle.c")
LIB = os.path.join(HERE, "libchela_oracle.so")
LIB_SAN = os.path.join(HERE, "libchela_oracle_san.so")


def build(force: bool = False, sanitize: bool = False) -> str:
    lib = LIB_SAN if sanitize else LIB
    if (not force) and os.path.exists(lib) and os.path.getmtime(lib) >= os.path.getmtime(SRC):
        return lib
    if sanitize:
        opt = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"]
    else:
        opt = ["-O2"]     # without -ffast-math: the summation order stays the one the source states
    cmd = ["gcc", *opt, "-std=c11", "-fopenmp", "-fPIC", "-shared", "-o", lib, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return lib


def asan_runtime() -> str:
    """Path of the AddressSanitizer runtime that a process loading the sanitized library has to preload."""
    return subprocess.run(["gcc", "-print-file-name=libasan.so"], check=True, stdout=subprocess.PIPE,
                          text=True).stdout.strip()


if __name__ == "__main__":
    print(build(force=True))

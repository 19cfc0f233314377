"""Compile the CPU oracles (test infrastructure) with g++: oracle/libgo_oracle.so and oracle/libhex_oracle.so.

`python oracle/build.py --sanitize` (or ORACLE_SANITIZE=1 in the environment of a test run) builds and selects
AddressSanitizer + UndefinedBehaviorSanitizer variants (lib*_san.so) of the same sources; a process that loads them
must have the ASan runtime preloaded (LD_PRELOAD=$(gcc -print-file-name=libasan.so)), as tests/test_oracle_sanitized.py does.
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "go_oracle.cpp")
HEX_SRC = os.path.join(HERE, "hex_oracle.cpp")
SANITIZE = os.environ.get("ORACLE_SANITIZE") == "1"
LIB = os.path.join(HERE, "libgo_oracle_san.so" if SANITIZE else "libgo_oracle.so")
HEX_LIB = os.path.join(HERE, "libhex_oracle_san.so" if SANITIZE else "libhex_oracle.so")
SAN_FLAGS = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g", "-O1"]


def _compile(src, lib, force, sanitize):
    if not force and os.path.exists(lib) and os.path.getmtime(lib) >= os.path.getmtime(src):
        return lib
    opt = SAN_FLAGS if sanitize else ["-O2"]
    subprocess.run(["g++", "-std=c++17", *opt, "-fPIC", "-shared", "-Wall", "-Wextra", "-o", lib, src], check=True)
    return lib


def build(force: bool = True, sanitize: bool = SANITIZE) -> str:
    return _compile(SRC, os.path.join(HERE, "libgo_oracle_san.so" if sanitize else "libgo_oracle.so"), force, sanitize)


def build_hex(force: bool = True, sanitize: bool = SANITIZE) -> str:
    return _compile(HEX_SRC, os.path.join(HERE, "libhex_oracle_san.so" if sanitize else "libhex_oracle.so"), force, sanitize)


def asan_runtime() -> str:
    """Path of the AddressSanitizer runtime a process must preload before it can load the sanitized oracles."""
    return subprocess.run(["g++", "-print-file-name=libasan.so"], check=True, capture_output=True, text=True).stdout.strip()


if __name__ == "__main__":
    san = "--sanitize" in sys.argv[1:]
    print(build(sanitize=san))
    print(build_hex(sanitize=san))

"""Compile the CPU oracles (test infrastructure) with g++: oracle/libgo_oracle.so and oracle/libhex_oracle.so."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "go_oracle.cpp")
LIB = os.path.join(HERE, "libgo_oracle.so")
HEX_SRC = os.path.join(HERE, "hex_oracle.cpp")
HEX_LIB = os.path.join(HERE, "libhex_oracle.so")


def _compile(src, lib, force):
    if not force and os.path.exists(lib) and os.path.getmtime(lib) >= os.path.getmtime(src):
        return lib
    subprocess.run(["g++", "-std=c++17", "-O2", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", lib, src], check=True)
    return lib


def build(force: bool = True) -> str:
    return _compile(SRC, LIB, force)


def build_hex(force: bool = True) -> str:
    return _compile(HEX_SRC, HEX_LIB, force)


if __name__ == "__main__":
    print(build())
    print(build_hex())

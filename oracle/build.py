"""Compile the C oracle into oracle/libf8ref.so with gcc (test infrastructure)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "f8_ref.c")
LIB = os.path.join(HERE, "libf8ref.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= max(
            os.path.getmtime(SRC), os.path.getmtime(os.path.join(HERE, "f8_ref.h"))):
        return LIB
    cmd = ["gcc", "-O2", "-std=c99", "-Wall", "-Wextra", "-fPIC", "-shared", "-o", LIB, SRC]
    subprocess.run(cmd, check=True)
    return LIB


SAN_LIB = os.path.join(HERE, "libf8ref_san.so")


def build_sanitized() -> str:
    """The same source under AddressSanitizer and UndefinedBehaviorSanitizer (bad shifts, signed
    overflow, out-of-bounds indexing abort the process): for the test that re-runs the pins on it."""
    cmd = ["gcc", "-O1", "-g", "-std=c99", "-Wall", "-Wextra", "-fPIC", "-shared",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-o", SAN_LIB, SRC]
    subprocess.run(cmd, check=True)
    return SAN_LIB


if __name__ == "__main__":
    print(build())

"""Compile the C oracle (oracle/svgd_oracle.c) into oracle/libsvgd_oracle.so with gcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "svgd_oracle.c")
LIB = os.path.join(HERE, "libsvgd_oracle.so")


def build(force: bool = False) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
           "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


SAN_SRC = os.path.join(HERE, "sanitize_check.c")
SAN_EXE = os.path.join(HERE, "sanitize_check")


def build_sanitized() -> str:
    """The oracle and its driver (sanitize_check.c) as one executable under AddressSanitizer and
    UndefinedBehaviorSanitizer (host code only); returns its path.  Run it: exit status 0 = clean."""
    cmd = ["gcc", "-O1", "-g", "-fopenmp", "-std=c11", "-Wall", "-Wextra",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           "-o", SAN_EXE, SAN_SRC, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return SAN_EXE


if __name__ == "__main__":
    print(build(force=True))

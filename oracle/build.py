"""Compile the CPU checker (oracle.c) into liboracle.so next to this file.

build(sanitize=True) makes a second library, liboracle_san.so, with AddressSanitizer and
UndefinedBehaviorSanitizer compiled in; the package loads it instead when ORACLE_SANITIZED=1 is set
(the sanitizer runtime then has to be preloaded into the Python process, see
tests/test_oracle_sanitized.py)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "oracle.c")
LIB = os.path.join(HERE, "liboracle.so")
LIB_SAN = os.path.join(HERE, "liboracle_san.so")


def build(force=False, sanitize=False):
    out = LIB_SAN if sanitize else LIB
    if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(SRC):
        return out
    flags = (["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer"]
             if sanitize else ["-O2"])
    cmd = ["gcc"] + flags + ["-std=c99", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                             "-ffp-contract=off", "-o", out, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return out


def sanitizer_runtime():
    """Path of the AddressSanitizer runtime the sanitized library needs preloaded."""
    return subprocess.run(["gcc", "-print-file-name=libasan.so"], check=True, capture_output=True, text=True).stdout.strip()


if __name__ == "__main__":
    import sys
    print(build(force=True, sanitize="--sanitize" in sys.argv))

"""Compile the CPU oracle (plain C, gcc) into oracle/liboracle_wk.so."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "wk_oracle.c")
LIB = os.path.join(HERE, "liboracle_wk.so")


def build(force: bool = True) -> str:
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-std=c99", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
           "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


def build_sanitized(out_path: str) -> str:
    """The same source with AddressSanitizer and UndefinedBehaviorSanitizer (host checks of the checker itself).
    The result must be loaded into a process that has gcc's libasan preloaded."""
    cmd = ["gcc", "-std=c99", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=undefined", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", out_path, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return out_path


def sanitizer_runtime() -> str:
    """Path of the libasan.so that a process loading a build_sanitized() library must preload."""
    return subprocess.run(["gcc", "-print-file-name=libasan.so"], check=True, capture_output=True, text=True).stdout.strip()


if __name__ == "__main__":
    print(build(force=True))
    sys.exit(0)

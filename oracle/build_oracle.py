"""Compile the CPU oracle (plain C, fp64) into oracle/liborc.so with gcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
LIB = os.path.join(HERE, "liborc.so")


def build_oracle(force: bool = True, sanitize: bool = False, out: str = LIB) -> str:
    """sanitize=True builds with AddressSanitizer and UndefinedBehaviorSanitizer (host code only); the
    tests then run as
        ORC_LIB=<out> LD_PRELOAD=$(gcc -print-file-name=libasan.so) ASAN_OPTIONS=detect_leaks=0 \
            python -m pytest tests -m "not gpu" -k "oracle or balance or table2"
    """
    src = os.path.join(HERE, "tj_oracle.c")
    if not force and os.path.exists(out) and os.path.getmtime(out) >= os.path.getmtime(src):
        return out
    opt = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-omit-frame-pointer"] if sanitize else ["-O2"]
    cmd = ["gcc"] + opt + ["-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra", src, "-o", out, "-lm"]
    subprocess.run(cmd, check=True)
    return out


if __name__ == "__main__":
    import sys

    if "--sanitize" in sys.argv:
        print(build_oracle(sanitize=True, out=os.path.join(HERE, "liborc_asan.so")))
    else:
        print(build_oracle())

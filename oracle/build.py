"""Compile oracle.c into liboracle.so with gcc (-O2, no fast-math, OpenMP over rows)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "oracle.c")
LIB = os.path.join(HERE, "liboracle.so")


def build(force: bool = False) -> str:
    if os.environ.get("MLORA_ORACLE_LIB"):             # a prebuilt variant (the sanitizer test sets this)
        return os.environ["MLORA_ORACLE_LIB"]
    if not force and os.path.exists(LIB) and os.path.getmtime(LIB) >= os.path.getmtime(SRC):
        return LIB
    cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-shared", "-fPIC", "-o", LIB, SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return LIB


def build_sanitized(outdir: str, cc: str) -> str:
    """The oracle under AddressSanitizer and UndefinedBehaviorSanitizer, compiled with `cc` (the
    clang whose sanitizer runtime the process preloads), for the CPU test that runs the pins that way."""
    os.makedirs(outdir, exist_ok=True)
    lib = os.path.join(outdir, "liboracle_san.so")
    subprocess.run([cc, "-O1", "-g", "-std=c99", "-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined",
                    "-fno-omit-frame-pointer", "-shared-libsan", "-shared", "-fPIC", "-o", lib, SRC, "-lm"], check=True)
    return lib


if __name__ == "__main__":
    print(build(force=True))

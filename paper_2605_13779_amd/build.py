"""Build libmlora.so (the C-ABI library) for gfx950 with hipcc, in-tree."""
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmlora.so")
SOURCES = ["api.hip", "plan.hip", "rows.hip", "seg_mfma.hip", "moe_down.hip", "resident.hip"]
# packed-fp32 VALU forms are switched off for all device code: hipcc forms them by itself from plain
# float code and some of those forms have given wrong results on this hardware
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def _compile(src: str) -> str:
    obj = os.path.join(CSRC, src.replace(".hip", ".o"))
    subprocess.run(["hipcc", *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj], check=True,
                   stderr=subprocess.PIPE if os.environ.get("MLORA_QUIET") else None)
    return obj


def build(verbose: bool = False) -> str:
    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(_compile, SOURCES))
    subprocess.run(["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB, *objs], check=True)
    if verbose:
        print("built", LIB)
    return LIB


SAN_HOST = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
            "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer"]


def build_sanitized(outdir: str) -> str:
    """The same library with its HOST code under AddressSanitizer and UndefinedBehaviorSanitizer (the
    device code is compiled as usual): for the CPU test that runs the host-side logic -- validation,
    the residency manager, the packing of per-expert tensors -- under the sanitizers.  Returns the
    path of the library in `outdir`; the process that loads it must preload the matching runtime
    (sanitizer_runtime())."""
    os.makedirs(outdir, exist_ok=True)
    flags = [f if f != "-O3" else "-O1" for f in FLAGS] + ["-g"] + SAN_HOST

    def one(src):
        obj = os.path.join(outdir, src.replace(".hip", ".o"))
        subprocess.run(["hipcc", *flags, "-c", os.path.join(CSRC, src), "-o", obj], check=True, stderr=subprocess.PIPE)
        return obj
    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(one, SOURCES))
    lib = os.path.join(outdir, "libmlora_san.so")
    subprocess.run(["hipcc", "-shared", "-fPIC", "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined",
                    "-shared-libsan", "-o", lib, *objs], check=True, stderr=subprocess.PIPE)
    return lib


def sanitizer_clang() -> str:
    """The clang that hipcc drives (its sanitizer runtime is the one build_sanitized links against)."""
    out = subprocess.run(["hipcc", "--version"], check=True, capture_output=True, text=True).stdout
    for line in out.splitlines():
        if line.startswith("InstalledDir:"):
            return os.path.join(line.split(":", 1)[1].strip(), "clang")
    raise RuntimeError("hipcc --version names no InstalledDir")


def sanitizer_runtime() -> str:
    return subprocess.run([sanitizer_clang(), "-print-file-name=libclang_rt.asan-x86_64.so"], check=True,
                          capture_output=True, text=True).stdout.strip()


if __name__ == "__main__":
    build(verbose=True)

"""Build the host translation units of libsaga against the CPU stand-in of the HIP runtime (g++, no GPU code):
tests/hoststub/_build/libsaga_hoststub_asan.so with AddressSanitizer and UBSan, libsaga_hoststub_tsan.so with
ThreadSanitizer. Test infrastructure only."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
CSRC = os.path.join(ROOT, "paper_1810_08403_amd", "csrc")
OUT_DIR = os.path.join(HERE, "_build")
HOST_UNITS = ["saga_api.hip", "chunked.hip", "backward.hip"]     # the units without kernels
STUB_UNITS = ["stub_runtime.cpp", "stub_kernels.cpp"]


def lib_path(sanitize=True):
    name = {True: "libsaga_hoststub_asan.so", False: "libsaga_hoststub.so", "thread": "libsaga_hoststub_tsan.so"}[sanitize]
    return os.path.join(OUT_DIR, name)


def build(sanitize=True, force=False):
    os.makedirs(OUT_DIR, exist_ok=True)
    out = lib_path(sanitize)
    srcs = [os.path.join(CSRC, u) for u in HOST_UNITS] + [os.path.join(HERE, u) for u in STUB_UNITS]
    deps = srcs + [os.path.join(CSRC, "saga_internal.h"), os.path.join(ROOT, "include", "saga.h"), os.path.join(HERE, "hip", "hip_runtime.h")]
    if not force and os.path.exists(out) and all(os.path.getmtime(out) >= os.path.getmtime(d) for d in deps):
        return out
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fPIC", "-shared", "-pthread", "-fno-omit-frame-pointer", f"-I{HERE}", f"-I{CSRC}"]
    if sanitize == "thread":
        cmd += ["-fsanitize=thread"]
    elif sanitize:
        cmd += ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"]
    cmd += ["-x", "c++"] + srcs + ["-o", out]
    subprocess.run(cmd, check=True)
    return out


def asan_runtime():
    return subprocess.run(["gcc", "-print-file-name=libasan.so"], check=True, capture_output=True, text=True).stdout.strip()


def tsan_runtime():
    return subprocess.run(["gcc", "-print-file-name=libtsan.so"], check=True, capture_output=True, text=True).stdout.strip()


if __name__ == "__main__":
    print(build(sanitize="--plain" not in sys.argv, force=True))

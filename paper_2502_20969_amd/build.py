"""Builds libivf.so (HIP kernels + C-ABI) for gfx950 with hipcc, in-tree."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(CSRC, "_build")
LIB = os.path.join(HERE, "libivf.so")

HIP_SOURCES = ["ivf_kernels.hip", "ivf_batched.hip", "ivf_sched.hip", "ivf_api.hip"]
HOST_SOURCES = ["host_scan.cpp", "host_plan.cpp"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
CLANG = os.environ.get("IVF_HOST_CLANG", "/opt/rocm/llvm/bin/clang")     # host compiler of the sanitizer builds (knows _Float16)
COMMON = ["-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-result"]
# packed-fp32 instructions are switched off for all device code.  The driver cannot forward
# -Xclang through -Xarch_device, so the host pass sees the feature too and says it does not know
# it; that one line is dropped from the compiler's output below.
DEVICE = ["--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
HOST_PASS_NOTE = "'-packed-fp32-ops' is not a recognized feature for this target"
HOST_SIMD = ["-mavx2", "-mfma", "-mf16c"]


def _compile(src):
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    path = os.path.join(CSRC, src)
    if src.endswith(".hip"):
        cmd = [HIPCC, *COMMON, *DEVICE, "-c", path, "-o", obj]
    else:
        cmd = [HIPCC, *COMMON, *HOST_SIMD, "-x", "c++", "-c", path, "-o", obj]
    r = subprocess.run(cmd, stderr=subprocess.PIPE, text=True)
    noise = [l for l in r.stderr.splitlines() if HOST_PASS_NOTE not in l]
    if noise:
        print("\n".join(noise), file=sys.stderr)
    if r.returncode != 0:
        raise subprocess.CalledProcessError(r.returncode, cmd)
    return obj


def build() -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(_compile, HIP_SOURCES + HOST_SOURCES))
    subprocess.run([HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", LIB, *objs, "-lpthread"],
                   check=True)
    return LIB


def build_sanitized() -> list:
    """CPU only: the host side of the library (host scan, planners) and the C oracle with a driver
    that checks one against the other, once under the address + undefined-behaviour sanitizers and
    once under the thread sanitizer.  Returns the two executables."""
    root = os.path.dirname(HERE)
    os.makedirs(OBJ, exist_ok=True)
    cxx_src = [os.path.join(CSRC, "host_scan.cpp"), os.path.join(CSRC, "host_plan.cpp"),
               os.path.join(root, "tests", "sanitize", "host_san_driver.cpp")]
    out = []
    for name, flags in (("asan", ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined"]),
                        ("tsan", ["-fsanitize=thread"])):
        oracle_obj = os.path.join(OBJ, f"oracle_{name}.o")
        subprocess.run([CLANG, "-O1", "-g", "-std=c11", "-fno-omit-frame-pointer", *flags, "-c",
                        os.path.join(root, "oracle", "ivf_oracle.c"), "-o", oracle_obj], check=True)
        exe = os.path.join(OBJ, f"host_san_{name}")
        subprocess.run([CLANG + "++", "-O1", "-g", "-std=c++17", "-fno-omit-frame-pointer", *HOST_SIMD, *flags, *cxx_src, oracle_obj,
                        "-o", exe, "-lpthread", "-lm"], check=True)
        out.append(exe)
    return out


if __name__ == "__main__":
    if "--sanitize" in sys.argv[1:]:
        for exe in build_sanitized():
            print(exe)
            subprocess.run([exe], check=True)
    else:
        print(build())

"""Compile the HIP sources under csrc/ for gfx950 into paper_2605_22718_amd/libwk.so."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libwk.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall",
    # packed-fp32 instructions are kept out of every kernel of this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def sources():
    return sorted(os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hip"))


# per-file additions: the attention kernels take row maxima of finite logits (and -inf), never NaN
EXTRA = {"wk_attention.hip": ["-fno-honor-nans"]}


def _compile(src: str) -> str:
    obj = os.path.join(OBJ, os.path.basename(src)[:-4] + ".o")
    extra = EXTRA.get(os.path.basename(src), [])
    r = subprocess.run([HIPCC, *FLAGS, *extra, "-c", src, "-o", obj], capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(force: bool = True) -> str:
    srcs = sources()
    deps = srcs + [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    deps.append(os.path.join(ROOT, "include", "wk.h"))
    if not force and os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(d) for d in deps):
        return LIB
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, len(srcs))) as ex:
        objs = list(ex.map(_compile, srcs))
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], check=True)
    return LIB


DRIVER_SRC = os.path.join(HERE, "profile_driver", "wk_profile_driver.cpp")
DRIVER = os.path.join(HERE, "profile_driver", "wk_profile_driver")


def build_profile_driver() -> str:
    """The torch-free program the hardware-counter profiles are taken on (host code only; it calls libwk.so)."""
    subprocess.run([HIPCC, "-O2", "-std=c++17", "-x", "c++", "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(ROOT, "include"),
                    "-I", "/opt/rocm/include", DRIVER_SRC, "-o", DRIVER, "-L", HERE, "-lwk", "-L", "/opt/rocm/lib", "-lamdhip64",
                    "-Wl,-rpath,$ORIGIN/..", "-Wl,-rpath,/opt/rocm/lib"], check=True)
    return DRIVER


PROBE_SRC = os.path.join(HERE, "profile_driver", "wk_mfma_duty_probe.hip")
PROBE = os.path.join(HERE, "profile_driver", "wk_mfma_duty_probe")


def build_mfma_duty_probe() -> str:
    """The matrix-instruction duty probe (clock and rate of bare bf16 MFMA loops): a program of its own, no libwk."""
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
                        "-packed-fp32-ops", PROBE_SRC, "-o", PROBE], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {PROBE_SRC}:\n{r.stderr}")
    return PROBE


SAN_HOST = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
            "-Xarch_host", "-fno-sanitize-recover=undefined", "-g"]


def build_host_sanitized(out_dir: str) -> str:
    """libwk with AddressSanitizer and UndefinedBehaviorSanitizer in its HOST code (argument checks, planners,
    the host-only entry points); device code is compiled as usual.  The result must be loaded into a process
    that has the runtime of sanitizer_runtime() preloaded.  Returns the library's path."""
    os.makedirs(out_dir, exist_ok=True)

    def one(src):
        obj = os.path.join(out_dir, os.path.basename(src)[:-4] + ".o")
        flags = [f for f in FLAGS if f != "-O3"] + ["-O1"]
        r = subprocess.run([HIPCC, *flags, *EXTRA.get(os.path.basename(src), []), *SAN_HOST, "-c", src, "-o", obj],
                           capture_output=True, text=True)
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed on {src}:\n{r.stderr}")
        return obj
    with ThreadPoolExecutor(max_workers=8) as ex:
        objs = list(ex.map(one, sources()))
    lib = os.path.join(out_dir, "libwk_hostsan.so")
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined",
                    "-fno-gpu-sanitize", "-shared-libsan", "-o", lib, *objs], check=True)
    return lib


def sanitizer_runtime() -> str:
    """Path of the AddressSanitizer runtime (clang's) that a process loading build_host_sanitized()'s library
    must preload."""
    clang = os.path.join(os.path.dirname(os.path.realpath(HIPCC)), "..", "llvm", "bin", "clang")
    if not os.path.exists(clang):
        clang = "/opt/rocm/llvm/bin/clang"
    return subprocess.run([clang, "-print-file-name=libclang_rt.asan-x86_64.so"], check=True, capture_output=True,
                          text=True).stdout.strip()


if __name__ == "__main__":
    print(build(force=True))

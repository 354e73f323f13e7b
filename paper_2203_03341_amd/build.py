"""Compiles the HIP sources into libecgemm.so for gfx950 (hipcc cross-compiles without a GPU).

The kernels are spread over several translation units (csrc/kernels_*.hip, see csrc/kernel_list.hpp) that are
compiled side by side; objects go to _build/ next to this file."""
from __future__ import annotations

import glob
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libecgemm.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# packed FP32 instructions are switched off on purpose (they have been seen to miscompute on this fleet)
# -fno-strict-enums: the C-ABI takes enumerations from C callers, for whom they are plain integers; the argument checks
# must see whatever value was passed, so the compiler may not assume that it is one of the enumerators
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-command-line-argument",
         "-fno-strict-enums", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
NOISE = "is not a recognized feature for this target"


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def _run(cmd):
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if NOISE not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed: " + " ".join(cmd) + "\n" + err)
    return err


def _check_no_kernel_left_undefined(lib: str) -> None:
    """Every kernel is compiled in one translation unit and only declared in the others; a kernel that its own unit
    failed to emit would stay an undefined symbol of the library and only show when it is first launched."""
    res = subprocess.run(["nm", "-D", "-C", "--undefined-only", lib], capture_output=True, text=True)
    missing = [l.strip() for l in res.stdout.splitlines() if "ecgemm::" in l]
    if missing:
        raise RuntimeError("kernels declared but compiled nowhere:\n" + "\n".join(missing))


def build(verbose: bool = False, extra_flags=(), lib: str = LIB, obj_dir: str = OBJ_DIR) -> str:
    os.makedirs(obj_dir, exist_ok=True)
    srcs = sources()
    objs = [os.path.join(obj_dir, os.path.basename(s)[:-4] + ".o") for s in srcs]
    jobs = min(len(srcs), max(1, min(16, os.cpu_count() or 1)))
    with ThreadPoolExecutor(jobs) as pool:
        logs = list(pool.map(lambda so: _run([HIPCC, *FLAGS, *extra_flags, "-c", so[0], "-o", so[1]]), zip(srcs, objs)))
    logs.append(_run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs]))
    _check_no_kernel_left_undefined(lib)
    if verbose:
        for log in logs:
            if log.strip():
                print(log)
    return lib


CLANGXX = os.environ.get("ECGEMM_CLANGXX", "/opt/rocm/lib/llvm/bin/clang++")
SANITIZED_LIB = os.path.join(OBJ_DIR, "libecgemm_sanitized.so")


def build_host_sanitized() -> str:
    """The same library with its host code (argument checks, planner, workspace logic: all of it in ecgemm.hip)
    compiled under AddressSanitizer and UndefinedBehaviorSanitizer, for CPU-only tests of the host side.  Device code
    is not instrumented.  The kernel translation units are reused from the ordinary build when they are up to date."""
    os.makedirs(OBJ_DIR, exist_ok=True)
    headers = glob.glob(os.path.join(CSRC, "*.hpp")) + glob.glob(os.path.join(HERE, "..", "include", "*.h"))
    newest_header = max(os.path.getmtime(h) for h in headers)
    jobs, objs = [], []
    for src in sources():
        name = os.path.basename(src)[:-4]
        host = name == "ecgemm"
        obj = os.path.join(OBJ_DIR, name + ("_sanitized.o" if host else ".o"))
        objs.append(obj)
        if not os.path.exists(obj) or os.path.getmtime(obj) < max(os.path.getmtime(src), newest_header):
            # (the enum check is left out: out-of-range enumeration arguments are legal input here, see FLAGS)
            sanitize = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
                        "-fno-sanitize=enum", "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host",
                        "-fno-omit-frame-pointer", "-g"] if host else []
            jobs.append([HIPCC, *FLAGS, *sanitize, "-c", src, "-o", obj])
    with ThreadPoolExecutor(max(1, min(8, len(jobs) or 1))) as pool:
        list(pool.map(_run, jobs))
    _run([CLANGXX, "-shared", "-fPIC", "-fsanitize=address,undefined", "-shared-libsan", "-o", SANITIZED_LIB, *objs,
          "-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath,/opt/rocm/lib"])
    return SANITIZED_LIB


if __name__ == "__main__":
    print(build(verbose=True))

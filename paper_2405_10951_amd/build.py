"""Build libbsr_hip.so (the HIP kernels and the C ABI of include/bsr.h) for gfx950, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libbsr_hip.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=fast",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument"]


def sources() -> list[str]:
    return sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))


def _compile(src: str, force: bool, obj_dir: str = OBJ, extra: tuple = ()) -> str:
    obj = os.path.join(obj_dir, src[:-4] + ".o")
    deps = [os.path.join(CSRC, src), os.path.join(CSRC, "bsr_internal.h"),
            os.path.join(HERE, "..", "include", "bsr.h")]
    if not force and os.path.exists(obj) and all(os.path.getmtime(obj) >= os.path.getmtime(d) for d in deps):
        return obj
    cmd = [HIPCC, *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    return obj


def build(force: bool = False, jobs: int = 8) -> str:
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, force), sources()))
    if force or not os.path.exists(LIB) or any(os.path.getmtime(o) > os.path.getmtime(LIB) for o in objs):
        subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs], check=True)
    return LIB


# host code only: the GPU side of a sanitized build is the ordinary one
SANITIZE = ("-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
            "-Xarch_host", "-fno-omit-frame-pointer", "-g")


def build_sanitized_program(main_c: str, out_dir: str, jobs: int = 8) -> str:
    """Link the C program main_c (which calls the C ABI of include/bsr.h) with the library's objects rebuilt with
    AddressSanitizer and UndefinedBehaviorSanitizer in their host code; -> path of the executable.  A program
    rather than a shared library: the sanitizer runtime is linked into it, nothing has to be preloaded."""
    obj_dir = os.path.join(out_dir, "obj")
    os.makedirs(obj_dir, exist_ok=True)
    with ThreadPoolExecutor(max_workers=jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, True, obj_dir, SANITIZE), sources()))
    exe = os.path.join(out_dir, os.path.splitext(os.path.basename(main_c))[0])
    r = subprocess.run([HIPCC, "--offload-arch=gfx950", "-fsanitize=address", "-fsanitize=undefined", "-fno-gpu-sanitize",
                        "-g", "-I", os.path.join(HERE, "..", "include"), "-x", "c", main_c, "-x", "none", *objs,
                        "-o", exe], capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"linking {exe} failed:\n{r.stderr}")
    return exe


if __name__ == "__main__":
    print(build(force="--force" in sys.argv))

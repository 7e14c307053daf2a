"""Builds libdsk.so (gfx950) from csrc/*.hip, libdsk_diag.so (device measurements for benchmarks) from
csrc/diag/*.hip, and dsk_c_demo (examples/c_abi_demo.c, plain C against the C ABI, compiled by gcc), in-tree, next to this
file; the libraries are compiled by hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
OBJ_DIR = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libdsk.so")
DIAG_LIB = os.path.join(HERE, "libdsk_diag.so")
C_DEMO = os.path.join(HERE, "dsk_c_demo")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def sources(sub: str = ""):
    d = os.path.join(CSRC, sub)
    return sorted(os.path.join(sub, f) for f in os.listdir(d) if f.endswith(".hip"))


def _compile(src: str, force: bool) -> str:
    obj = os.path.join(OBJ_DIR, src[:-4].replace(os.sep, "_") + ".o")
    spath = os.path.join(CSRC, src)
    deps = [spath] + [os.path.join(CSRC, h) for h in os.listdir(CSRC) if h.endswith(".h")]
    deps += [os.path.join(ROOT, "include", h) for h in os.listdir(os.path.join(ROOT, "include"))]
    if not force and os.path.exists(obj) and all(os.path.getmtime(obj) >= os.path.getmtime(d) for d in deps):
        return obj
    cmd = [HIPCC, *FLAGS, "-c", spath, "-o", obj]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed for {src}:\n{r.stdout}\n{r.stderr}")
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in r.stderr.splitlines() if noise not in l).strip()
    if err:
        sys.stderr.write(err + "\n")
    return obj


def _link(lib: str, objs) -> None:
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"link failed:\n{r.stdout}\n{r.stderr}")


def _build_c_demo() -> None:
    """examples/c_abi_demo.c: a plain C program against include/dsk.h, libdsk.so and the HIP runtime."""
    src = os.path.join(HERE, "examples", "c_abi_demo.c")
    rocm = os.path.dirname(os.path.dirname(os.path.realpath(HIPCC)))
    cmd = ["gcc", "-std=c11", "-O2", "-Wall", "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(rocm, "include"),
           "-I", os.path.join(ROOT, "include"), src, "-L", HERE, "-ldsk", "-L", os.path.join(rocm, "lib"), "-lamdhip64", "-lm",
           "-Wl,-rpath,$ORIGIN", "-Wl,-rpath," + os.path.join(rocm, "lib"), "-o", C_DEMO]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError(f"building the C demo failed:\n{r.stdout}\n{r.stderr}")


def build(force: bool = True, jobs: int = 8) -> str:
    os.makedirs(OBJ_DIR, exist_ok=True)
    main, diag = sources(), sources("diag")
    with ThreadPoolExecutor(jobs) as ex:
        objs = list(ex.map(lambda s: _compile(s, force), main + diag))
    _link(LIB, objs[:len(main)])
    _link(DIAG_LIB, objs[len(main):])
    _build_c_demo()
    return LIB


if __name__ == "__main__":
    print(build(force="--incremental" not in sys.argv))

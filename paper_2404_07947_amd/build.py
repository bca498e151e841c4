"""Builds libexe.so (HIP kernels + runtime + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libexe.so")
SOURCES = ["kernels_elementwise.hip", "kernels_gemm.hip", "kernels_attn.hip", "runtime.hip", "probe.hip", "sched.cpp"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _headers_mtime() -> float:
    hs = [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".h")]
    inc = os.path.join(HERE, "..", "include")
    hs += [os.path.join(inc, f) for f in os.listdir(inc) if f.endswith(".h")]
    return max(os.path.getmtime(h) for h in hs)


def build(force: bool = False, verbose: bool = True) -> str:
    os.makedirs(OBJ, exist_ok=True)
    hm = _headers_mtime()

    def compile_one(src: str) -> str:
        s = os.path.join(CSRC, src)
        o = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
        if not force and os.path.exists(o) and os.path.getmtime(o) >= max(os.path.getmtime(s), hm):
            return o
        cmd = [HIPCC, *FLAGS, "-c", s, "-o", o]
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, capture_output=True, text=True)
        msgs = "\n".join(l for l in (r.stdout + r.stderr).splitlines()
                         if "packed-fp32-ops" not in l and l.strip())
        if r.returncode != 0:
            raise RuntimeError(f"hipcc failed for {src}:\n{msgs}")
        if msgs and verbose:
            print(msgs, flush=True)
        return o

    with ThreadPoolExecutor(max_workers=4) as ex:
        objs = list(ex.map(compile_one, SOURCES))
    if force or not os.path.exists(LIB) or any(os.path.getmtime(o) > os.path.getmtime(LIB) for o in objs):
        cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB + ".tmp", *objs]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
        os.replace(LIB + ".tmp", LIB)
    return LIB


def build_variant(tag: str, defines, verbose: bool = True) -> str:
    """Builds libexe_<tag>.so: the library with the tile GEMM compiled as a measurement variant (defines such as
    -DEXE_GEMM_ABLATE=1 or -DEXE_GEMM_ISSUE_AT=1, see csrc/kernels_gemm.hip; an ablated variant's results are
    meaningless, its timing isolates a part of the kernel).  The other objects are the library's own."""
    build(verbose=verbose)
    obj = os.path.join(OBJ, f"kernels_gemm_{tag}.o")
    cmd = [HIPCC, *FLAGS, *defines, "-c", os.path.join(CSRC, "kernels_gemm.hip"), "-o", obj]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + "\n".join(l for l in (r.stdout + r.stderr).splitlines() if "packed-fp32-ops" not in l))
    objs = [obj if src == "kernels_gemm.hip" else os.path.join(OBJ, os.path.splitext(src)[0] + ".o") for src in SOURCES]
    lib = os.path.join(HERE, f"libexe_{tag}.so")
    subprocess.run([HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib, *objs], check=True)
    return lib


if __name__ == "__main__":
    if "--variant" in sys.argv:
        print(build_variant(sys.argv[sys.argv.index("--variant") + 1], [a for a in sys.argv if a.startswith("-D")]))
    else:
        build(force="--force" in sys.argv)

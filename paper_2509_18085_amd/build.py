"""Compile csrc/*.hip for gfx950 into paper_2509_18085_amd/libspiffy.so (in-tree).

Usage: python -m paper_2509_18085_amd.build     (cross-compiles without a GPU)
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libspiffy.so")
SOURCES = ["api.hip", "generic_kernels.hip", "graph_accept.hip", "draft_prune.hip", "head_topk.hip", "subgraph_search.hip", "mfma_gemm.hip", "mfma_attn.hip"]
PROBE_LIB = os.path.join(HERE, "libspiffy_probe.so")     # bench-only: measured peaks of the machine (csrc/probe.hip)
# -ffp-contract=on: a multiply and an add are fused only where the source writes them in one expression, so the
# rounding of a kernel does not depend on how the optimiser inlined or ordered it (different instantiations of one
# kernel body have to agree bit for bit)
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden", "-ffp-contract=on",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def _hipcc() -> str:
    for c in (shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if c and os.path.exists(c):
            return c
    raise RuntimeError("hipcc not found")


def _run(cmd):
    p = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in p.stdout.splitlines() if "not a recognized feature for this target" not in l)
    if p.returncode != 0:
        raise RuntimeError("command failed: %s\n%s" % (" ".join(cmd), out))
    return out


def build(verbose: bool = False) -> str:
    os.makedirs(OBJ, exist_ok=True)
    hipcc = _hipcc()
    objs = [os.path.join(OBJ, s.replace(".hip", ".o")) for s in SOURCES]

    def one(i):
        return _run([hipcc] + FLAGS + ["-c", os.path.join(CSRC, SOURCES[i]), "-o", objs[i]])

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as ex:
        outs = list(ex.map(one, range(len(SOURCES))))
    outs.append(_run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs))
    outs.append(_run([hipcc] + FLAGS + ["-shared", "-o", PROBE_LIB, os.path.join(CSRC, "probe.hip")]))
    if verbose:
        print("\n".join(o for o in outs if o.strip()))
    return LIB


def build_host_sanitized() -> tuple:
    """The same library with the HOST code of the launcher (csrc/api.hip: argument checks, workspace carving, kernel
    selection) compiled under AddressSanitizer and UndefinedBehaviorSanitizer; device code and the kernel translation
    units are the normal ones.  Returns (library path, sanitizer runtime to preload).  For the CPU tests only."""
    if not all(os.path.exists(os.path.join(OBJ, s.replace(".hip", ".o"))) for s in SOURCES):
        build()
    out_dir = os.path.join(OBJ, "asan")
    os.makedirs(out_dir, exist_ok=True)
    hipcc = _hipcc()
    api_o = os.path.join(out_dir, "api.o")
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
           "-fno-sanitize-recover=undefined"]
    flags = [f if f != "-O3" else "-O1" for f in FLAGS] + ["-g"]
    _run([hipcc] + flags + san + ["-c", os.path.join(CSRC, "api.hip"), "-o", api_o])
    objs = [api_o] + [os.path.join(OBJ, s.replace(".hip", ".o")) for s in SOURCES if s != "api.hip"]
    lib = os.path.join(out_dir, "libspiffy_asan.so")
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address,undefined", "-o", lib] + objs)
    clang = os.path.join(os.path.dirname(os.path.realpath(hipcc)), "..", "lib", "llvm", "bin", "clang")
    if not os.path.exists(clang):
        clang = "/opt/rocm/lib/llvm/bin/clang"
    rt = subprocess.run([clang, "-print-file-name=libclang_rt.asan-x86_64.so"], stdout=subprocess.PIPE, text=True).stdout.strip()
    return lib, rt


if __name__ == "__main__":
    print(build(verbose=True))
    sys.exit(0)

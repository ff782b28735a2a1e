"""Builds libw4a8.so (gfx950 only) next to this file with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libw4a8.so")
SOURCES = ["api.hip", "gemm_decode.hip", "gemm_decode_wide.hip", "gemm_decode_swiglu.hip", "gemm_decode_norm.hip", "gemm_prefill.hip", "gemm_prefill_dma.hip", "gemm_prefill_tiled.hip", "probes.hip",
           "quantize.hip"]
HEADERS = ["common.hpp", "kernels.hpp", "gemm_decode_resident.hpp", os.path.join("..", "..", "include", "w4a8.h"),
           os.path.join("..", "..", "include", "w4a8_tuning.h")]

# -packed-fp32-ops: keep the compiler from forming packed fp32 VALU instructions.
# -ffp-contract=off: no fused multiply-adds are formed from separate fp32 operations, as in the build of the CPU
# oracle; every intermediate the quantisers and epilogues round is then the one their source states.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-ffp-contract=off", "-Xclang", "-target-feature",
         "-Xclang", "-packed-fp32-ops", "-Wno-unused-command-line-argument"]


def source_hash() -> str:
    """Hash of the code of the kernel sources and public headers (comments and white space left out, so that an edit
    of the documentation does not count as another build): ties a profile of hardware counters to the build it was
    taken from (bench.py reports a counter figure only when the hashes agree)."""
    import hashlib
    import re
    h = hashlib.sha256()
    for d in (CSRC, os.path.join(HERE, "..", "include")):
        for name in sorted(os.listdir(d)):
            if name.endswith((".hip", ".hpp", ".h")):
                with open(os.path.join(d, name), "r", encoding="utf-8") as f:
                    text = f.read()
                text = re.sub(r"/\*.*?\*/", " ", text, flags=re.S)   # block comments
                text = re.sub(r"//[^\n]*", " ", text)                 # line comments (no string here holds "//")
                h.update(name.encode())
                h.update(" ".join(text.split()).encode())
    return h.hexdigest()[:16]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def build_library(force: bool = True, verbose: bool = False) -> str:
    """Compile every HIP source for gfx950 and link the shared library."""
    srcs = [os.path.join(CSRC, s) for s in SOURCES]
    deps = srcs + [os.path.join(CSRC, h) for h in HEADERS]
    if not force and os.path.exists(LIB) and all(os.path.getmtime(LIB) >= os.path.getmtime(d) for d in deps):
        return LIB
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    procs = []
    objs = []
    for s in srcs:
        o = os.path.join(objdir, os.path.basename(s) + ".o")
        objs.append(o)
        cmd = [hipcc(), *FLAGS, "-c", s, "-o", o]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for cmd, p in procs:
        out, _ = p.communicate()
        if p.returncode != 0:
            sys.stderr.write(out)
            raise RuntimeError("hipcc failed: " + " ".join(cmd))
    cmd = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    subprocess.run(cmd, check=True)
    return LIB


def build_host_sanitized(verbose: bool = False) -> str:
    """The library with its HOST code under AddressSanitizer and UndefinedBehaviorSanitizer (device code as usual), and
    the C driver tests/abi_selftest.c linked against it.  Returns the driver's path; running it needs no GPU."""
    root = os.path.dirname(HERE)
    objdir = os.path.join(HERE, "_build", "hostsan")
    os.makedirs(objdir, exist_ok=True)
    san = ["-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-Xarch_host",
           "-fno-sanitize-recover=all", "-Xarch_host", "-fno-omit-frame-pointer", "-g"]
    procs, objs = [], []
    for src in SOURCES:
        o = os.path.join(objdir, src + ".o")
        objs.append(o)
        cmd = [hipcc(), *FLAGS, *san, "-c", os.path.join(CSRC, src), "-o", o]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for cmd, p in procs:
        out, _ = p.communicate()
        if p.returncode != 0:
            sys.stderr.write(out)
            raise RuntimeError("hipcc failed: " + " ".join(cmd))
    lib = os.path.join(objdir, "libw4a8_hostsan.so")
    subprocess.run([hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined",
                    "-shared-libsan", "-o", lib, *objs], check=True)
    exe = os.path.join(objdir, "abi_selftest")
    # the sanitizer runtime of hipcc's clang lives outside the loader's default path
    rt = subprocess.run([hipcc(), "-print-file-name=libclang_rt.asan-x86_64.so"], capture_output=True, text=True).stdout.strip()
    rpaths = ["-Wl,-rpath," + objdir] + (["-Wl,-rpath," + os.path.dirname(rt)] if os.path.isabs(rt) else [])
    subprocess.run([hipcc(), "-x", "c", os.path.join(root, "tests", "abi_selftest.c"), "-x", "none", "-fsanitize=address",
                    "-fsanitize=undefined", "-fno-sanitize-recover=all", "-shared-libsan", "-g", "-o", exe, lib, *rpaths],
                   check=True)
    return exe


if __name__ == "__main__":
    if "--host-sanitize" in sys.argv[1:]:
        print(build_host_sanitized(verbose=True))
    else:
        print(build_library(force=True, verbose=True))

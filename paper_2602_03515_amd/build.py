"""Build the C-ABI HIP library for gfx950 with hipcc (in-tree, no JIT cache)."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB_NAME = "libbr_hip.so"
LIB_PATH = os.path.join(HERE, LIB_NAME)
SOURCES = ["br_api.hip", "br_gemm.hip", "br_lowp.hip", "br_elementwise.hip", "br_qr.hip", "br_static.hip"]
ARCH = "gfx950"

HIPCC_FLAGS = [
    "-O3", "-std=c++17", "-fPIC", f"--offload-arch={ARCH}",
    # packed-FP32 instructions stay off for every kernel of this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unused-command-line-argument",
]


def hipcc_path() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found; this library only builds with ROCm's hipcc")


def build_library(verbose: bool = False) -> str:
    """Compile every HIP source and link libbr_hip.so next to this file."""
    hipcc = hipcc_path()
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    procs = []
    objs = []
    for src in SOURCES:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        objs.append(obj)
        cmd = [hipcc, *HIPCC_FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            failed = True
            print(f"[build] {src} FAILED\n{out}", file=sys.stderr)
        elif out.strip() and verbose:
            print(out)
    if failed:
        raise RuntimeError("hipcc failed")
    tmp = LIB_PATH + ".tmp"
    cmd = [hipcc, "-shared", "-fPIC", f"--offload-arch={ARCH}", *objs, "-o", tmp]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        print(res.stdout, file=sys.stderr)
        raise RuntimeError("link failed")
    os.replace(tmp, LIB_PATH)
    # stand-alone executables: the C driver of the ABI (hardware-counter runs; includes br.h only) and the
    # measurement probes (machine peaks, single-kernel timings through the internal launchers)
    for name in ("br_native_bench", "br_probes"):
        exe = os.path.join(HERE, name)
        cmd = [hipcc, *HIPCC_FLAGS, os.path.join(CSRC, name + ".hip"), "-o", exe + ".tmp",
               f"-L{HERE}", "-lbr_hip", "-Wl,-rpath,$ORIGIN"]
        res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        if res.returncode != 0:
            print(res.stdout, file=sys.stderr)
            raise RuntimeError(f"{name} build failed")
        os.replace(exe + ".tmp", exe)
    return LIB_PATH


def build_sanitized(verbose: bool = False) -> str:
    """The C driver and every library source in ONE executable whose HOST code is instrumented with
    AddressSanitizer and UndefinedBehaviorSanitizer (device code is compiled as usual: GPU sanitizers are
    not used).  `br_native_bench_san --host-only` needs no GPU; with one, `--small --steps 6 --freq 2` runs every
    call of the ABI under the sanitizers."""
    hipcc = hipcc_path()
    exe = os.path.join(HERE, "br_native_bench_san")
    flags = [f for f in HIPCC_FLAGS if f != "-O3"] + ["-O1", "-g", "-fno-omit-frame-pointer"]
    for san in ("address", "undefined"):
        flags += ["-Xarch_host", f"-fsanitize={san}"]
    flags += ["-Xarch_host", "-fno-sanitize-recover=undefined"]
    srcs = [os.path.join(CSRC, s) for s in SOURCES + ["br_native_bench.hip"]]
    cmd = [hipcc, *flags, *srcs, "-o", exe + ".tmp"]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        print(res.stdout, file=sys.stderr)
        raise RuntimeError("sanitizer build failed")
    os.replace(exe + ".tmp", exe)
    return exe


if __name__ == "__main__":
    if "--sanitize" in sys.argv:
        print(build_sanitized(verbose="-v" in sys.argv))
    else:
        print(build_library(verbose="-v" in sys.argv))

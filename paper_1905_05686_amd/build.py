"""Builds liblrbi.so (gfx950) in-tree with hipcc.  Run: python -m paper_1905_05686_amd.build"""
from __future__ import annotations

import os
import re
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "liblrbi.so")
SOURCES = ["lrbi_host.cpp", "lrbi_decode.hip", "lrbi_gemv.hip", "lrbi_gemm_mfma.hip", "lrbi_gemm_pipe.hip", "lrbi_gemm_stream.hip", "lrbi_gemm_pipe_t.hip", "lrbi_alg1.hip", "lrbi_backward.hip", "lrbi_lstm.hip", "lrbi_nmf.hip"]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "-std=c++17", "-fPIC", "--offload-arch=gfx950", "-x", "hip",
    # packed fp32 ALU forms are kept out of the generated code on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
    # per-kernel register / private-memory report, checked below
    "-Rpass-analysis=kernel-resource-usage",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def _private_memory_users(remarks: str):
    """Kernels whose compiled code keeps per-lane data in private (scratch) memory.

    Every kernel here is written to live in registers: private memory means that a register
    array was indexed in a way the compiler could not resolve, which turns prefetches into
    synchronous round trips through memory."""
    bad = []
    name = None
    for line in remarks.splitlines():
        m = re.search(r"Function Name: (\S+)", line)
        if m:
            name = m.group(1)
        m = re.search(r"ScratchSize \[bytes/lane\]: (\d+)", line)
        if m and int(m.group(1)) > 0:
            bad.append((name, int(m.group(1))))
    return bad


def _up_to_date(obj: str, src: str) -> bool:
    """True when `obj` is newer than its source and every header it can include."""
    if not os.path.exists(obj):
        return False
    deps = [os.path.join(CSRC, src), os.path.abspath(__file__)]
    deps += [os.path.join(CSRC, f) for f in os.listdir(CSRC) if f.endswith(".hpp")]
    deps += [os.path.join(ROOT, "include", f) for f in os.listdir(os.path.join(ROOT, "include"))]
    return all(os.path.getmtime(d) < os.path.getmtime(obj) for d in deps)


def build(verbose: bool = False, extra_flags=(), incremental: bool = False) -> str:
    """Compiles every source (always, unless `incremental`: then only what changed) and links liblrbi.so."""
    objs = []
    procs = []
    for src in SOURCES:
        obj = os.path.join(CSRC, os.path.splitext(src)[0] + ".o")
        if incremental and not extra_flags and _up_to_date(obj, src):
            objs.append(obj)
            continue
        cmd = [HIPCC] + FLAGS + list(extra_flags) + ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        for name, nbytes in _private_memory_users(out):
            failed = True
            if os.path.exists(os.path.join(CSRC, os.path.splitext(src)[0] + ".o")):
                os.remove(os.path.join(CSRC, os.path.splitext(src)[0] + ".o"))  # not to be linked by a later incremental build
            print("FAILED: %s: kernel %s uses %d bytes of private memory per lane" % (src, name, nbytes),
                  file=sys.stderr)
        out = "\n".join(l for l in out.splitlines()
                        if "packed-fp32-ops" not in l and "-Rpass-analysis" not in l and l.strip()
                        and not re.match(r"\s*(\d+\s*)?\|", l))
        if p.returncode != 0:
            failed = True
            print("FAILED: %s\n%s" % (src, out), file=sys.stderr)
        elif verbose and out:
            print(out)
    if failed:
        raise RuntimeError("hipcc failed")
    tmp = LIB + ".tmp.%d" % os.getpid()
    cmd = [HIPCC, "-shared", "-fPIC", "--offload-arch=gfx950", "-o", tmp] + objs
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, incremental="--incremental" in sys.argv))

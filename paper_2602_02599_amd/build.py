"""Build librap.so in-tree with hipcc for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "librap.so")
SOURCES = ["rap_api.hip", "rap_append.hip", "rap_decode_valu.hip", "rap_decode_mfma.hip", "rap_decode_mfma_q8.hip", "rap_decode_mfma_mx4.hip", "rap_merge.hip", "rap_stream.hip", "rap_prefill.hip",
           "rap_prefill_k1.hip", "rap_prefill_k2.hip", "rap_prefill_k3.hip", "rap_prefill_k4.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def hipcc() -> str:
    for p in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if p and (os.path.isabs(p) and os.path.exists(p) or not os.path.isabs(p)):
            return p
    raise RuntimeError("hipcc not found")


def build(verbose: bool = False, jobs: int = 8) -> str:
    """Compile every source (in parallel) and link the shared library; returns its path."""
    bdir = os.path.join(HERE, "_build")
    os.makedirs(bdir, exist_ok=True)
    cc = hipcc()
    procs = []
    objs = []
    for src in SOURCES:
        obj = os.path.join(bdir, src.replace(".hip", ".o"))
        objs.append(obj)
        cmd = [cc, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((src, cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        while sum(p.poll() is None for _, _, p in procs) >= jobs:
            procs[0][2].wait()
    for src, cmd, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "is not a recognized feature" not in l)
        if p.returncode != 0:
            raise RuntimeError("hipcc failed for %s:\n%s\n%s" % (src, " ".join(cmd), out))
        if verbose and out.strip():
            print(out)
    cmd = [cc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout)
    return LIB


HOST_TEST_SRC = os.path.join(os.path.dirname(HERE), "tests", "host", "rap_arith_host.hip")
HOST_TEST_BIN = os.path.join(HERE, "_build", "rap_arith_host")


def build_host_tests() -> str:
    """Compile the CPU-side harness around csrc/rap_arith.h (host pass of hipcc only, address and
    undefined-behaviour sanitizers on); returns the path of the program.  No GPU is involved."""
    os.makedirs(os.path.dirname(HOST_TEST_BIN), exist_ok=True)
    cmd = [hipcc(), "--offload-host-only", "-O1", "-g", "-std=c++17", "-Xarch_host", "-fsanitize=address",
           "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fno-sanitize-recover=undefined",
           HOST_TEST_SRC, "-o", HOST_TEST_BIN]
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("host test build failed:\n%s\n%s" % (" ".join(cmd), r.stdout))
    return HOST_TEST_BIN


if __name__ == "__main__":
    print(build(verbose=True))

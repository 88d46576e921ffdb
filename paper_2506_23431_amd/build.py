"""Builds libpd.so (the C-ABI library) in-tree with hipcc for gfx950."""

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpd.so")
# (source, extra defines, object name); gemm.hip is compiled once per epilogue (its kernels are many
# template instances) and once for the parts all epilogues share
SOURCES = [("pd_api.hip", [], "pd_api.o"), ("sched.hip", [], "sched.o"), ("simple.hip", [], "simple.o"),
           ("mfma.hip", [], "mfma.o"), ("attn.hip", [], "attn.o"), ("attn_ctx.hip", [], "attn_ctx.o"), ("encdec.hip", [], "encdec.o"), ("gemm.hip", [], "gemm.o")] + \
          [("gemm.hip", [f"-DPD_GEMM_EPI={e}"], f"gemm_epi{e}.o") for e in range(8)]


def hipcc():
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.sep not in cand or os.path.exists(cand)):
            return cand
    raise RuntimeError("hipcc not found")


def build(verbose=True):
    """Compiles every HIP source for gfx950 and links libpd.so.  Always rebuilds."""
    objs = []
    flags = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    build_dir = os.path.join(HERE, "_build")
    os.makedirs(build_dir, exist_ok=True)
    procs = []
    for src, defines, oname in SOURCES:
        obj = os.path.join(build_dir, oname)
        cmd = [hipcc()] + flags + defines + ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((oname, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)))
        objs.append(obj)
    failed = False
    for src, p in procs:
        out = p.communicate()[0].decode()
        lines = [l for l in out.splitlines() if "packed-fp32-ops" not in l]
        if p.returncode != 0 or (verbose and lines):
            sys.stdout.write("\n".join(lines) + "\n")
        failed = failed or p.returncode != 0
    if failed:
        raise RuntimeError("hipcc failed")
    cmd = [hipcc(), "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    print(build())

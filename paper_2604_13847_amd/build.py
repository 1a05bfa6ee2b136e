"""Compile the HIP sources into paper_2604_13847_amd/libsparsebal.so for gfx950."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsparsebal.so")
SOURCES = ["sb_host.hip", "sb_scores.hip", "sb_topk.hip", "sb_plan.hip", "sb_attn_fwd.hip", "sb_attn_bwd.hip", "sb_coverage.hip", "sb_sab.hip"]
FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-variable", "-Wno-inline-asm", "-Wno-pass-failed", "-I" + os.path.join(ROOT, "include"), "-I" + CSRC]


def build_lib(verbose: bool = False, extra=()) -> str:
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    procs = []
    objs = []
    for src in SOURCES:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        objs.append(obj)
        cmd = ["hipcc", *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for src, pr in procs:
        out, _ = pr.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l and "is not a recognized feature" not in l)
        if pr.returncode != 0:
            failed = True
            print(f"--- {src} failed\n{out}", file=sys.stderr)
        elif verbose and out.strip():
            print(f"--- {src}\n{out}")
    if failed:
        raise RuntimeError("hipcc failed")
    tmp = LIB + f".{os.getpid()}.tmp"
    subprocess.check_call(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", tmp, *objs])
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build_lib(verbose=True, extra=sys.argv[1:]))

"""Build libcodistill.so (gfx950) in-tree with hipcc."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libcodistill.so")
SOURCES = ["runtime.hip", "loss.hip", "sgd.hip", "kernels_simple.hip", "norm.hip", "layernorm.hip", "attention.hip", "conv_grouped.hip", "conv_mfma.hip", "model.hip"]
FLAGS = ["-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-fno-gpu-rdc",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-function", "-Wno-unknown-warning-option",
         "-I", os.path.join(ROOT, "include"), "-I", CSRC]


def build(verbose=True, jobs=8):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    procs = []
    objs = []
    for src in SOURCES:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        objs.append(obj)
        cmd = [hipcc] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT)))
        while sum(p.poll() is None for _, p in procs) >= jobs:
            procs[0][1].wait()
    failed = False
    for src, p in procs:
        out = p.communicate()[0].decode()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l and l.strip())
        if p.returncode != 0:
            failed = True
            sys.stderr.write("FAILED %s\n%s\n" % (src, out))
        elif verbose and out:
            sys.stderr.write("%s:\n%s\n" % (src, out))
    if failed:
        raise RuntimeError("hipcc failed")
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB] + objs)
    return LIB


def build_layer_bench():
    """The per-layer convolution timing program (bench_src/conv_layer_bench.hip), linked against libcodistill.so."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    exe = os.path.join(HERE, "conv_layer_bench")
    subprocess.check_call([hipcc, "-O2", "-std=c++17", "--offload-arch=gfx950", "-w", "-I", os.path.join(ROOT, "include"),
                           "-I", CSRC, "-o", exe, os.path.join(HERE, "bench_src", "conv_layer_bench.hip"), "-L", HERE,
                           "-lcodistill", "-Wl,-rpath,$ORIGIN"])
    return exe


if __name__ == "__main__":
    print(build())
    if "--layer-bench" in sys.argv:
        print(build_layer_bench())

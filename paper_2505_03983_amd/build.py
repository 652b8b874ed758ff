"""Builds libasd.so (the sampling library) and libasd_probe.so (a measurement probe for bench.py) in-tree
with hipcc for gfx950.  Run: python -m paper_2505_03983_amd.build"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libasd.so")
PROBE_LIB = os.path.join(HERE, "libasd_probe.so")
SOURCES = ["api.hip", "round.hip", "gmm.hip", "gmm_chain.hip", "mlp.hip"]
PROBE_SOURCES = ["probe/ceiling.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fvisibility=hidden",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def build(verbose=True, defines=(), lib=LIB, tag=""):
    _build_one(SOURCES, lib, verbose, defines, tag)
    _build_one(PROBE_SOURCES, PROBE_LIB, verbose, (), tag)
    return lib


def _build_one(sources, lib, verbose, defines, tag):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    procs = []
    for src in sources:
        obj = os.path.join(CSRC, src.replace(".hip", tag + ".o"))
        cmd = [hipcc] + [f for f in FLAGS if f != "-shared"] + ["-D" + d for d in defines] + ["-c", os.path.join(CSRC, src), "-o", obj]
        procs.append((src, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
        objs.append(obj)
    for src, p in procs:
        out, _ = p.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if p.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (src, out))
        if verbose and out.strip():
            print(out)
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib] + objs
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stdout)
    if verbose:
        print("built", lib)
    return lib


if __name__ == "__main__":
    build()
    sys.exit(0)

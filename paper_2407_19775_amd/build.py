"""Build libmmd8.so (HIP, gfx950) in-tree with hipcc.  `python -m paper_2407_19775_amd.build`."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmmd8.so")
SOURCES = ["api.hip", "codec_kernels.hip", "activation_kernels.hip", "weight_kernels.hip", "gemm_kernels.hip",
           "skinny_kernels.hip", "lora_kernels.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++20", "-fPIC", "-ffp-contract=off",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


def hipcc() -> str:
    for cand in (os.environ.get("HIPCC"), "/opt/rocm/bin/hipcc", "hipcc"):
        if cand and (os.path.isabs(cand) and os.path.exists(cand) or not os.path.isabs(cand)):
            return cand
    return "hipcc"


def _run(cmd):
    proc = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in proc.stderr.splitlines() if noise not in l)
    if proc.returncode != 0:
        raise RuntimeError("command failed: %s\n%s\n%s" % (" ".join(cmd), proc.stdout, err))
    return err


def build(verbose: bool = False) -> str:
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    cc = hipcc()

    def compile_one(src):
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        err = _run([cc, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj])
        if verbose and err.strip():
            print(err, file=sys.stderr)
        return obj

    with ThreadPoolExecutor(max_workers=min(8, len(SOURCES))) as pool:
        objs = list(pool.map(compile_one, SOURCES))
    _run([cc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs])
    # the graph partitioner: plain host C++, a library of its own (include/mtpp.h)
    _run(["g++", "-O2", "-std=c++17", "-shared", "-fPIC", "-o", os.path.join(HERE, "libmtpp.so"),
          os.path.join(CSRC, "mtpp.cpp")])
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))

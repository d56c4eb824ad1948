"""Builds libpeqa_hip.so (the C-ABI library) in-tree with hipcc for gfx950."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpeqa_hip.so")
SOURCES = ["peqa_api.hip", "peqa_quantize.hip", "peqa_small.hip", "peqa_gemm.hip", "peqa_gemv.hip", "peqa_dw.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument", "-Rpass-analysis=kernel-resource-usage"]
# Kernels that queue global -> LDS DMA from inline assembly and count s_waitcnt vmcnt by hand: a
# register spill would add scratch loads and stores (also counted by vmcnt) that the hand count does
# not know about, so the build refuses any scratch use in them.
NO_SCRATCH = ("gemm_kernel", "gemm_bwd_pair_kernel", "gemv_kernel", "dw_kernel")


def check_no_scratch(remarks):
    name = None
    bad = []
    for line in remarks.splitlines():
        if "Function Name:" in line:
            name = line.split("Function Name:")[1].split("[")[0].strip()
        elif "ScratchSize [bytes/lane]:" in line and name is not None:
            size = int(line.split("ScratchSize [bytes/lane]:")[1].split("[")[0])
            if size > 0 and any(k in name for k in NO_SCRATCH):
                bad.append("%s uses %d bytes of scratch per lane" % (name, size))
    return bad


def build(verbose=False, extra=()):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + list(extra) + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l and "remark:" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    bad = check_no_scratch(r.stdout)
    if bad:
        os.remove(LIB)
        raise RuntimeError("register spills in kernels that count vmcnt by hand:\n" + "\n".join(bad))
    if verbose and out.strip():
        print(out)
    return LIB


if __name__ == "__main__":
    build(verbose=True, extra=sys.argv[1:])

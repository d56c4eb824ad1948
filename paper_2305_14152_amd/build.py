"""Builds libpeqa_hip.so (the C-ABI library) in-tree with hipcc for gfx950."""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libpeqa_hip.so")
SOURCES = ["peqa_api.hip", "peqa_quantize.hip", "peqa_small.hip", "peqa_gemm.hip", "peqa_gemv.hip", "peqa_dw.hip",
           "peqa_block.hip"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wno-unused-command-line-argument", "-Rpass-analysis=kernel-resource-usage"]
# Kernels that queue global -> LDS DMA from inline assembly and count s_waitcnt vmcnt by hand: a
# register spill would add scratch loads and stores (also counted by vmcnt) that the hand count does
# not know about, so the build refuses any scratch use in them.
NO_SCRATCH = ("gemm_kernel", "gemm_bwd_pair_kernel", "gemm_multi_kernel", "gemv_kernel", "dw_kernel")


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


def _quiet(text):
    return "\n".join(l for l in text.splitlines() if "packed-fp32-ops" not in l and "remark:" not in l)


def build(verbose=False, extra=(), jobs=None):
    """Every source is compiled (always: no time stamps are consulted) to an object of its own, in
    parallel, then the objects are linked into the shared library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    if os.path.exists(LIB):
        os.remove(LIB)

    def compile_one(src):
        obj = os.path.join(OBJ, src.replace(".hip", ".o"))
        cmd = [hipcc] + FLAGS + list(extra) + ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        return src, obj, r

    jobs = jobs or min(len(SOURCES), int(os.environ.get("MAX_JOBS", "8")), os.cpu_count() or 1)
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        results = list(pool.map(compile_one, SOURCES))
    remarks = ""
    for src, _, r in results:
        if r.returncode != 0:
            raise RuntimeError("hipcc failed on %s:\n%s" % (src, _quiet(r.stdout)))
        remarks += r.stdout
    with open(os.path.join(OBJ, "remarks.txt"), "w") as f:     # registers, LDS and occupancy of every kernel
        f.write(remarks)
    bad = check_no_scratch(remarks)
    if bad:
        raise RuntimeError("register spills in kernels that count vmcnt by hand:\n" + "\n".join(bad))
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + [obj for _, obj, _ in results] + ["-o", LIB]
    if verbose:
        print(" ".join(link), flush=True)
    r = subprocess.run(link, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + _quiet(r.stdout))
    out = _quiet(remarks)
    if verbose and out.strip():
        print(out)
    return LIB


if __name__ == "__main__":
    build(verbose=True, extra=sys.argv[1:])

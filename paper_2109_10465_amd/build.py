"""Builds the HIP library (libmoe_hip.so) for gfx950 with hipcc, in-tree.

    python -m paper_2109_10465_amd.build
"""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libmoe_hip.so")
SOURCES = ["api.hip", "route.hip", "gate.hip", "aux_loss.hip", "permute.hip", "expert_gemm.hip", "microbench.hip"]
FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         # packed-fp32 VALU forms are kept out of generated code on purpose
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


# Kernels whose loads are issued by hand (inline asm, completion awaited by hand): a register that is
# spilled while its load is still in flight would be saved before the data lands, so these kernels must
# not use scratch memory at all.  Checked from the compiler's resource-usage remarks on every build.
NO_SCRATCH = {"gate.hip": ["gate_logits_lds_kernel"]}


def check_no_scratch(src, remarks):
    name = None
    for line in remarks.splitlines():
        if "Function Name:" in line:
            name = line.split("Function Name:")[1].split()[0]
        elif "ScratchSize [bytes/lane]:" in line and name and any(k in name for k in NO_SCRATCH[src]):
            if int(line.split("ScratchSize [bytes/lane]:")[1].split()[0]) != 0:
                raise RuntimeError(f"{src}: {name} uses scratch memory; its hand-issued loads do not allow that")


def build(verbose=True):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    procs = []
    os.makedirs(os.path.join(HERE, "_build"), exist_ok=True)
    for src in SOURCES:
        obj = os.path.join(HERE, "_build", src.replace(".hip", ".o"))
        extra = ["-Rpass-analysis=kernel-resource-usage", "-fno-caret-diagnostics"] if src in NO_SCRATCH else []
        cmd = [hipcc, *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, stderr=subprocess.PIPE, text=True)))
        objs.append(obj)
    failed = False
    for src, p in procs:
        _, err = p.communicate()
        if src in NO_SCRATCH and p.returncode == 0:
            check_no_scratch(src, err)
        err = "\n".join(l for l in err.splitlines() if "packed-fp32-ops" not in l and "-Rpass-analysis" not in l and " remark: " not in l)
        if err.strip() and verbose:
            print(err, file=sys.stderr)
        failed |= p.returncode != 0
    if failed:
        raise RuntimeError("hipcc failed")
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    build()

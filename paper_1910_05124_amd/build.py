"""Builds libpipemare.so (HIP, gfx950) in-tree with hipcc.  `python paper_1910_05124_amd/build.py`."""
import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libpipemare.so")
OBJ = os.path.join(PKG, "_build")

FLAGS = ["-std=c++17", "-O3", "--offload-arch=gfx950", "-fPIC",
         # keep the compiler from forming packed-fp32 instructions
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]
# translation units and their extra flags.  The attention kernels keep the accumulators of the matrix
# instructions in ordinary vector registers (no copies between the two register files around the
# softmax arithmetic); the GEMMs with 256 accumulator registers per lane need the second file.
UNITS = [("pipemare.hip", []),
         ("pm_attn.hip", ["-mllvm", "-amdgpu-mfma-vgpr-form=1"])]


def build(verbose: bool = True) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)

    def finish(cmd, r_out, rc):
        out = "\n".join(l for l in r_out.splitlines() if "not a recognized feature" not in l)
        if rc != 0:
            raise RuntimeError("hipcc failed (" + " ".join(cmd[-3:]) + "):\n" + out)
        if verbose and out.strip():
            print(out)

    # the translation units compile side by side
    objs, procs = [], []
    for src, extra in UNITS:
        obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
        objs.append(obj)
        cmd = [hipcc] + FLAGS + extra + ["-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for cmd, pr in procs:
        out, _ = pr.communicate()
        finish(cmd, out, pr.returncode)
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB + ".tmp"]
    if verbose:
        print(" ".join(link), flush=True)
    r = subprocess.run(link, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    finish(link, r.stdout, r.returncode)
    os.replace(LIB + ".tmp", LIB)
    return LIB


if __name__ == "__main__":
    build()
    sys.exit(0)

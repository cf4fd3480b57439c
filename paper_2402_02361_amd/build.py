"""Build the HIP library for gfx950 in-tree (paper_2402_02361_amd/libpruner_hip.so)."""
import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpruner_hip.so")
SOURCES = ("common.hip", "draft_score.hip", "topk.hip", "verify_mlp.hip", "prior_filter.hip", "lse.hip", "random_init.hip", "moa.hip", "pacm.hip")

# -packed-fp32-ops off: no v_pk_*_f32.  Contraction off and correctly rounded division: the draft model's
# binary32 sequence is one IEEE operation per step.  MFMA accumulators in ordinary vector registers (the weights
# of the verify kernel fill the accumulation registers): the epilogues then read them without register copies.
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fno-gpu-rdc",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-ffp-contract=off", "-fhip-fp32-correctly-rounded-divide-sqrt",
    "-mllvm", "-amdgpu-mfma-vgpr-form",
    "-Wall", "-Wno-unused-function",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def build(verbose=False, keep_temps=False):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(HERE, "_build")
    os.makedirs(objdir, exist_ok=True)
    procs = []
    objs = []
    for src in SOURCES:
        obj = os.path.join(objdir, src.replace(".hip", ".o"))
        objs.append(obj)
        cmd = [hipcc, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
        if keep_temps:
            cmd += ["-save-temps=obj"]
        if verbose:
            print(" ".join(cmd), flush=True)
        procs.append((src, subprocess.Popen(cmd, cwd=objdir, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    failed = False
    for src, p in procs:
        out, _ = p.communicate()
        # the host pass does not know the packed-fp32 feature and says so: harmless
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if out.strip() and (verbose or p.returncode):
            print(out)
        if p.returncode:
            print(f"hipcc failed on {src}", file=sys.stderr)
            failed = True
    if failed:
        raise RuntimeError("HIP build failed")
    tmp = LIB + f".tmp{os.getpid()}"
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fno-gpu-rdc", "-o", tmp, *objs])
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-v" in sys.argv, keep_temps="--keep" in sys.argv))

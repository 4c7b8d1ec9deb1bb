"""Build the HIP library (csrc/ -> liblpg.so, in-tree) for gfx950 with hipcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "liblpg.so")
OBJ = os.path.join(HERE, "_build")
COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
          "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-Wall", "-Wno-unused-function", "-Wno-inline-asm"]
# source -> extra flags.  MFMA accumulators are pinned to VGPRs: with the default the compiler
# parks VGPR spills in AGPRs for the 4-wave 256 x 128 tiles and halves their occupancy.
VGPR_FORM = ["-mllvm", "-amdgpu-mfma-vgpr-form=1"]
SOURCES = {"lpg_api.cpp": [], "lpg_kernels.hip": VGPR_FORM, "lpg_gemm_f32.hip": VGPR_FORM,
           "lpg_gemm_bf16.hip": VGPR_FORM, "lpg_gemm_bf16_f32.hip": VGPR_FORM}


def _run(cmd, verbose):
    if verbose:
        print(" ".join(cmd))
    r = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in r.stdout.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + out)
    if verbose and out.strip():
        print(out)


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ, exist_ok=True)
    objs = []
    procs = []
    for src, extra in SOURCES.items():
        obj = os.path.join(OBJ, src + ".o")
        objs.append(obj)
        cmd = [hipcc] + COMMON + extra + ["-x", "hip", "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd))
        procs.append((cmd, subprocess.Popen(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)))
    for cmd, pr in procs:
        out, _ = pr.communicate()
        out = "\n".join(l for l in out.splitlines() if "packed-fp32-ops" not in l)
        if pr.returncode != 0:
            raise RuntimeError("hipcc failed: " + " ".join(cmd) + "\n" + out)
        if verbose and out.strip():
            print(out)
    _run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"] + objs + ["-o", LIB], verbose)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))

"""Build the HIP library in-tree for gfx950 with hipcc (cross-compiles without a GPU)."""
import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB_PATH = os.path.join(HERE, "libkan_hip.so")

# packed fp32 instructions are switched off for every translation unit
HIPCC_FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-shared",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               # matrix-core accumulators in ordinary VGPRs: the walk kernel reads and clears single
               # accumulator rows between MFMAs, which through AGPRs costs a copy of all of them per record
               "-mllvm", "-amdgpu-mfma-vgpr-form=1",
               "-Wno-unused-command-line-argument"]


def sources():
    return sorted(glob.glob(os.path.join(HERE, "csrc", "*.hip")))


def build(verbose=False):
    """Compile csrc/*.hip into libkan_hip.so next to this file.  Always recompiles."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + ["-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc")]
    cmd += sources() + ["-L/opt/rocm/lib", "-lrocblas", "-Wl,-rpath,/opt/rocm/lib", "-o", LIB_PATH]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    out = "\n".join(l for l in res.stdout.splitlines()
                    if "packed-fp32-ops' is not a recognized feature" not in l)
    if verbose or res.returncode != 0:
        print(out)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed (%d)" % res.returncode)
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))

"""Build the HIP library in-tree for gfx950 with hipcc (cross-compiles without a GPU)."""
import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB_PATH = os.path.join(HERE, "libkan_hip.so")            # the layer library (HIP runtime only)
BENCH_LIB_PATH = os.path.join(HERE, "libkan_bench.so")    # benchmark companion: event timing, rocBLAS dense baseline

# packed fp32 instructions are switched off for every translation unit
HIPCC_FLAGS = ["-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC", "-shared",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               # matrix-core accumulators in ordinary VGPRs: the walk kernel reads and clears single
               # accumulator rows between MFMAs, which through AGPRs costs a copy of all of them per record
               "-mllvm", "-amdgpu-mfma-vgpr-form=1",
               "-Wno-unused-command-line-argument"]


def sources():
    return sorted(glob.glob(os.path.join(HERE, "csrc", "*.hip")))


def bench_sources():
    return sorted(glob.glob(os.path.join(HERE, "csrc_bench", "*.hip")))


def build(verbose=False, jobs=None):
    """Compile csrc/*.hip into libkan_hip.so and csrc_bench/*.hip into libkan_bench.so next to this file.
    Always recompiles.

    Every source is compiled to an object file in its own hipcc process (a few at a time), then each
    library is linked from its own objects; only the benchmark library links rocBLAS."""
    import concurrent.futures
    import tempfile
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in HIPCC_FLAGS if f != "-shared"]
    inc = ["-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc")]
    jobs = jobs or min(8, os.cpu_count() or 1)
    log = []

    def run(cmd):
        res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        out = "\n".join(l for l in res.stdout.splitlines()
                        if "packed-fp32-ops' is not a recognized feature" not in l)
        return res.returncode, out

    with tempfile.TemporaryDirectory(prefix="kan_build_") as tmp:
        objs = [os.path.join(tmp, os.path.basename(src) + ".o") for src in sources()]
        bench_objs = [os.path.join(tmp, os.path.basename(src) + ".o") for src in bench_sources()]
        with concurrent.futures.ThreadPoolExecutor(max_workers=jobs) as pool:
            results = list(pool.map(lambda so: run([hipcc] + flags + inc + ["-c", so[0], "-o", so[1]]),
                                    zip(sources() + bench_sources(), objs + bench_objs)))
        failed = [out for rc, out in results if rc != 0]
        log += [out for rc, out in results if out]
        link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC"]
        for these, libs, path in ((objs, [], LIB_PATH),
                                  (bench_objs, ["-L/opt/rocm/lib", "-lrocblas", "-Wl,-rpath,/opt/rocm/lib"],
                                   BENCH_LIB_PATH)):
            if failed:
                break
            rc, out = run(link + these + libs + ["-o", path])
            if out:
                log.append(out)
            if rc != 0:
                failed.append(out)
    if verbose or failed:
        print("\n".join(log))
    if failed:
        raise RuntimeError("hipcc failed")
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))

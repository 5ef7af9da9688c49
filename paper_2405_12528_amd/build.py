"""Compile the HIP sources under csrc/ into paper_2405_12528_amd/libsirllm.so for gfx950 (and the
plain-C example that calls it).  Every translation unit is compiled on its own (in parallel) into
_build/ and the objects are linked; `python -m paper_2405_12528_amd.build --incremental` skips the
units whose object is newer than every source and header."""
import glob
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libsirllm.so")
OBJ_DIR = os.path.join(ROOT, "_build", "libsirllm")
ARCH = "gfx950"

FLAGS = [
    f"--offload-arch={ARCH}", "-O3", "-std=c++17", "-fPIC",
    "-fno-gpu-flush-denormals-to-zero",            # binary32 denormals survive the decay multiply
    "-ffp-contract=on",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def sources():
    return sorted(glob.glob(os.path.join(HERE, "csrc", "*.hip")))


def headers():
    return sorted(glob.glob(os.path.join(HERE, "csrc", "*.h"))) + sorted(glob.glob(os.path.join(ROOT, "include", "*.h")))


def build(verbose: bool = False, incremental: bool = False, jobs: int | None = None) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    os.makedirs(OBJ_DIR, exist_ok=True)
    inc = ["-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc")]
    newest_header = max(os.path.getmtime(h) for h in headers())
    jobs = jobs or min(8, os.cpu_count() or 1)

    def compile_one(src):
        obj = os.path.join(OBJ_DIR, os.path.basename(src)[:-4] + ".o")
        if incremental and os.path.exists(obj) and os.path.getmtime(obj) >= max(os.path.getmtime(src), newest_header):
            return obj
        cmd = [hipcc] + FLAGS + inc + ["-c", src, "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        r = subprocess.run(cmd, capture_output=True, text=True)
        noise = "is not a recognized feature for this target"       # the host pass does not know the GPU feature
        err = "\n".join(l for l in r.stderr.splitlines() if noise not in l)
        if err.strip():
            print(err, file=sys.stderr, flush=True)
        if r.returncode != 0:
            raise subprocess.CalledProcessError(r.returncode, cmd)
        return obj

    with ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(compile_one, sources()))
    cmd = [hipcc, f"--offload-arch={ARCH}", "-shared", "-fPIC"] + objs + ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


MEMBENCH_LIB = os.path.join(HERE, "libmembench.so")


def build_membench() -> str:
    """Compile membench/membench.hip (streaming read / write / copy reference kernels for bench.py)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, f"--offload-arch={ARCH}", "-O3", "-std=c++17", "-fPIC", "-shared", "-Xclang", "-target-feature",
           "-Xclang", "-packed-fp32-ops", os.path.join(HERE, "membench", "membench.hip"), "-o", MEMBENCH_LIB]
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "is not a recognized feature for this target" not in l)
    if err.strip():
        print(err, file=sys.stderr, flush=True)
    if r.returncode != 0:
        raise subprocess.CalledProcessError(r.returncode, cmd)
    return MEMBENCH_LIB


def build_example() -> str:
    """Compile examples/step_example.c (plain C, HIP runtime + libsirllm only) next to its source."""
    src = os.path.join(ROOT, "examples", "step_example.c")
    exe = os.path.join(ROOT, "examples", "step_example")
    rocm = os.environ.get("ROCM_PATH", "/opt/rocm")
    cmd = ["gcc", "-std=c11", "-O2", src, "-I", os.path.join(ROOT, "include"), "-I", os.path.join(rocm, "include"),
           "-L", HERE, "-L", os.path.join(rocm, "lib"), "-lsirllm", "-lamdhip64", "-lm",
           "-Wl,-rpath,$ORIGIN/../paper_2405_12528_amd", "-Wl,-rpath," + os.path.join(rocm, "lib"), "-o", exe]
    subprocess.run(cmd, check=True)
    return exe


if __name__ == "__main__":
    print(build(verbose=True, incremental="--incremental" in sys.argv))
    print(build_membench())
    print(build_example())

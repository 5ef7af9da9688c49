"""Compile the HIP sources under csrc/ into paper_2405_12528_amd/libsirllm.so for gfx950 (and the
plain-C example that calls it)."""
import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libsirllm.so")
ARCH = "gfx950"

FLAGS = [
    f"--offload-arch={ARCH}", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-fno-gpu-flush-denormals-to-zero",            # binary32 denormals survive the decay multiply
    "-ffp-contract=on",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def sources():
    return sorted(glob.glob(os.path.join(HERE, "csrc", "*.hip")))


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + FLAGS + ["-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc")] + \
        sources() + ["-o", LIB]
    if verbose:
        print(" ".join(cmd))
    subprocess.run(cmd, check=True)
    return LIB


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
    print(build(verbose=True))
    print(build_example())

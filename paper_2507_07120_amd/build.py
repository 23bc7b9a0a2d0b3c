"""Builds the HIP library (gfx950) in-tree: paper_2507_07120_amd/libhelix_attn.so."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "helix_attn.hip")
LIB = os.path.join(HERE, "libhelix_attn.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # keep the compiler from forming packed-fp32 VALU ops out of scalar float code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # no implicit fused multiply-add: the softmax weights are split into bf16 hi + lo, and an ulp-level
    # change of a weight near a rounding boundary of the lo part moves the result by 2^-17; with
    # contraction the compiler fuses differently in different code paths (full tile / ragged tile),
    # which would make the same token's weight depend on where a shard boundary falls
    "-ffp-contract=off",
    "-Wall", "-Wno-unused-command-line-argument",
]


def _torch_lib_dir() -> str:
    import torch
    return os.path.join(os.path.dirname(torch.__file__), "lib")


def build(verbose: bool = False) -> str:
    """Compiles csrc/helix_attn.hip for gfx950.

    The library is linked against the HIP runtime that PyTorch ships (torch/lib/libamdhip64.so), not
    the one under /opt/rocm: callers hand over torch's device pointers and stream handles, and a
    second copy of the runtime in the process would neither know those streams nor be covered by
    torch.cuda.synchronize().
    """
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tl = _torch_lib_dir()
    cmd = [hipcc] + HIPCC_FLAGS + ["-no-hip-rt", "-o", LIB, SRC, "-L" + tl, "-lamdhip64", "-Wl,-rpath," + tl]
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(line for line in res.stderr.splitlines() if noise not in line)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if err.strip():
        print(err)
    return LIB


if __name__ == "__main__":
    print(build())

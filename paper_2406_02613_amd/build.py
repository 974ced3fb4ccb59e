"""Build libacco.so (HIP kernels + C ABI) in-tree for gfx950."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
ACCO_SO = os.path.join(HERE, "libacco.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# -ffp-contract=off: the kernels spell out their fused multiply-adds; nothing else is fused.
# packed-fp32-ops is switched off: the packed FP32 instructions are not to be generated.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off",
         "-fvisibility=hidden", "-Wall", "-Wextra",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build_acco(extra=()) -> str:
    cmd = [HIPCC, *FLAGS, *extra, os.path.join(CSRC, "acco_api.hip"), "-o", ACCO_SO]
    subprocess.run(cmd, check=True, cwd=HERE)
    return ACCO_SO


if __name__ == "__main__":
    print(build_acco())

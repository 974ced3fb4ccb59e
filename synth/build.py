"""Build the generator's two shared libraries in-tree (host: gcc, device: hipcc gfx950)."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
HOST_SO = os.path.join(HERE, "libsynth_host.so")
DEVICE_SO = os.path.join(HERE, "libsynth_device.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def build_host() -> str:
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
           "-fvisibility=hidden", "-Wall", "-Wextra",
           os.path.join(HERE, "synth_host.c"), "-o", HOST_SO]
    subprocess.run(cmd, check=True, cwd=HERE)
    return HOST_SO


def build_device() -> str:
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-fPIC", "-shared", "-ffp-contract=off",
           "-fvisibility=hidden", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           os.path.join(HERE, "synth_device.hip"), "-o", DEVICE_SO]
    subprocess.run(cmd, check=True, cwd=HERE)
    return DEVICE_SO


def build_all() -> None:
    build_host()
    build_device()


if __name__ == "__main__":
    build_all()
    print(HOST_SO)
    print(DEVICE_SO)

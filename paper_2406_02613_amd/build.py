"""Build libacco.so (HIP kernels + C ABI) in-tree for gfx950."""
import hashlib
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
ACCO_SO = os.path.join(HERE, "libacco.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
SOURCES = [os.path.join(CSRC, "acco_api.hip"), os.path.join(CSRC, "kernels.hpp"),
           os.path.join(os.path.dirname(HERE), "include", "acco.h")]

# -ffp-contract=off: the kernels spell out their fused multiply-adds; nothing else is fused.
# packed-fp32-ops is switched off: the packed FP32 instructions are not to be generated.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off",
         "-fvisibility=hidden", "-Wall", "-Wextra",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def source_hash(extra=()) -> str:
    h = hashlib.sha256(" ".join([*FLAGS, *extra]).encode())
    for path in SOURCES:
        h.update(open(path, "rb").read())
    return h.hexdigest()


def is_current() -> bool:
    """Was libacco.so built from the sources and flags as they are now?"""
    try:
        return os.path.exists(ACCO_SO) and open(ACCO_SO + ".srchash").read() == source_hash()
    except OSError:
        return False


def build_acco(extra=()) -> str:
    cmd = [HIPCC, *FLAGS, *extra, SOURCES[0], "-o", ACCO_SO]
    subprocess.run(cmd, check=True, cwd=HERE)
    open(ACCO_SO + ".srchash", "w").write(source_hash(extra))
    return ACCO_SO


if __name__ == "__main__":
    print(build_acco())

"""Build libacco.so (HIP kernels + C ABI) in-tree for gfx950."""
import hashlib
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
ACCO_SO = os.path.join(HERE, "libacco.so")
# the same source with its HOST half under AddressSanitizer + UndefinedBehaviorSanitizer (the
# device code is built as usual): for the tests of the host logic - validation, counters,
# folded scalars, launch settings
ACCO_HOST_SAN_SO = os.path.join(HERE, "libacco_hostsan.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
SOURCES = [os.path.join(CSRC, "acco_api.hip"), os.path.join(CSRC, "kernels.hpp"),
           os.path.join(os.path.dirname(HERE), "include", "acco.h")]

# -ffp-contract=off: the kernels spell out their fused multiply-adds; nothing else is fused.
# packed-fp32-ops is switched off: the packed FP32 instructions are not to be generated.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-ffp-contract=off",
         "-fvisibility=hidden", "-Wall", "-Wextra",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


HOST_SAN_FLAGS = [f if f != "-O3" else "-O1" for f in FLAGS] + [
    "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
    "-Xarch_host", "-fno-sanitize-recover=undefined", "-Xarch_host", "-fno-omit-frame-pointer",
    "-shared-libsan"]


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


def selected_so() -> str:
    """The library the binding loads: the host-sanitized build when ACCO_SANITIZE_HOST=1 (the
    process must then run with clang's sanitizer runtime preloaded, see sanitizer_runtime)."""
    return ACCO_HOST_SAN_SO if os.environ.get("ACCO_SANITIZE_HOST") == "1" else ACCO_SO


def sanitizer_runtime():
    """Path of the shared AddressSanitizer runtime of the compiler hipcc drives, or None."""
    out = subprocess.run([HIPCC, "-print-file-name=libclang_rt.asan-x86_64.so"],
                         capture_output=True, text=True).stdout.strip()
    if os.path.isabs(out) and os.path.exists(out):
        return out
    res = subprocess.run([HIPCC, "-print-resource-dir"], capture_output=True, text=True).stdout.strip()
    cand = os.path.join(res, "lib", "linux", "libclang_rt.asan-x86_64.so")
    return cand if os.path.exists(cand) else None


def ensure_host_sanitized() -> str:
    """libacco_hostsan.so, rebuilt if its sources or flags changed."""
    def digest():
        h = hashlib.sha256(" ".join(HOST_SAN_FLAGS).encode())
        for path in SOURCES:
            h.update(open(path, "rb").read())
        return h.hexdigest()
    tag = ACCO_HOST_SAN_SO + ".srchash"
    try:
        if os.path.exists(ACCO_HOST_SAN_SO) and open(tag).read() == digest():
            return ACCO_HOST_SAN_SO
    except OSError:
        pass
    subprocess.run([HIPCC, *HOST_SAN_FLAGS, SOURCES[0], "-o", ACCO_HOST_SAN_SO], check=True, cwd=HERE)
    open(tag, "w").write(digest())
    return ACCO_HOST_SAN_SO


if __name__ == "__main__":
    print(build_acco())

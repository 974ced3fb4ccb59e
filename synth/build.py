"""Build the generator's two shared libraries in-tree (host: gcc, device: hipcc gfx950)."""
import hashlib
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
HOST_SO = os.path.join(HERE, "libsynth_host.so")
HOST_SAN_SO = os.path.join(HERE, "libsynth_host_san.so")   # AddressSanitizer + UBSan build
DEVICE_SO = os.path.join(HERE, "libsynth_device.so")
CORE = os.path.join(HERE, "synth_core.h")
HOST_SRC = [os.path.join(HERE, "synth_host.c"), CORE]
DEVICE_SRC = [os.path.join(HERE, "synth_device.hip"), CORE]

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

HOST_FLAGS = ["-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
              "-fvisibility=hidden", "-Wall", "-Wextra"]
HOST_SAN_FLAGS = ["-O1", "-g", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
                  "-fvisibility=hidden", "-Wall", "-Wextra", "-fsanitize=address,undefined",
                  "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"]
DEVICE_FLAGS = ["--offload-arch=gfx950", "-O3", "-fPIC", "-shared", "-ffp-contract=off",
                "-fvisibility=hidden", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def source_hash(sources, flags) -> str:
    h = hashlib.sha256(" ".join(flags).encode())
    for path in sources:
        h.update(open(path, "rb").read())
    return h.hexdigest()


def is_current(so, sources, flags) -> bool:
    try:
        return os.path.exists(so) and open(so + ".srchash").read() == source_hash(sources, flags)
    except OSError:
        return False


def _build(compiler, so, sources, flags) -> str:
    subprocess.run([compiler, *flags, sources[0], "-o", so], check=True, cwd=HERE)
    open(so + ".srchash", "w").write(source_hash(sources, flags))
    return so


def build_host() -> str:
    return _build("gcc", HOST_SO, HOST_SRC, HOST_FLAGS)


def build_host_sanitized() -> str:
    return _build("gcc", HOST_SAN_SO, HOST_SRC, HOST_SAN_FLAGS)


def build_device() -> str:
    return _build(HIPCC, DEVICE_SO, DEVICE_SRC, DEVICE_FLAGS)


def host_current() -> bool:
    return is_current(HOST_SO, HOST_SRC, HOST_FLAGS)


def device_current() -> bool:
    return is_current(DEVICE_SO, DEVICE_SRC, DEVICE_FLAGS)


def selected_host_so() -> str:
    """The host library the Python wrapper loads: the sanitized build when ACCO_SANITIZE=1."""
    return HOST_SAN_SO if os.environ.get("ACCO_SANITIZE") == "1" else HOST_SO


def ensure_host(so: str) -> str:
    if so == HOST_SAN_SO:
        if not is_current(so, HOST_SRC, HOST_SAN_FLAGS):
            build_host_sanitized()
    elif not host_current():
        build_host()
    return so


def build_all() -> None:
    build_host()
    build_device()


if __name__ == "__main__":
    build_all()
    print(HOST_SO)
    print(DEVICE_SO)

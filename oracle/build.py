"""Build the CPU oracle (test infrastructure) in-tree with gcc."""
import hashlib
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ORACLE_SO = os.path.join(HERE, "libacco_oracle.so")
# the same source under AddressSanitizer + UndefinedBehaviorSanitizer (host code only)
ORACLE_SAN_SO = os.path.join(HERE, "libacco_oracle_san.so")
SOURCES = [os.path.join(HERE, "acco_oracle.c")]

FLAGS = ["-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off", "-fno-fast-math",
         "-fvisibility=hidden", "-Wall", "-Wextra"]
SAN_FLAGS = ["-O1", "-g", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
             "-fno-fast-math", "-fvisibility=hidden", "-Wall", "-Wextra",
             "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"]


def source_hash(flags) -> str:
    h = hashlib.sha256(" ".join(flags).encode())
    for path in SOURCES:
        h.update(open(path, "rb").read())
    return h.hexdigest()


def is_current(so: str = ORACLE_SO, flags=FLAGS) -> bool:
    """Was `so` built from the sources and flags as they are now?"""
    try:
        return os.path.exists(so) and open(so + ".srchash").read() == source_hash(flags)
    except OSError:
        return False


def _build(so, flags) -> str:
    subprocess.run(["gcc", *flags, *SOURCES, "-o", so, "-lm"], check=True, cwd=HERE)
    open(so + ".srchash", "w").write(source_hash(flags))
    return so


def build_oracle() -> str:
    return _build(ORACLE_SO, FLAGS)


def build_oracle_sanitized() -> str:
    return _build(ORACLE_SAN_SO, SAN_FLAGS)


def selected_so() -> str:
    """The library the Python wrapper loads: the sanitized build when ACCO_SANITIZE=1 (the
    process must then run with the sanitizer runtime preloaded)."""
    return ORACLE_SAN_SO if os.environ.get("ACCO_SANITIZE") == "1" else ORACLE_SO


def ensure(so: str) -> str:
    if so == ORACLE_SAN_SO:
        if not is_current(so, SAN_FLAGS):
            build_oracle_sanitized()
    elif not is_current(so, FLAGS):
        build_oracle()
    return so


if __name__ == "__main__":
    print(build_oracle())

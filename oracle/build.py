"""Build the CPU oracle (test infrastructure) in-tree with gcc."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ORACLE_SO = os.path.join(HERE, "libacco_oracle.so")


def build_oracle() -> str:
    cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-ffp-contract=off",
           "-fno-fast-math", "-fvisibility=hidden", "-Wall", "-Wextra",
           os.path.join(HERE, "acco_oracle.c"), "-o", ORACLE_SO, "-lm"]
    subprocess.run(cmd, check=True, cwd=HERE)
    return ORACLE_SO


if __name__ == "__main__":
    print(build_oracle())

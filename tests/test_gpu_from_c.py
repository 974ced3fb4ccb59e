"""The library driven from a plain C program (tests/c/round_from_c.c): device memory from
hipMalloc, a stream from hipStreamCreate, one ACCO round through the five base entry points and
one through the fused forms - no Python and no torch in that process.  The program's inputs are
drawn here, its outputs are compared here with the oracle's binary32 form, bit for bit."""
import os
import subprocess

import numpy as np
import pytest

import oracle
from parity import adam_state, bit_mismatches

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HP = (6e-4, 0.9, 0.95, 1e-8, 0.1)
HYPER = dict(lr=HP[0], b1=HP[1], b2=HP[2], eps=HP[3], wd=HP[4])
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")


@pytest.fixture(scope="module")
def exe(tmp_path_factory):
    from paper_2406_02613_amd import build
    if not os.path.exists(build.ACCO_SO):
        pytest.fail("libacco.so is not built")
    libdir = os.path.dirname(build.ACCO_SO)
    path = str(tmp_path_factory.mktemp("c") / "round_from_c")
    subprocess.run(["gcc", "-std=c99", "-O1", "-Wall", "-Wextra", "-Werror", "-D__HIP_PLATFORM_AMD__",
                    "-I", os.path.join(ROCM, "include"), "-I", os.path.join(ROOT, "include"),
                    os.path.join(ROOT, "tests", "c", "round_from_c.c"), "-o", path,
                    "-L", libdir, "-lacco", "-L", os.path.join(ROCM, "lib"), "-lamdhip64",
                    f"-Wl,-rpath,{libdir}", f"-Wl,-rpath,{os.path.join(ROCM, 'lib')}"], check=True)
    return path


def _read(f, dtype, count):
    a = np.fromfile(f, dtype=dtype, count=count)
    assert a.size == count, "output file too short"
    return a


@pytest.mark.parametrize("n,W,K,kind,step0", [
    (100_037, 3, 1, "cold", 0),
    (100_037, 3, 2, "warm", 7),
    (70_001, 5, 4, "wide", 12345),
    (5, 2, 3, "warm", 1),
    (262_144, 9, 2, "warm", 99),          # more shards than one reduction pass takes
])
def test_round_driven_from_c_meets_the_oracle(exe, tmp_path, n, W, K, kind, step0):
    print(f"round from C: n={n} W={W} K={K} kind={kind} step0={step0}", flush=True)
    rng = np.random.default_rng(n + 31 * W + K)
    theta, m, v, _ = adam_state(rng, n, kind, HYPER, step0 + 1, 2 * W * K)
    grads = [[[oracle.cast((rng.standard_normal(n) * 1e-3).astype(np.float32)) for _ in range(K)]
              for _ in range(W)] for _ in range(2)]
    fin, fout = str(tmp_path / "in.bin"), str(tmp_path / "out.bin")
    with open(fin, "wb") as f:
        np.array([n, W, K, step0], np.int64).tofile(f)
        np.array(HP, np.float64).tofile(f)
        for a in (theta, m, v):
            a.astype(np.float32).tofile(f)
        for stage in grads:
            for worker in stage:
                for g in worker:
                    g.astype(np.uint16).tofile(f)
    r = subprocess.run([exe, fin, fout], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, (r.returncode, r.stdout, r.stderr)
    assert "round_from_c ok" in r.stdout

    # the same round in the oracle (Alg. 1, communication stream), binary32 form
    ohp = oracle.make_hyper(*HP)
    gsum = np.empty(n, np.float32)
    want = {}
    th, mm, vv = theta.copy(), m.copy(), v.copy()
    total = 0
    for stage in range(2):
        shards = []
        for w in range(W):
            acc = np.empty(n, np.float32)
            for k in range(K):
                oracle.accumulate(acc, grads[stage][w][k], init=(k == 0))
            shards.append(oracle.cast(acc))
        oracle.reduce(gsum, shards, accumulate_=(stage == 1))
        total += W * K
        if stage == 0:
            _, want["tilde16"] = oracle.estimate(th, mm, vv, gsum, ohp, step0 + 1, total,
                                                 want_f32=False, precision="f32")
        else:
            want["theta16"] = oracle.commit(th, mm, vv, gsum, ohp, step0 + 1, total, precision="f32")

    with open(fout, "rb") as f:
        for path in ("base", "fused"):
            got16 = _read(f, np.uint16, n)
            assert np.array_equal(got16, want["tilde16"]), (path, "theta~ bf16")
            for name, ref in (("theta", th), ("m", mm), ("v", vv)):
                assert bit_mismatches(_read(f, np.float32, n), ref) == 0, (path, name)
            assert np.array_equal(_read(f, np.uint16, n), want["theta16"]), (path, "theta bf16")
            step, tot = _read(f, np.int64, 2)
            assert (step, tot) == (step0 + 1, 2 * W * K), path
        assert f.read() == b""

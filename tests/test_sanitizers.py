"""The CPU-side C code (the oracle and the host half of the input generator) under
AddressSanitizer + UndefinedBehaviorSanitizer: the oracle's pins and the generator's tests are
run once more in a child interpreter that loads the sanitized builds, plus edge cases chosen
for out-of-bounds hazards (n = 0, n = 1, ragged tails, 64 workers).  Host code only; nothing
here touches a GPU or the HIP library."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

EDGE_CASES = r"""
import numpy as np
import oracle, synth
hp = oracle.make_hyper(6e-4, 0.9, 0.95, 1e-8, 0.1)
rng = np.random.default_rng(0)
for n in (0, 1, 2, 3, 7, 8, 9, 63, 64, 65, 4096 + 37):
    g = oracle.cast((rng.standard_normal(n) * 1e-3).astype(np.float32))
    acc = np.zeros(n, np.float32)
    oracle.accumulate(acc, g, init=True)
    oracle.accumulate(acc, g, init=False)
    run = g.copy()
    oracle.accumulate_bf16(run, g, init=False)
    for W in (1, 2, 64):
        shards = [oracle.cast(acc) for _ in range(W)]
        gsum = np.zeros(n, np.float32)
        oracle.reduce(gsum, shards, accumulate_=False)
        oracle.reduce(gsum, [acc] * W, accumulate_=True)
    th, m, v = (rng.standard_normal(n).astype(np.float32) for _ in range(3))
    v = np.abs(v)
    for prec in ("f32", "f64"):
        oracle.estimate(th, m, v, gsum, hp, 3, 5, precision=prec)
        oracle.commit(th.copy(), m.copy(), v.copy(), gsum, hp, 3, 5, precision=prec)
        oracle.sgd_step(th.copy(), gsum, 1e-3, 0.1, 5, commit=True, precision=prec)
    for name in ("tiny", "gpt2s", "1b", "7b_hetero"):
        w = synth.WORKLOADS[name]
        for j0 in (0, max(0, w.n - n)):
            assert synth.host_grad_bf16(w.grad_spec(1, 2, w.workers - 1, 1), j0, n).shape == (n,)
            assert w.host_theta(j0, n).shape == (n,)
sh = oracle.OracleShard(np.zeros(37, np.float32), 64, hp, precision="f32")
for stage in (1, 2):
    for w in range(64):
        sh.add_microbatch(w, np.full(37, 0x3C00, np.uint16))
    sh.stage1() if stage == 1 else sh.stage2()
assert sh.step == 1
print("edge cases ok")
"""


def _sanitizer_env():
    def runtime(name):
        out = subprocess.run(["gcc", f"-print-file-name={name}"], capture_output=True, text=True,
                             check=True).stdout.strip()
        return out if os.path.isabs(out) and os.path.exists(out) else None
    asan, ubsan = runtime("libasan.so"), runtime("libubsan.so")
    if asan is None or ubsan is None:
        pytest.skip("gcc's sanitizer runtimes are not installed")
    env = dict(os.environ)
    env["ACCO_SANITIZE"] = "1"
    # the interpreter itself is not instrumented: the runtimes come in by preload, and the leak
    # check (which would report the interpreter's own allocations) is off
    env["LD_PRELOAD"] = " ".join(filter(None, [asan, ubsan, env.get("LD_PRELOAD")]))
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0:exitcode=66"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1:exitcode=66"
    env["PYTHONPATH"] = os.pathsep.join(filter(None, [ROOT, os.path.join(ROOT, "tests"),
                                                      env.get("PYTHONPATH")]))
    return env


def _build_sanitized():
    from oracle import build as ob
    from synth import build as sb
    ob.ensure(ob.ORACLE_SAN_SO)
    sb.ensure_host(sb.HOST_SAN_SO)


def _run(args, env):
    r = subprocess.run([sys.executable, *args], cwd=ROOT, env=env, capture_output=True, text=True,
                       timeout=900)
    tail = (r.stdout[-3000:] + "\n" + r.stderr[-3000:])
    assert "ERROR: AddressSanitizer" not in tail and "runtime error:" not in tail, tail
    assert r.returncode == 0, tail
    return r.stdout


def test_the_sanitized_builds_are_the_ones_loaded_and_they_do_catch_errors():
    _build_sanitized()
    env = _sanitizer_env()
    out = _run(["-c", "import oracle, synth; from oracle import build as ob; "
                      "from synth import build as sb; oracle.lib(); synth.host_lib(); "
                      "maps = open('/proc/self/maps').read(); "
                      "print(int(ob.ORACLE_SAN_SO in maps), int(sb.HOST_SAN_SO in maps), "
                      "int(ob.ORACLE_SO in maps), int(sb.HOST_SO in maps))"], env)
    assert out.split()[-4:] == ["1", "1", "0", "0"]
    # a planted overrun in the CALLER (a buffer one element too short) must be reported: the
    # check is live, not a no-op
    bad = ("import numpy as np, oracle, ctypes; a = np.zeros(8, np.float32); "
           "g = np.zeros(8, np.uint16); "
           "oracle.lib().oracle_accumulate(a.ctypes.data, g.ctypes.data, 4096, 0)")
    r = subprocess.run([sys.executable, "-c", bad], cwd=ROOT, env=env, capture_output=True,
                       text=True, timeout=300)
    assert r.returncode != 0 and "AddressSanitizer" in r.stderr


def test_edge_cases_under_the_sanitizers():
    _build_sanitized()
    assert "edge cases ok" in _run(["-c", EDGE_CASES], _sanitizer_env())


def test_oracle_pins_and_generator_tests_under_the_sanitizers():
    _build_sanitized()
    files = ["tests/test_oracle_bf16.py", "tests/test_oracle_sums.py", "tests/test_oracle_adamw.py",
             "tests/test_oracle_round.py", "tests/test_oracle_schemes.py", "tests/test_synth.py",
             "tests/test_parity_bound.py"]
    out = _run(["-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider", *files],
               _sanitizer_env())
    assert " passed" in out and "failed" not in out


def _hip_host_sanitizer_env():
    """Environment of a child interpreter that loads the HIP library's host-sanitized build.
    That build comes from clang (hipcc), so it needs clang's runtime, not gcc's: the two cannot
    share a process, hence a child of its own with the oracle in its plain build."""
    from paper_2406_02613_amd import build as ab
    runtime = ab.sanitizer_runtime()
    if runtime is None:
        pytest.skip("clang's shared AddressSanitizer runtime is not installed")
    ab.ensure_host_sanitized()
    env = dict(os.environ)
    env.pop("ACCO_SANITIZE", None)
    env["ACCO_SANITIZE_HOST"] = "1"
    env["LD_PRELOAD"] = " ".join(filter(None, [runtime, env.get("LD_PRELOAD")]))
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0:exitcode=66"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1:exitcode=66"
    env["PYTHONPATH"] = os.pathsep.join(filter(None, [ROOT, os.path.join(ROOT, "tests"),
                                                      env.get("PYTHONPATH")]))
    return env


def test_host_half_of_the_hip_library_under_the_sanitizers():
    """Validation, host counters, folded scalars and launch settings of the C-ABI library with
    its host code instrumented (no device work: every call here stops before a launch)."""
    env = _hip_host_sanitizer_env()
    from paper_2406_02613_amd import build as ab
    out = _run(["-c", "import paper_2406_02613_amd.binding as B; B.lib(); "
                      "maps = open('/proc/self/maps').read(); "
                      f"print(int({ab.ACCO_HOST_SAN_SO!r} in maps), int({ab.ACCO_SO!r} in maps))"], env)
    assert out.split()[-2:] == ["1", "0"]
    # a planted overrun in the CALLER (64 counts announced, 63 there) must be reported
    bad = ("import ctypes, paper_2406_02613_amd.binding as B; L = B.lib(); "
           "counts = (ctypes.c_int64 * 80)(*([1] * 80)); total = ctypes.c_int64(0); "
           "shards = (ctypes.c_void_p * 64)(*([0x100000] * 64)); "
           "p = ctypes.cast(ctypes.addressof(counts) + 8 * 17, ctypes.POINTER(ctypes.c_int64)); "
           "L.acco_reduce_shards(0x200000, shards, 64, 0, 0, 0, p, ctypes.byref(total), None, "
           "None, None)")
    r = subprocess.run([sys.executable, "-c", bad], cwd=ROOT, env=env, capture_output=True,
                       text=True, timeout=300)
    assert r.returncode != 0 and "AddressSanitizer" in r.stderr, (r.returncode, r.stderr[-2000:])
    out = _run(["-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "tests/test_abi_host.py"], env)
    assert " passed" in out and "failed" not in out

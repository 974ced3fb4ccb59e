"""The C-ABI library on a machine without a GPU: it loads, exports what the header declares,
validates arguments before any launch, and keeps the host counters exactly."""
import ctypes
import os
import re

import pytest

from paper_2406_02613_amd import binding as B
from paper_2406_02613_amd import layout

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "acco.h")

A, Bp, C, D, E, F = (0x10000 * k for k in range(1, 7))   # fake, aligned "device" addresses
NONE = None


def vp(x):
    return ctypes.c_void_p(x)


def test_every_symbol_declared_in_the_header_is_exported():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(acco_[a-z0-9_]+)\s*\(", text))
    assert declared == set(B.EXPORTS)
    L = B.lib()
    for name in declared:
        assert getattr(L, name) is not None
    assert B.version() >= 100
    assert "ALIGN" in B.status_string(B.ACCO_ERR_ALIGN)
    assert "unknown" in B.status_string(-99)


def test_struct_layout_matches_the_header():
    assert ctypes.sizeof(B.AdamW) == 5 * 8
    assert [f[0] for f in B.AdamW._fields_] == ["lr", "beta1", "beta2", "eps", "weight_decay"]


def test_accumulate_validation_and_counter():
    L = B.lib()
    c = ctypes.c_int64(0)
    assert L.acco_accumulate(NONE, vp(Bp), 4, 0, ctypes.byref(c), NONE) == B.ACCO_ERR_NULL
    assert L.acco_accumulate(vp(A), NONE, 4, 0, ctypes.byref(c), NONE) == B.ACCO_ERR_NULL
    assert L.acco_accumulate(NONE, NONE, 0, 1, NONE, NONE) == 0    # empty shard: no addresses
    assert L.acco_accumulate(vp(A), vp(Bp), -1, 0, ctypes.byref(c), NONE) == B.ACCO_ERR_SIZE
    assert L.acco_accumulate(vp(A), vp(Bp), (1 << 40) + 1, 0, NONE, NONE) == B.ACCO_ERR_SIZE
    assert L.acco_accumulate(vp(A + 4), vp(Bp), 0, 0, NONE, NONE) == B.ACCO_ERR_ALIGN
    assert L.acco_accumulate(vp(A), vp(Bp + 2), 0, 0, NONE, NONE) == B.ACCO_ERR_ALIGN
    assert L.acco_accumulate(vp(A), vp(Bp), 0, 2, NONE, NONE) == B.ACCO_ERR_ARG
    assert L.acco_accumulate(vp(A), vp(A + 16), 64, 0, NONE, NONE) == B.ACCO_ERR_ALIAS
    assert c.value == 0                      # errors leave the counter alone
    # n == 0: no device work, bookkeeping still happens
    for want in (1, 2, 3):
        assert L.acco_accumulate(vp(A), vp(Bp), 0, int(want == 1), ctypes.byref(c), NONE) == 0
        assert c.value == want
    assert L.acco_accumulate(vp(A), vp(Bp), 0, 1, ctypes.byref(c), NONE) == 0 and c.value == 1
    c.value = -3
    assert L.acco_accumulate(vp(A), vp(Bp), 0, 0, ctypes.byref(c), NONE) == B.ACCO_ERR_ARG
    c.value = 2 ** 63 - 1
    assert L.acco_accumulate(vp(A), vp(Bp), 0, 0, ctypes.byref(c), NONE) == B.ACCO_ERR_ARG


def test_cast_validation():
    L = B.lib()
    assert L.acco_cast_params(NONE, vp(A), 4, NONE) == B.ACCO_ERR_NULL
    assert L.acco_cast_params(vp(A), vp(Bp), -5, NONE) == B.ACCO_ERR_SIZE
    assert L.acco_cast_params(vp(A + 8), vp(Bp), 0, NONE) == B.ACCO_ERR_ALIGN
    assert L.acco_cast_params(vp(A), vp(A), 16, NONE) == B.ACCO_ERR_ALIAS
    assert L.acco_cast_params(vp(A), vp(Bp), 0, NONE) == 0


def _shards(*addrs):
    return (ctypes.c_void_p * len(addrs))(*addrs)


def test_reduce_validation_and_count_totals():
    L = B.lib()
    s2 = _shards(Bp, C)
    cnt = (ctypes.c_int64 * 2)(3, 4)
    tot = ctypes.c_int64(100)
    r = L.acco_reduce_shards
    assert r(NONE, s2, 2, 0, 4, 0, cnt, ctypes.byref(tot), NONE, NONE, NONE) == B.ACCO_ERR_NULL
    assert r(vp(A), NONE, 2, 0, 0, 0, cnt, ctypes.byref(tot), NONE, NONE, NONE) == B.ACCO_ERR_NULL
    assert r(vp(A), s2, 0, 0, 0, 0, cnt, ctypes.byref(tot), NONE, NONE, NONE) == B.ACCO_ERR_SIZE
    assert r(vp(A), s2, 65, 0, 0, 0, cnt, ctypes.byref(tot), NONE, NONE, NONE) == B.ACCO_ERR_SIZE
    assert r(vp(A), s2, 2, 7, 0, 0, cnt, ctypes.byref(tot), NONE, NONE, NONE) == B.ACCO_ERR_ARG
    assert r(vp(A), s2, 2, 0, 0, 3, cnt, ctypes.byref(tot), NONE, NONE, NONE) == B.ACCO_ERR_ARG
    assert r(vp(A), s2, 2, 0, 0, 0, cnt, NONE, NONE, NONE, NONE) == B.ACCO_ERR_NULL      # counts w/o total
    assert r(vp(A), s2, 2, 0, 0, 0, NONE, ctypes.byref(tot), NONE, NONE, NONE) == B.ACCO_ERR_NULL
    assert r(vp(A), _shards(Bp, 0), 2, 0, 4, 0, NONE, NONE, NONE, NONE, NONE) == B.ACCO_ERR_NULL
    assert r(vp(A), _shards(Bp, C + 2), 2, 0, 0, 0, NONE, NONE, NONE, NONE, NONE) == B.ACCO_ERR_ALIGN
    assert r(vp(A), _shards(Bp, A), 2, 0, 8, 0, NONE, NONE, NONE, NONE, NONE) == B.ACCO_ERR_ALIAS
    neg = (ctypes.c_int64 * 2)(3, -1)
    assert r(vp(A), s2, 2, 0, 0, 0, neg, ctypes.byref(tot), NONE, NONE, NONE) == B.ACCO_ERR_ARG
    big = (ctypes.c_int64 * 2)(2 ** 62, 2 ** 62)
    assert r(vp(A), s2, 2, 0, 0, 0, big, ctypes.byref(tot), NONE, NONE, NONE) == B.ACCO_ERR_ARG
    assert tot.value == 100
    # stage 1: total = sum(counts); stage 2: total += sum(counts)
    assert r(vp(A), s2, 2, 0, 0, 0, cnt, ctypes.byref(tot), NONE, NONE, NONE) == 0 and tot.value == 7
    cnt2 = (ctypes.c_int64 * 2)(5, 6)
    assert r(vp(A), s2, 2, 1, 0, 1, cnt2, ctypes.byref(tot), NONE, NONE, NONE) == 0 and tot.value == 18
    # 64 workers are accepted
    many = _shards(*[Bp + 0x1000 * k for k in range(64)])
    assert r(vp(A), many, 64, 0, 0, 0, NONE, NONE, NONE, NONE, NONE) == 0


GOOD = B.make_hyper(6e-4, 0.9, 0.95, 1e-8, 0.1)


@pytest.mark.parametrize("field,value", [("lr", -1.0), ("lr", float("nan")), ("lr", float("inf")),
                                         ("beta1", 1.0), ("beta1", -0.1), ("beta2", 1.5),
                                         ("beta2", float("nan")), ("eps", -1e-8),
                                         ("eps", float("inf")), ("weight_decay", -0.1),
                                         ("weight_decay", float("nan"))])
def test_bad_hyper_parameters_are_rejected(field, value):
    L = B.lib()
    hp = B.make_hyper(6e-4, 0.9, 0.95, 1e-8, 0.1)
    setattr(hp, field, value)
    step = ctypes.c_int64(0)
    rc = L.acco_estimate_step(vp(A), vp(Bp), vp(C), vp(D), vp(E), NONE, 0, ctypes.byref(hp), 0, 1,
                              NONE, NONE)
    assert rc == B.ACCO_ERR_ARG
    rc = L.acco_commit_step(vp(A), vp(Bp), vp(C), vp(D), NONE, 0, ctypes.byref(hp),
                            ctypes.byref(step), 1, NONE, NONE)
    assert rc == B.ACCO_ERR_ARG and step.value == 0


def test_estimate_validation():
    L = B.lib()
    e = L.acco_estimate_step
    hp = ctypes.byref(GOOD)
    assert e(NONE, vp(Bp), vp(C), vp(D), vp(E), NONE, 4, hp, 0, 1, NONE, NONE) == B.ACCO_ERR_NULL
    assert e(vp(A), vp(Bp), vp(C), vp(D), NONE, NONE, 4, hp, 0, 1, NONE, NONE) == B.ACCO_ERR_NULL
    assert e(vp(A), vp(Bp), vp(C), vp(D), vp(E), NONE, 0, NONE, 0, 1, NONE, NONE) == B.ACCO_ERR_NULL
    assert e(vp(A), vp(Bp), vp(C), vp(D), vp(E), NONE, -1, hp, 0, 1, NONE, NONE) == B.ACCO_ERR_SIZE
    assert e(vp(A), vp(Bp + 4), vp(C), vp(D), vp(E), NONE, 0, hp, 0, 1, NONE, NONE) == B.ACCO_ERR_ALIGN
    assert e(vp(A), vp(Bp), vp(C), vp(D), vp(E), vp(F + 2), 0, hp, 0, 1, NONE, NONE) == B.ACCO_ERR_ALIGN
    assert e(vp(A), vp(Bp), vp(C), vp(D), vp(E), NONE, 0, hp, -1, 1, NONE, NONE) == B.ACCO_ERR_ARG
    assert e(vp(A), vp(Bp), vp(C), vp(D), vp(E), NONE, 0, hp, 0, 0, NONE, NONE) == B.ACCO_ERR_ARG
    # the speculative output may not land on theta, m, v or gsum
    for alias in (A, Bp, C, D):
        assert e(vp(A), vp(Bp), vp(C), vp(D), vp(alias), NONE, 8, hp, 0, 1, NONE, NONE) == B.ACCO_ERR_ALIAS
        assert e(vp(A), vp(Bp), vp(C), vp(D), NONE, vp(alias), 8, hp, 0, 1, NONE, NONE) == B.ACCO_ERR_ALIAS
    assert e(vp(A), vp(Bp), vp(C), vp(D), vp(E), vp(E), 8, hp, 0, 1, NONE, NONE) == B.ACCO_ERR_ALIAS
    assert e(vp(A), vp(Bp), vp(C), vp(D), vp(E), vp(F), 0, hp, 5, 3, NONE, NONE) == 0


def test_commit_validation_and_step_counter():
    L = B.lib()
    c = L.acco_commit_step
    hp = ctypes.byref(GOOD)
    step = ctypes.c_int64(0)
    st = ctypes.byref(step)
    assert c(vp(A), vp(Bp), vp(C), NONE, NONE, 4, hp, st, 1, NONE, NONE) == B.ACCO_ERR_NULL
    assert c(vp(A), vp(Bp), vp(C), vp(D), NONE, 0, hp, NONE, 1, NONE, NONE) == B.ACCO_ERR_NULL
    assert c(vp(A), vp(Bp), vp(C), vp(D), NONE, -2, hp, st, 1, NONE, NONE) == B.ACCO_ERR_SIZE
    assert c(vp(A + 12), vp(Bp), vp(C), vp(D), NONE, 0, hp, st, 1, NONE, NONE) == B.ACCO_ERR_ALIGN
    assert c(vp(A), vp(Bp), vp(C), vp(D), NONE, 0, hp, st, 0, NONE, NONE) == B.ACCO_ERR_ARG
    assert c(vp(A), vp(A), vp(C), vp(D), NONE, 4, hp, st, 1, NONE, NONE) == B.ACCO_ERR_ALIAS
    assert c(vp(A), vp(Bp), vp(C), vp(C + 16), NONE, 64, hp, st, 1, NONE, NONE) == B.ACCO_ERR_ALIAS
    assert c(vp(A), vp(Bp), vp(C), vp(D), vp(A), 4, hp, st, 1, NONE, NONE) == B.ACCO_ERR_ALIAS
    assert step.value == 0
    for want in (1, 2, 3):
        assert c(vp(A), vp(Bp), vp(C), vp(D), vp(E), 0, hp, st, 4, NONE, NONE) == 0
        assert step.value == want
    step.value = -1
    assert c(vp(A), vp(Bp), vp(C), vp(D), NONE, 0, hp, st, 1, NONE, NONE) == B.ACCO_ERR_ARG


def test_launch_shape_validation():
    B.set_launch_shape("commit", 256, 2, 0)
    for bad in (("commit", 100, 2, 0), ("commit", 1024, 2, 0), ("commit", 256, 3, 0),
                ("commit", 256, 2, -1), ("nope", 256, 2, 0)):
        with pytest.raises(B.AccoError):
            B.set_launch_shape(*bad)
    B.reset_launch_settings()


def test_resident_wave_bound_validation():
    for ok in (0, 3, 9, 32):
        B.set_resident_waves("cast", ok)
    for bad in (("cast", 1), ("cast", 2), ("cast", 33), ("cast", -4), ("nope", 8)):
        with pytest.raises(B.AccoError):
            B.set_resident_waves(*bad)
    # the bound counts wavefronts: workgroups of four need room for at least three of them
    B.set_launch_shape("cast", 256, 1, 0)
    with pytest.raises(B.AccoError):
        B.set_resident_waves("cast", 8)
    B.set_resident_waves("cast", 12)
    B.reset_launch_settings()


def test_binding_rejects_host_tensors_before_touching_the_library():
    import torch
    t = torch.zeros(8)
    with pytest.raises(ValueError):
        B.acco_cast_params(torch.zeros(8, dtype=torch.bfloat16), t)


def test_buffer_inventory_reproduces_the_papers_memory_table():
    path = os.path.join(os.path.dirname(__file__), "golden", "memory_table.txt")
    rows = [ln.split() for ln in open(path) if ln.strip() and not ln.startswith("#")]
    names = {"ACCO": "acco", "ZeRO-1": "zero1", "DDP": "ddp"}
    assert len(rows) == 3
    for method, _formula, printed in rows:
        gb = layout.replica_bytes_per_param(names[method], 64) * 7.5e9 / 1e9
        assert round(gb) == int(printed)
    assert layout.STATE_F32 == 12
    assert layout.BYTES_PER_ELEM["commit"] == 28 and layout.BYTES_PER_ELEM["commit_bf16"] == 30
    assert layout.reduce_bytes_per_elem(8, True, False) == 20
    assert layout.reduce_bytes_per_elem(8, True, True) == 24


def test_accumulate_publish_validation_and_counter():
    L = B.lib()
    f = L.acco_accumulate_publish
    c = ctypes.c_int64(4)
    cr = ctypes.byref(c)
    assert f(vp(A), NONE, vp(C), 4, 0, 0, cr, NONE) == B.ACCO_ERR_NULL
    assert f(vp(A), vp(Bp), NONE, 4, 0, 0, cr, NONE) == B.ACCO_ERR_NULL
    assert f(NONE, vp(Bp), vp(C), 4, 0, 0, cr, NONE) == B.ACCO_ERR_NULL      # needs acc to add to
    assert f(NONE, vp(Bp), vp(C), 4, 1, 1, cr, NONE) == B.ACCO_ERR_NULL      # needs acc to keep
    assert f(vp(A), vp(Bp), vp(C), 4, 2, 0, cr, NONE) == B.ACCO_ERR_ARG
    assert f(vp(A), vp(Bp), vp(C), 4, 0, 5, cr, NONE) == B.ACCO_ERR_ARG
    assert f(vp(A), vp(Bp), vp(C + 6), 4, 0, 0, cr, NONE) == B.ACCO_ERR_ALIGN
    assert f(vp(A), vp(Bp), vp(Bp), 8, 0, 0, cr, NONE) == B.ACCO_ERR_ALIAS
    assert f(vp(A), vp(Bp), vp(A + 16), 64, 0, 0, cr, NONE) == B.ACCO_ERR_ALIAS
    assert f(vp(A), vp(Bp), vp(C), -1, 0, 0, cr, NONE) == B.ACCO_ERR_SIZE
    assert c.value == 4
    assert f(vp(A), vp(Bp), vp(C), 0, 0, 0, cr, NONE) == 0 and c.value == 5
    assert f(NONE, vp(Bp), vp(C), 0, 1, 0, cr, NONE) == 0 and c.value == 1


def test_fused_reduce_steps_validation_and_counters():
    L = B.lib()
    hp = ctypes.byref(GOOD)
    s2 = _shards(E, F)
    cnt = (ctypes.c_int64 * 2)(3, 4)
    tot = ctypes.c_int64(50)
    tr = ctypes.byref(tot)
    est, com = L.acco_reduce_estimate_step, L.acco_reduce_commit_step
    G, H = 0x70000, 0x80000
    # estimate
    assert est(vp(A), vp(Bp), vp(C), vp(D), s2, 2, 0, NONE, tr, vp(G), NONE, 0, hp, 0, NONE, NONE, NONE) == B.ACCO_ERR_NULL
    assert est(vp(A), vp(Bp), vp(C), vp(D), s2, 2, 0, cnt, NONE, vp(G), NONE, 0, hp, 0, NONE, NONE, NONE) == B.ACCO_ERR_NULL
    assert est(vp(A), vp(Bp), vp(C), NONE, s2, 2, 0, cnt, tr, vp(G), NONE, 4, hp, 0, NONE, NONE, NONE) == B.ACCO_ERR_NULL
    assert est(vp(A), vp(Bp), vp(C), vp(D), s2, 2, 0, cnt, tr, NONE, NONE, 4, hp, 0, NONE, NONE, NONE) == B.ACCO_ERR_NULL
    assert est(vp(A), vp(Bp), vp(C), vp(D), s2, 0, 0, cnt, tr, vp(G), NONE, 0, hp, 0, NONE, NONE, NONE) == B.ACCO_ERR_SIZE
    assert est(vp(A), vp(Bp), vp(C), vp(D), s2, 2, 3, cnt, tr, vp(G), NONE, 0, hp, 0, NONE, NONE, NONE) == B.ACCO_ERR_ARG
    assert est(vp(A), vp(Bp), vp(C), vp(D), s2, 2, 0, cnt, tr, vp(G), NONE, 0, hp, -1, NONE, NONE, NONE) == B.ACCO_ERR_ARG
    zero = (ctypes.c_int64 * 2)(0, 0)
    assert est(vp(A), vp(Bp), vp(C), vp(D), s2, 2, 0, zero, tr, vp(G), NONE, 0, hp, 0, NONE, NONE, NONE) == B.ACCO_ERR_ARG
    assert est(vp(A), vp(Bp), vp(C), vp(A), s2, 2, 0, cnt, tr, vp(G), NONE, 8, hp, 0, NONE, NONE, NONE) == B.ACCO_ERR_ALIAS
    assert est(vp(A), vp(Bp), vp(C), vp(D), s2, 2, 0, cnt, tr, vp(E), NONE, 8, hp, 0, NONE, NONE, NONE) == B.ACCO_ERR_ALIAS
    assert est(vp(A), vp(Bp), vp(C), vp(D), _shards(E, D), 2, 0, cnt, tr, vp(G), NONE, 8, hp, 0, NONE, NONE, NONE) == B.ACCO_ERR_ALIAS
    assert tot.value == 50
    assert est(vp(A), vp(Bp), vp(C), vp(D), s2, 2, 0, cnt, tr, vp(G), vp(H), 0, hp, 0, NONE, NONE, NONE) == 0
    assert tot.value == 7                     # stage 1: the total starts afresh
    # commit
    step = ctypes.c_int64(9)
    sr = ctypes.byref(step)
    assert com(vp(A), vp(Bp), vp(C), vp(D), s2, 2, 0, cnt, tr, vp(G), 0, hp, NONE, NONE, NONE, NONE) == B.ACCO_ERR_NULL
    assert com(vp(A), vp(Bp), vp(C), vp(D), s2, 2, 0, NONE, tr, vp(G), 0, hp, sr, NONE, NONE, NONE) == B.ACCO_ERR_NULL
    assert com(vp(A), vp(Bp), vp(A), vp(D), s2, 2, 0, cnt, tr, vp(G), 8, hp, sr, NONE, NONE, NONE) == B.ACCO_ERR_ALIAS
    assert com(vp(A), vp(Bp), vp(C), vp(D), _shards(E, Bp), 2, 0, cnt, tr, vp(G), 8, hp, sr, NONE, NONE, NONE) == B.ACCO_ERR_ALIAS
    assert com(vp(A), vp(Bp), vp(C), vp(D), s2, 2, 0, cnt, tr, vp(E), 8, hp, sr, NONE, NONE, NONE) == B.ACCO_ERR_ALIAS
    assert com(vp(A), vp(Bp), vp(C), vp(D + 4), s2, 2, 0, cnt, tr, vp(G), 8, hp, sr, NONE, NONE, NONE) == B.ACCO_ERR_ALIGN
    assert tot.value == 7 and step.value == 9
    assert com(vp(A), vp(Bp), vp(C), vp(D), s2, 2, 0, cnt, tr, vp(G), 0, hp, sr, NONE, NONE, NONE) == 0
    assert tot.value == 14 and step.value == 10      # stage 2 adds onto the stage-1 total


def test_sgd_steps_validation_and_step_counter():
    L = B.lib()
    hp = B.make_sgd(0.1, 0.0)
    h = ctypes.byref(hp)
    est, com = L.acco_sgd_estimate_step, L.acco_sgd_commit_step
    assert est(NONE, vp(Bp), vp(C), NONE, 4, h, 1, NONE) == B.ACCO_ERR_NULL
    assert est(vp(A), vp(Bp), NONE, NONE, 4, h, 1, NONE) == B.ACCO_ERR_NULL
    assert est(vp(A), vp(Bp), vp(C), NONE, 4, NONE, 1, NONE) == B.ACCO_ERR_NULL
    assert est(vp(A), vp(Bp), vp(C), NONE, 4, h, 0, NONE) == B.ACCO_ERR_ARG
    assert est(vp(A), vp(Bp), vp(A), NONE, 4, h, 1, NONE) == B.ACCO_ERR_ALIAS
    assert est(vp(A), vp(Bp), vp(C + 8), NONE, 4, h, 1, NONE) == B.ACCO_ERR_ALIGN
    assert est(vp(A), vp(Bp), vp(C), vp(D), 0, h, 1, NONE) == 0
    bad = B.make_sgd(-1.0, 0.0)
    assert est(vp(A), vp(Bp), vp(C), NONE, 0, ctypes.byref(bad), 1, NONE) == B.ACCO_ERR_ARG
    bad = B.make_sgd(0.1, float("nan"))
    assert est(vp(A), vp(Bp), vp(C), NONE, 0, ctypes.byref(bad), 1, NONE) == B.ACCO_ERR_ARG
    step = ctypes.c_int64(0)
    sr = ctypes.byref(step)
    assert com(vp(A), vp(Bp), NONE, 4, h, NONE, 1, NONE) == B.ACCO_ERR_NULL
    assert com(vp(A), vp(A), NONE, 4, h, sr, 1, NONE) == B.ACCO_ERR_ALIAS
    assert com(vp(A), vp(Bp), vp(A), 4, h, sr, 1, NONE) == B.ACCO_ERR_ALIAS
    assert com(vp(A), vp(Bp), NONE, -1, h, sr, 1, NONE) == B.ACCO_ERR_SIZE
    assert step.value == 0
    assert com(vp(A), vp(Bp), NONE, 0, h, sr, 2, NONE) == 0 and step.value == 1


def test_state_layout_validation_and_interleaved_aliasing_rules():
    L = B.lib()
    hp = ctypes.byref(GOOD)
    step = ctypes.c_int64(0)
    sr = ctypes.byref(step)
    com = L.acco_commit_step
    blk = 1024                                    # elements per block; 4 KiB per component
    base = 0x100000
    th, m, v, g = (base + 4 * blk * k for k in range(4))     # one block apart in one buffer
    out = 0x4000000
    n = 10 * blk + 5

    def lay(b, s):
        return ctypes.byref(B.Layout(b, s))

    # the interleaved arrangement is legal although the four extents overlap as byte ranges
    # (with n > 0 a launch would follow, so the accepted case is checked with n = 0 here and
    #  with real buffers in the GPU tests)
    assert com(vp(th), vp(m), vp(v), vp(g), vp(out), 0, hp, sr, 1, lay(blk, 4 * blk), NONE) == 0
    # the same pointers WITHOUT the layout are overlapping planar arrays
    assert com(vp(th), vp(m), vp(v), vp(g), vp(out), n, hp, sr, 1, NONE, NONE) == B.ACCO_ERR_ALIAS
    # two components on the same block slot, or half a block apart, do collide
    assert com(vp(th), vp(th), vp(v), vp(g), vp(out), n, hp, sr, 1, lay(blk, 4 * blk), NONE) == \
        B.ACCO_ERR_ALIAS
    assert com(vp(th), vp(th + 2 * blk), vp(v), vp(g), vp(out), n, hp, sr, 1, lay(blk, 4 * blk),
               NONE) == B.ACCO_ERR_ALIAS
    # a planar output inside the state buffer's extent is refused
    assert com(vp(th), vp(m), vp(v), vp(g), vp(base + 64 * blk), n, hp, sr, 1, lay(blk, 4 * blk),
               NONE) == B.ACCO_ERR_ALIAS
    # malformed layouts
    for b, s in ((3, 12), (1000, 4000), (blk, blk - 4), (blk, 4 * blk + 2), (2, 8), (-4, 16)):
        assert com(vp(th), vp(m), vp(v), vp(g), vp(out), 0, hp, sr, 1, lay(b, s), NONE) == \
            B.ACCO_ERR_ARG, (b, s)
    # block_elems == 0 means planar
    far = [0x10000000 * k for k in range(1, 5)]
    assert com(vp(far[0]), vp(far[1]), vp(far[2]), vp(far[3]), vp(out), 0, hp, sr, 1, lay(0, 0),
               NONE) == 0
    # reduce accepts a layout for gsum
    s2 = _shards(0x8000000, 0x9000000)
    assert L.acco_reduce_shards(vp(g), s2, 2, 0, 0, 0, NONE, NONE, lay(blk, 4 * blk), NONE, NONE) == 0
    assert L.acco_reduce_shards(vp(g), s2, 2, 0, 0, 0, NONE, NONE, lay(blk, 3), NONE, NONE) == B.ACCO_ERR_ARG


def test_cosine_schedule_closed_forms_and_oracle():
    import math
    import oracle
    base, lo, T = 6e-4, 6e-5, 50_000          # the paper's pre-training table: 6e-4, 50000 steps
    f = B.acco_lr_cosine
    assert f(base, lo, 0, 0, T) == base                                   # starts at the peak
    assert abs(f(base, lo, T, 0, T) - lo) < 1e-18                         # ends at the floor
    assert abs(f(base, lo, T // 2, 0, T) - (base + lo) / 2) < 1e-18       # half-way: the mean
    assert abs(f(base, lo, T // 3 * 1, 0, T // 3 * 3) - (lo + 0.75 * (base - lo))) < 1e-15
    assert f(base, lo, 10 * T, 0, T) == f(base, lo, T, 0, T)              # clamps after the end
    assert f(base, 0.0, T, 0, T) < 1e-18
    vals = [f(base, lo, s, 0, T) for s in range(0, T + 1, 500)]
    assert all(a > b for a, b in zip(vals, vals[1:]))                     # monotone
    for s in (0, 123, 4999, 25_000, 49_999):                              # symmetry of the cosine
        assert abs(f(base, lo, s, 0, T) + f(base, lo, T - s, 0, T) - (base + lo)) < 1e-15
    # linear warm-up, then the cosine measured from the end of the warm-up
    assert f(base, lo, 0, 100, T) == base / 100 and f(base, lo, 99, 100, T) == base
    assert f(base, lo, 100, 100, T) == base
    for s in range(0, 2 * T, 777):
        for wu in (0, 100):
            assert math.isclose(f(base, lo, s, wu, T), oracle.lr_cosine(base, lo, s, wu, T),
                                rel_tol=1e-13, abs_tol=1e-20)
    for bad in ((-1.0, 0.0, 0, 0, 10), (1.0, 2.0, 0, 0, 10), (1.0, 0.0, -1, 0, 10),
                (1.0, 0.0, 0, -1, 10), (1.0, 0.0, 0, 20, 10), (float("nan"), 0.0, 0, 0, 10)):
        assert math.isnan(f(*bad))


def test_first_and_second_micro_batch_entry_points_validation_and_counter():
    L = B.lib()
    first, second = L.acco_accumulate_first, L.acco_accumulate_second
    c = ctypes.c_int64(7)
    cr = ctypes.byref(c)
    assert first(NONE, vp(Bp), 4, 0, cr, NONE) == B.ACCO_ERR_NULL
    assert first(vp(A), NONE, 4, 0, cr, NONE) == B.ACCO_ERR_NULL
    assert first(vp(A), vp(Bp), -1, 0, cr, NONE) == B.ACCO_ERR_SIZE
    assert first(vp(A), vp(Bp), 4, 2, cr, NONE) == B.ACCO_ERR_ARG
    assert first(vp(A + 2), vp(Bp), 4, 0, cr, NONE) == B.ACCO_ERR_ALIGN
    assert first(vp(A), vp(A + 16), 64, 0, cr, NONE) == B.ACCO_ERR_ALIAS
    assert c.value == 7
    assert first(vp(A), vp(Bp), 0, 0, cr, NONE) == 0 and c.value == 1      # a new accumulation
    # second: exactly one output, and the counter must stand at one
    assert second(NONE, NONE, vp(C), vp(D), 4, cr, NONE) == B.ACCO_ERR_NULL
    assert second(NONE, NONE, NONE, NONE, 0, NONE, NONE) == 0          # an empty shard
    assert second(vp(A), vp(Bp), vp(C), vp(D), 4, cr, NONE) == B.ACCO_ERR_NULL
    assert second(vp(A), NONE, NONE, vp(D), 4, cr, NONE) == B.ACCO_ERR_NULL
    assert second(vp(A), NONE, vp(C), vp(D + 8), 4, cr, NONE) == B.ACCO_ERR_ALIGN
    assert second(vp(A), NONE, vp(A), vp(D), 4, cr, NONE) == B.ACCO_ERR_ALIAS
    assert second(NONE, vp(Bp), vp(C), vp(Bp), 4, cr, NONE) == B.ACCO_ERR_ALIAS
    assert c.value == 1
    assert second(vp(A), NONE, vp(C), vp(D), 0, cr, NONE) == 0 and c.value == 2
    assert second(vp(A), NONE, vp(C), vp(D), 0, cr, NONE) == B.ACCO_ERR_ARG   # not the second
    c.value = 1
    assert second(NONE, vp(Bp), vp(C), vp(D), 0, cr, NONE) == 0 and c.value == 2


def test_bf16_running_sum_entry_point_validation_and_counter():
    f = B.lib().acco_accumulate_bf16
    c = ctypes.c_int64(3)
    cr = ctypes.byref(c)
    assert f(NONE, vp(Bp), 4, 0, cr, NONE) == B.ACCO_ERR_NULL
    assert f(vp(A), NONE, 4, 1, cr, NONE) == B.ACCO_ERR_NULL
    assert f(vp(A), vp(Bp), -2, 0, cr, NONE) == B.ACCO_ERR_SIZE
    assert f(vp(A), vp(Bp), 4, 2, cr, NONE) == B.ACCO_ERR_ARG
    assert f(vp(A + 2), vp(Bp), 4, 0, cr, NONE) == B.ACCO_ERR_ALIGN
    assert f(vp(A), vp(A + 16), 64, 0, cr, NONE) == B.ACCO_ERR_ALIAS
    bad = ctypes.c_int64(-1)
    assert f(vp(A), vp(Bp), 0, 0, ctypes.byref(bad), NONE) == B.ACCO_ERR_ARG and bad.value == -1
    assert c.value == 3
    assert f(NONE, NONE, 0, 0, cr, NONE) == 0 and c.value == 4            # an empty shard still counts
    assert f(vp(A), vp(Bp), 0, 1, cr, NONE) == 0 and c.value == 1         # init starts a new sum


def test_probe_entry_points_validate_like_the_rest():
    L = B.lib()
    assert L.acco_probe_copy(NONE, vp(A), 4, NONE) == B.ACCO_ERR_NULL
    assert L.acco_probe_copy(vp(A), vp(A + 16), 64, NONE) == B.ACCO_ERR_ALIAS
    assert L.acco_probe_copy(vp(A + 4), vp(Bp), 4, NONE) == B.ACCO_ERR_ALIGN
    assert L.acco_probe_copy(vp(A), vp(Bp), 0, NONE) == 0
    assert L.acco_probe_triad(vp(A), vp(Bp), vp(C), NONE, 4, NONE) == B.ACCO_ERR_NULL
    assert L.acco_probe_triad(vp(A), vp(Bp), vp(A), vp(D), 4, NONE) == B.ACCO_ERR_ALIAS
    assert L.acco_probe_triad(vp(A), vp(Bp), vp(C), vp(D), -1, NONE) == B.ACCO_ERR_SIZE
    assert L.acco_probe_triad(vp(A), vp(Bp), vp(C), vp(D), 0, NONE) == 0


def test_accumulate_batch_validation_and_counters():
    L = B.lib()
    f = L.acco_accumulate_batch
    acc = _shards(A, Bp)
    out = _shards(C, D)
    stash = _shards(E, F)
    grad = _shards(0x70000, 0x80000)
    cnt = (ctypes.c_int64 * 2)(5, 7)
    ops = B
    # unknown operation, worker count out of range, bad n
    assert f(9, 2, acc, out, stash, grad, 0, cnt, NONE, NONE) == B.ACCO_ERR_ARG
    assert f(-1, 2, acc, out, stash, grad, 0, cnt, NONE, NONE) == B.ACCO_ERR_ARG
    assert f(ops.BATCH_ACCUMULATE, 0, acc, out, stash, grad, 0, cnt, NONE, NONE) == B.ACCO_ERR_SIZE
    assert f(ops.BATCH_ACCUMULATE, 65, acc, out, stash, grad, 0, cnt, NONE, NONE) == B.ACCO_ERR_SIZE
    assert f(ops.BATCH_ACCUMULATE, 2, acc, out, stash, grad, -1, cnt, NONE, NONE) == B.ACCO_ERR_SIZE
    # a column the operation uses is missing; columns it does not use may be NULL
    assert f(ops.BATCH_ACCUMULATE, 2, NONE, NONE, NONE, grad, 0, cnt, NONE, NONE) == B.ACCO_ERR_NULL
    assert f(ops.BATCH_ACCUMULATE, 2, acc, NONE, NONE, NONE, 0, cnt, NONE, NONE) == B.ACCO_ERR_NULL
    assert f(ops.BATCH_SECOND_PUBLISH, 2, NONE, out, NONE, grad, 0, cnt, NONE, NONE) == B.ACCO_ERR_NULL
    assert f(ops.BATCH_PUBLISH, 2, acc, NONE, NONE, NONE, 0, NONE, NONE, NONE) == B.ACCO_ERR_NULL
    assert f(ops.BATCH_ACCUMULATE, 2, acc, NONE, NONE, _shards(0x70000, 0), 4, NONE, NONE, NONE) == B.ACCO_ERR_NULL
    assert f(ops.BATCH_ACCUMULATE, 2, _shards(A, Bp + 4), NONE, NONE, grad, 0, NONE, NONE, NONE) == B.ACCO_ERR_ALIGN
    # a written buffer meets another buffer of the call: same worker, or another worker's
    assert f(ops.BATCH_ACCUMULATE, 2, _shards(A, A + 16), NONE, NONE, grad, 64, NONE, NONE, NONE) == B.ACCO_ERR_ALIAS
    assert f(ops.BATCH_FIRST, 2, NONE, _shards(C, C), NONE, grad, 8, NONE, NONE, NONE) == B.ACCO_ERR_ALIAS
    assert f(ops.BATCH_FIRST, 2, NONE, _shards(C, 0x70000), NONE, grad, 8, NONE, NONE, NONE) == B.ACCO_ERR_ALIAS
    assert f(ops.BATCH_SECOND, 2, acc, NONE, _shards(E, A), grad, 8, NONE, NONE, NONE) == B.ACCO_ERR_ALIAS
    # read-only buffers may be shared between workers
    assert f(ops.BATCH_FIRST, 2, NONE, out, NONE, _shards(0x70000, 0x70000), 0, NONE, NONE, NONE) == 0
    # counters: errors leave them alone; each operation's rule
    assert (cnt[0], cnt[1]) == (5, 7)
    assert f(ops.BATCH_SECOND, 2, acc, NONE, stash, grad, 0, cnt, NONE, NONE) == B.ACCO_ERR_ARG   # not 1
    assert f(ops.BATCH_ACCUMULATE, 2, acc, NONE, NONE, grad, 0, cnt, NONE, NONE) == 0
    assert (cnt[0], cnt[1]) == (6, 8)
    assert f(ops.BATCH_ACCUMULATE_PUBLISH, 2, acc, out, NONE, grad, 0, cnt, NONE, NONE) == 0
    assert (cnt[0], cnt[1]) == (7, 9)
    assert f(ops.BATCH_RUNNING_BF16, 2, NONE, out, NONE, grad, 0, cnt, NONE, NONE) == 0
    assert (cnt[0], cnt[1]) == (8, 10)
    assert f(ops.BATCH_PUBLISH, 2, acc, out, NONE, NONE, 0, cnt, NONE, NONE) == 0
    assert (cnt[0], cnt[1]) == (8, 10)
    for op in (ops.BATCH_ACCUMULATE_INIT, ops.BATCH_FIRST, ops.BATCH_FIRST_PUBLISH):
        cnt[0], cnt[1] = 3, 4
        assert f(op, 2, acc, out, NONE, grad, 0, cnt, NONE, NONE) == 0 and (cnt[0], cnt[1]) == (1, 1)
    assert f(ops.BATCH_SECOND_PUBLISH, 2, NONE, out, stash, grad, 0, cnt, NONE, NONE) == 0
    assert (cnt[0], cnt[1]) == (2, 2)
    neg = (ctypes.c_int64 * 2)(1, -1)
    assert f(ops.BATCH_ACCUMULATE, 2, acc, NONE, NONE, grad, 0, neg, NONE, NONE) == B.ACCO_ERR_ARG
    # 64 workers (four launches of 16) are accepted
    many = _shards(*[0x100000 + 0x1000 * k for k in range(64)])
    gmany = _shards(*[0x900000 + 0x1000 * k for k in range(64)])
    assert f(ops.BATCH_FIRST, 64, NONE, many, NONE, gmany, 0, NONE, NONE, NONE) == 0


def test_layouts_of_interleaved_communication_buffers():
    """out_layout of acco_accumulate_batch and shard_layout of the reduction entry points: the
    workers' bf16 buffers as the interleaved blocks of one buffer."""
    L = B.lib()
    f = L.acco_accumulate_batch

    def lay(b, st):
        return ctypes.byref(B.Layout(b, st))

    blk, W, n = 64, 2, 1000
    base = 0x4000000
    out = _shards(base, base + 2 * blk)                       # worker w at base + w * blk bf16
    grad = _shards(0x70000, 0x80000)
    stash = _shards(0x90000, 0xA0000)
    acc = _shards(0xB0000, 0xC0000)
    il = lay(blk, W * blk)
    # interleaved outputs overlap in extent but share no element: accepted, with every
    # operation that writes out_bf16 ...
    for op in (B.BATCH_FIRST, B.BATCH_FIRST_PUBLISH, B.BATCH_SECOND_PUBLISH,
               B.BATCH_ACCUMULATE_PUBLISH, B.BATCH_PUBLISH):
        cnt = (ctypes.c_int64 * 2)(1, 1)
        assert f(op, 2, acc, out, stash, grad, 0, cnt, il, NONE) == 0, op
    # ... the same pointers without the layout are overlapping planar buffers
    assert f(B.BATCH_FIRST, 2, NONE, out, NONE, grad, n, NONE, NONE, NONE) == B.ACCO_ERR_ALIAS
    # two workers on the same block slot, or half a block apart, do collide
    assert f(B.BATCH_FIRST, 2, NONE, _shards(base, base), NONE, grad, n, NONE, il, NONE) == B.ACCO_ERR_ALIAS
    assert f(B.BATCH_FIRST, 2, NONE, _shards(base, base + blk), NONE, grad, n, NONE, il, NONE) == \
        B.ACCO_ERR_ALIAS
    # an input inside the interleaved buffer's extent is refused
    assert f(B.BATCH_FIRST, 2, NONE, out, NONE, _shards(0x70000, base + 8 * blk), n, NONE, il,
             NONE) == B.ACCO_ERR_ALIAS
    # no layout where there is no output, nor for the in-place running sum, nor blocks < 8
    assert f(B.BATCH_ACCUMULATE, 2, acc, NONE, NONE, grad, 0, NONE, il, NONE) == B.ACCO_ERR_ARG
    assert f(B.BATCH_RUNNING_BF16, 2, NONE, out, NONE, grad, 0, NONE, il, NONE) == B.ACCO_ERR_ARG
    assert f(B.BATCH_FIRST, 2, NONE, out, NONE, grad, 0, NONE, lay(4, 8), NONE) == B.ACCO_ERR_ARG
    assert f(B.BATCH_FIRST, 2, NONE, out, NONE, grad, 0, NONE, lay(48, 96), NONE) == B.ACCO_ERR_ARG
    assert f(B.BATCH_FIRST, 2, NONE, out, NONE, grad, 0, NONE, lay(blk, blk - 8), NONE) == B.ACCO_ERR_ARG
    assert f(B.BATCH_FIRST, 2, NONE, out, NONE, grad, 0, NONE, lay(0, 0), NONE) == 0     # planar

    # the reduction side
    hp = ctypes.byref(GOOD)
    th, m, v, g, o16 = (0x10000000 * k for k in range(1, 6))
    cnt = (ctypes.c_int64 * 2)(3, 4)
    tot, step = ctypes.c_int64(0), ctypes.c_int64(0)
    tr, sr = ctypes.byref(tot), ctypes.byref(step)
    red, est, com = L.acco_reduce_shards, L.acco_reduce_estimate_step, L.acco_reduce_commit_step
    assert red(vp(g), out, 2, 0, 0, 0, cnt, tr, NONE, il, NONE) == 0
    assert est(vp(th), vp(m), vp(v), vp(g), out, 2, 0, cnt, tr, NONE, vp(o16), 0, hp, 0, NONE, il,
               NONE) == 0
    assert com(vp(th), vp(m), vp(v), vp(g), out, 2, 0, cnt, tr, vp(o16), 0, hp, sr, NONE, il,
               NONE) == 0
    assert tot.value == 14 and step.value == 1      # n = 0 throughout: nothing is launched
    # a blocked layout is for bf16 shards only
    assert red(vp(g), out, 2, 1, 0, 0, cnt, tr, NONE, il, NONE) == B.ACCO_ERR_ARG
    assert est(vp(th), vp(m), vp(v), vp(g), out, 2, 1, cnt, tr, NONE, vp(o16), 0, hp, 0, NONE, il,
               NONE) == B.ACCO_ERR_ARG
    assert com(vp(th), vp(m), vp(v), vp(g), out, 2, 1, cnt, tr, vp(o16), 0, hp, sr, NONE, il,
               NONE) == B.ACCO_ERR_ARG
    # the interleaved buffer's whole extent counts against the state and the outputs
    assert red(vp(base + 64), out, 2, 0, n, 0, cnt, tr, NONE, il, NONE) == B.ACCO_ERR_ALIAS
    assert com(vp(th), vp(m), vp(v), vp(g), out, 2, 0, cnt, tr, vp(base + 16 * blk), n, hp, sr,
               NONE, il, NONE) == B.ACCO_ERR_ALIAS
    assert red(vp(g), out, 2, 0, 0, 0, cnt, tr, NONE, lay(blk, 3), NONE) == B.ACCO_ERR_ARG


def test_folded_scalars_are_the_double_precision_values_rounded_once():
    """acco_fold_adamw against the scalars written out with Python's doubles and exact
    fractions: grad scale, betas, their complements, step size with the first bias correction,
    the second bias correction's reciprocal root, decay, epsilon."""
    import math
    from fractions import Fraction

    import numpy as np
    for lr, b1, b2, eps, wd in ((6e-4, 0.9, 0.95, 1e-8, 0.1), (1e-3, 0.0, 0.999, 1e-6, 0.0),
                                (2e-5, 0.8, 0.9, 0.0, 0.05)):
        hp = B.AdamW(lr, b1, b2, eps, wd)
        for step, count in ((0, 1), (1, 3), (99, 32), (49_999, 7)):
            got = list(B.acco_fold_adamw(hp, step, count).f)
            t = step + 1
            want = [1.0 / count, b1, b2, 1.0 - b1, 1.0 - b2, lr / (1.0 - b1 ** t),
                    1.0 / math.sqrt(1.0 - b2 ** t), lr * wd, eps]
            assert got[:9] == [float(np.float32(x)) for x in want], (hp, step, count)
            assert got[9:] == [0.0] * 7
            # the grad scale is the correctly rounded reciprocal (exact for powers of two)
            assert abs(Fraction(got[0]) - Fraction(1, count)) <= Fraction(got[0]) * Fraction(1, 2 ** 24)
    out = B.StepScalars()
    L = B.lib()
    good = ctypes.byref(GOOD)
    assert L.acco_fold_adamw(good, 0, 1, NONE) == B.ACCO_ERR_NULL
    assert L.acco_fold_adamw(NONE, 0, 1, ctypes.byref(out)) == B.ACCO_ERR_NULL
    assert L.acco_fold_adamw(good, -1, 1, ctypes.byref(out)) == B.ACCO_ERR_ARG
    assert L.acco_fold_adamw(good, 0, 0, ctypes.byref(out)) == B.ACCO_ERR_ARG
    bad = B.AdamW(6e-4, 1.0, 0.95, 1e-8, 0.1)
    assert L.acco_fold_adamw(ctypes.byref(bad), 0, 1, ctypes.byref(out)) == B.ACCO_ERR_ARG
    assert ctypes.sizeof(B.StepScalars) == 64


def test_device_scalar_entry_points_validation():
    L = B.lib()
    S = 0x90000                                    # the scalar block's "device" address
    G = 0x70000
    src = (B.StepScalars * 4)()
    stage = L.acco_stage_scalars
    assert stage(NONE, src, 1, NONE) == B.ACCO_ERR_NULL
    assert stage(vp(S), NONE, 1, NONE) == B.ACCO_ERR_NULL
    assert stage(vp(S), src, 0, NONE) == B.ACCO_ERR_SIZE
    assert stage(vp(S), src, B.STAGE_BLOCKS_MAX + 1, NONE) == B.ACCO_ERR_SIZE
    assert stage(vp(S + 8), src, 1, NONE) == B.ACCO_ERR_ALIGN

    e, c = L.acco_estimate_step_dev, L.acco_commit_step_dev
    assert e(vp(A), vp(Bp), vp(C), vp(D), vp(E), 0, NONE, NONE, NONE) == B.ACCO_ERR_NULL
    assert e(vp(A), vp(Bp), vp(C), vp(D), NONE, 4, vp(S), NONE, NONE) == B.ACCO_ERR_NULL
    assert e(NONE, vp(Bp), vp(C), vp(D), vp(E), 4, vp(S), NONE, NONE) == B.ACCO_ERR_NULL
    assert e(vp(A), vp(Bp), vp(C), vp(D), vp(E), -1, vp(S), NONE, NONE) == B.ACCO_ERR_SIZE
    assert e(vp(A), vp(Bp), vp(C), vp(D), vp(E), 0, vp(S + 4), NONE, NONE) == B.ACCO_ERR_ALIGN
    assert e(vp(A), vp(Bp), vp(C), vp(D), vp(A), 8, vp(S), NONE, NONE) == B.ACCO_ERR_ALIAS
    assert e(vp(A), vp(Bp), vp(C), vp(D), vp(E), 64, vp(E + 32), NONE, NONE) == B.ACCO_ERR_ALIAS
    assert e(vp(A), vp(Bp), vp(C), vp(D), vp(E), 0, vp(S), NONE, NONE) == 0
    assert c(vp(A), vp(Bp), vp(C), vp(D), NONE, 0, NONE, NONE, NONE) == B.ACCO_ERR_NULL
    assert c(vp(A), vp(Bp), vp(C), NONE, NONE, 4, vp(S), NONE, NONE) == B.ACCO_ERR_NULL
    assert c(vp(A), vp(A), vp(C), vp(D), NONE, 4, vp(S), NONE, NONE) == B.ACCO_ERR_ALIAS
    # the scalar block may not lie inside anything the step writes; gsum is only read
    for k, written in enumerate((A, Bp, C)):
        assert c(vp(A), vp(Bp), vp(C), vp(D), NONE, 64, vp(written + 64), NONE, NONE) == B.ACCO_ERR_ALIAS, k
    assert c(vp(A), vp(Bp), vp(C), vp(D), vp(E), 64, vp(E + 16), NONE, NONE) == B.ACCO_ERR_ALIAS
    assert c(vp(A), vp(Bp), vp(C), vp(D), vp(E), 0, vp(S), NONE, NONE) == 0

    s2 = _shards(E, F)
    re_, rc_ = L.acco_reduce_estimate_step_dev, L.acco_reduce_commit_step_dev
    assert re_(vp(A), vp(Bp), vp(C), vp(D), NONE, 2, 0, vp(G), 0, vp(S), NONE, NONE, NONE) == B.ACCO_ERR_NULL
    assert re_(vp(A), vp(Bp), vp(C), vp(D), s2, 2, 0, NONE, 4, vp(S), NONE, NONE, NONE) == B.ACCO_ERR_NULL
    assert re_(vp(A), vp(Bp), vp(C), vp(D), s2, 2, 0, vp(G), 0, NONE, NONE, NONE, NONE) == B.ACCO_ERR_NULL
    assert re_(vp(A), vp(Bp), vp(C), vp(D), s2, 65, 0, vp(G), 0, vp(S), NONE, NONE, NONE) == B.ACCO_ERR_SIZE
    assert re_(vp(A), vp(Bp), vp(C), vp(D), s2, 2, 7, vp(G), 0, vp(S), NONE, NONE, NONE) == B.ACCO_ERR_ARG
    assert re_(vp(A), vp(Bp), vp(C), vp(D), _shards(E, D), 2, 0, vp(G), 8, vp(S), NONE, NONE, NONE) == B.ACCO_ERR_ALIAS
    assert re_(vp(A), vp(Bp), vp(C), vp(D), s2, 2, 0, vp(G), 64, vp(D + 16), NONE, NONE, NONE) == B.ACCO_ERR_ALIAS   # gsum is written
    assert re_(vp(A), vp(Bp), vp(C), vp(D), s2, 2, 0, vp(G), 0, vp(S), NONE, NONE, NONE) == 0
    assert rc_(vp(A), vp(Bp), vp(C), vp(D), NONE, 2, 0, vp(G), 0, vp(S), NONE, NONE, NONE) == B.ACCO_ERR_NULL
    assert rc_(vp(A), vp(Bp), vp(C), vp(D), s2, 2, 0, vp(G), 0, vp(S + 2), NONE, NONE, NONE) == B.ACCO_ERR_ALIGN
    assert rc_(vp(A), vp(Bp), vp(C), vp(D), s2, 2, 0, vp(E), 8, vp(S), NONE, NONE, NONE) == B.ACCO_ERR_ALIAS
    assert rc_(vp(A), vp(Bp), vp(C), vp(D), s2, 2, 0, vp(G), 64, vp(Bp + 128), NONE, NONE, NONE) == B.ACCO_ERR_ALIAS
    lay = B.Layout(8, 32)
    assert rc_(vp(A), vp(A + 32), vp(A + 64), vp(A + 96), s2, 2, 0, vp(G), 0, vp(S), ctypes.byref(lay), NONE, NONE) == 0
    assert rc_(vp(A), vp(Bp), vp(C), vp(D), s2, 2, 0, NONE, 0, vp(S), NONE, NONE, NONE) == 0


def test_resident_commit_step_validation():
    L = B.lib()
    r = L.acco_commit_step_resident
    sc = B.acco_fold_adamw(GOOD, 0, 1)
    ref = ctypes.byref(sc)
    assert r(vp(A), vp(Bp), vp(C), vp(D), NONE, 0, NONE, 0, NONE, NONE) == B.ACCO_ERR_NULL
    assert r(vp(A), vp(Bp), vp(C), NONE, NONE, 4, ref, 0, NONE, NONE) == B.ACCO_ERR_NULL
    assert r(vp(A), vp(Bp), vp(C), vp(D), NONE, -1, ref, 0, NONE, NONE) == B.ACCO_ERR_SIZE
    for slot in (-1, B.RESIDENT_SLOTS, 2 ** 31 - 1):
        assert r(vp(A), vp(Bp), vp(C), vp(D), NONE, 0, ref, slot, NONE, NONE) == B.ACCO_ERR_SIZE
    assert "slot" in B.status_string(B.ACCO_ERR_SIZE)
    assert r(vp(A + 4), vp(Bp), vp(C), vp(D), NONE, 0, ref, 0, NONE, NONE) == B.ACCO_ERR_ALIGN
    assert r(vp(A), vp(A), vp(C), vp(D), NONE, 4, ref, 0, NONE, NONE) == B.ACCO_ERR_ALIAS
    assert r(vp(A), vp(Bp), vp(C), vp(D), vp(A), 4, ref, 0, NONE, NONE) == B.ACCO_ERR_ALIAS
    bad = B.Layout(6, 24)
    assert r(vp(A), vp(Bp), vp(C), vp(D), NONE, 0, ref, 0, ctypes.byref(bad), NONE) == B.ACCO_ERR_ARG
    for slot in (0, B.RESIDENT_SLOTS - 1):
        assert r(vp(A), vp(Bp), vp(C), vp(D), vp(E), 0, ref, slot, NONE, NONE) == 0
    assert B.RESIDENT_SLOTS == 64


def test_header_is_plain_c_and_the_library_is_callable_from_c(tmp_path):
    """include/acco.h as a strict C99 (and C++17) translation unit, and a C program linked
    against libacco.so that walks one round's host bookkeeping with n == 0."""
    import subprocess
    from paper_2406_02613_amd import build
    inc = os.path.join(ROOT, "include")
    src = os.path.join(ROOT, "tests", "c", "abi_from_c.c")
    libdir = os.path.dirname(build.ACCO_SO)
    exe = str(tmp_path / "abi_from_c")
    rocm = "/opt/rocm/lib"
    subprocess.run(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", inc, src,
                    "-o", exe, "-L", libdir, "-lacco", f"-Wl,-rpath,{libdir}",
                    f"-Wl,-rpath-link,{rocm}", f"-Wl,-rpath,{rocm}"], check=True)
    out = subprocess.run([exe], capture_output=True, text=True, timeout=60)
    assert out.returncode == 0, out.stderr
    assert "acco C ABI ok" in out.stdout
    cpp = tmp_path / "hdr.cpp"
    cpp.write_text('#include "acco.h"\nint main() { return acco_version() > 0 ? 0 : 1; }\n')
    subprocess.run(["g++", "-std=c++17", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", inc,
                    "-fsyntax-only", str(cpp)], check=True)


def test_memory_class_probe_validation():
    L = B.lib()
    c = L.acco_hbm_classify
    out = (ctypes.c_int32 * 8)()
    ncls = ctypes.c_int32(-1)
    o, nr = out, ctypes.byref(ncls)
    MiB = 1 << 20
    S = 0x7f0000000000                                   # scratch well away from the region
    assert c(NONE, 64 * MiB, 8 * MiB, 8 * MiB, vp(S), o, 8, nr, NONE) == B.ACCO_ERR_NULL
    assert c(vp(A), 64 * MiB, 8 * MiB, 8 * MiB, NONE, o, 8, nr, NONE) == B.ACCO_ERR_NULL
    assert c(vp(A), 64 * MiB, 8 * MiB, 8 * MiB, vp(S), None, 8, nr, NONE) == B.ACCO_ERR_NULL
    assert c(vp(A), 64 * MiB, 8 * MiB, 8 * MiB, vp(S), o, 8, None, NONE) == B.ACCO_ERR_NULL
    assert c(vp(A + 4), 64 * MiB, 8 * MiB, 8 * MiB, vp(S), o, 8, nr, NONE) == B.ACCO_ERR_ALIGN
    assert c(vp(A), 64 * MiB, 8 * MiB + 1, 8 * MiB, vp(S), o, 8, nr, NONE) == B.ACCO_ERR_SIZE
    assert c(vp(A), 64 * MiB, 8 * MiB, 100, vp(S), o, 8, nr, NONE) == B.ACCO_ERR_SIZE
    assert c(vp(A), 4 * MiB, 8 * MiB, 8 * MiB, vp(S), o, 1, nr, NONE) == B.ACCO_ERR_SIZE   # region < probe
    assert c(vp(A), 64 * MiB, 8 * MiB, 8 * MiB, vp(S), o, 7, nr, NONE) == B.ACCO_ERR_SIZE  # count is 8
    assert c(vp(A), 64 * MiB, 8 * MiB, 8 * MiB, vp(A + 16 * MiB), o, 8, nr, NONE) == B.ACCO_ERR_ALIAS
    assert ncls.value == -1


def test_arena_bookkeeping_on_a_given_classification():
    from paper_2406_02613_amd.arena import ALIGN, HbmArena, plan_roles
    GiB = 1 << 30
    # 12 GiB, a position per GiB, probes of 512 MiB: classes 0 0 0 1 1 0 0 2 2 2 2 2
    cls = [0, 0, 0, 1, 1, 0, 0, 2, 2, 2, 2, 2]
    a = HbmArena(12 * GiB, step_bytes=GiB, probe_bytes=GiB // 2, classes=cls)
    assert a.n_classes == 3
    H = GiB // 4                                          # half a probe: the guard at a boundary
    assert [(c, s, e) for c, s, e, _ in a.runs] == [
        (0, 0, 2 * GiB + H), (1, 3 * GiB + H, 4 * GiB + H), (0, 5 * GiB + H, 6 * GiB + H),
        (2, 7 * GiB + H, 12 * GiB)]
    assert a.free_bytes() == {0: 3 * GiB + H, 1: GiB, 2: 5 * GiB - H}
    off, c = a.take(GiB + 5, 0)
    assert (off, c) == (0, 0)
    off, c = a.take(GiB, 0)
    assert (off, c) == (GiB + ALIGN, 0)                   # hand-outs start on 2 MiB boundaries
    off, c = a.take(GiB, 0)                               # does not fit the rest of run 0: next run of class 0
    assert (off, c) == (5 * GiB + H, 0)
    off, c = a.take(GiB, 0)                               # class 0 has no stretch of 1 GiB left: spills
    assert c == 2 and off == 7 * GiB + H
    with pytest.raises(MemoryError):
        a.take(GiB, 0, spill=False)
    with pytest.raises(MemoryError):
        a.take(6 * GiB, 1)
    with pytest.raises(RuntimeError):
        a.alloc(16, None, 0)
    # roles: the bigger reader gets the class with more room, the outputs a third class
    b = HbmArena(12 * GiB, step_bytes=GiB, probe_bytes=GiB // 2, classes=cls)
    plan = plan_roles(b, {"owner": 2 * GiB, "compute": 3 * GiB})
    assert plan == {"compute": 2, "owner": 0, "out": 1}
    one = HbmArena(4 * GiB, step_bytes=GiB, probe_bytes=GiB // 2, classes=[0, 0, 0, 0])
    assert plan_roles(one, {"owner": 1, "compute": 2}) == {"compute": 0, "owner": 0, "out": 0}
    assert plan_roles(None, {}) == {}
    with pytest.raises(ValueError):
        HbmArena(4 * GiB, step_bytes=GiB, probe_bytes=GiB // 2, classes=[0, 0])

"""Randomly drawn configurations of the whole path (shard length, worker count, launch shape,
bound on resident wavefronts, state layout, communication dtype, hyper-parameters, update index,
micro-batch counts, which fused entry points are used, whether the first gradient is adopted in
place, whether the workers' accumulation steps share launches, whether the communication
buffers are interleaved, whether the step kernels take their scalars by value or from device
memory) against the oracle's binary32 form: two
rounds each, every output compared bit for bit."""
import numpy as np
import pytest

import oracle
from parity import adam_state, bf16_tensor, bit_mismatches, bits_of

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

ENTRIES = ["accumulate", "cast", "reduce", "estimate", "commit", "accumulate_publish",
           "reduce_estimate", "reduce_commit", "stash", "second"]


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_random_configurations_are_bit_exact(seed):
    import paper_2406_02613_amd as A
    rng = np.random.default_rng(1000 + seed)
    sizes = [0, 1, 3, 5, 63, 64, 65, 255, 257, 1023, 4099, 70_001, 262_144 + 5, 1 << 20]
    shapes = [(64, 1, 0), (64, 1, 0), (128, 1, 0), (256, 2, 0), (512, 4, 0), (256, 4, 2),
              (128, 2, 1), (64, 2, 3)]
    try:
        for it in range(40):
            n = int(rng.choice(sizes))
            W = int(rng.choice([1, 2, 3, 7, 8, 9, 17]))
            shape = shapes[rng.integers(0, len(shapes))]
            bound = int(rng.choice([0, 0, 3, 8, 9, 12, 24, 32]))
            for e in ENTRIES:
                A.set_resident_waves(e, 0)
                A.set_launch_shape(e, *shape)
                if bound and bound // (shape[0] // 64) >= 3:
                    A.set_resident_waves(e, bound)
            blocked, block = bool(rng.integers(0, 2)), int(rng.choice([4, 64, 1024, 8192]))
            f32comm = bool(rng.integers(0, 4) == 0)
            hyper = (float(rng.choice([0.0, 2e-5, 6e-4, 1e-2])), float(rng.choice([0.0, 0.9, 0.99])),
                     float(rng.choice([0.5, 0.95, 0.999])), float(rng.choice([1e-8, 1e-6, 1e-3])),
                     float(rng.choice([0.0, 0.01, 0.1, 0.3])))
            step0 = int(rng.choice([0, 1, 7, 99, 4999]))
            ks = [[int(rng.integers(1, 5)) for _ in range(W)] for _ in range(2)]
            stash, fp, fr, adopt, batched = (bool(rng.integers(0, 2)) for _ in range(5))
            b16acc = (not f32comm) and rng.integers(0, 5) == 0
            ilv = (not b16acc) and bool(rng.integers(0, 2))
            cblk = int(rng.choice([8, 64, 4096, 16384]))
            devsc = bool(np.random.default_rng(77 * seed + it).integers(0, 2))   # its own stream
            print(f"seed {seed} case {it}: n={n} W={W} shape={shape} bound={bound} "
                  f"blocked={blocked}/{block} f32comm={f32comm} hyper={hyper} step0={step0} "
                  f"stash={stash} adopt={adopt} publish={fp} reduce={fr} bf16acc={b16acc} "
                  f"batched={batched} interleaved_comm={ilv}/{cblk} device_scalars={devsc}", flush=True)
            # every other case starts from a state no run of Adam need have produced (m and v
            # unrelated, |m|/sqrt(v) up to 1e3, zero and denormal v); all comparisons below are
            # bit for bit with the binary32 form, so no tolerance is involved
            theta, m, v, _ = adam_state(rng, n, "wide" if it % 2 else "warm")
            own = A.ShardOwner(n, W, A.make_hyper(*hyper), comm_bf16=not f32comm, fused_publish=fp,
                               fused_reduce=fr, blocked_state=blocked, block_elems=block,
                               bf16_stash=stash, bf16_accumulate=bool(b16acc), adopt_first=adopt,
                               batched=batched, interleaved_comm=ilv, comm_block_elems=cblk,
                               device_scalars=devsc)
            for name, x in (("theta", theta), ("m", m), ("v", v)):
                own.set_state(name, torch.from_numpy(x.copy()).cuda())
            own.step.value = step0
            ref = oracle.OracleShard(theta, W, oracle.make_hyper(*hyper), m=m, v=v, step=step0,
                                     precision="f32", comm_dtype="f32" if f32comm else "bf16",
                                     acc_dtype="bf16" if b16acc else "f32")
            for _ in range(2):
                for stage in (0, 1):
                    rows = []
                    for w in range(W):
                        row = []
                        for k in range(ks[stage][w]):
                            g = oracle.cast((rng.standard_normal(n) * 1e-3).astype(np.float32))
                            row.append(bf16_tensor(g))
                            ref.add_microbatch(w, g)
                        rows.append(row)
                    own.add_microbatch_rows(rows)
                    if stage == 0:
                        own.stage1()
                        ref.stage1()
                        assert np.array_equal(bits_of(own.theta_tilde_bf16), ref.theta_tilde_bf16)
                    else:
                        own.stage2()
                        ref.stage2()
                        assert np.array_equal(bits_of(own.theta_bf16), ref.theta_bf16)
                    assert own.step.value == ref.step
                for name in ("theta", "m", "v"):
                    assert bit_mismatches(own.get_state(name).cpu().numpy(), getattr(ref, name)) == 0
    finally:
        A.reset_launch_settings()

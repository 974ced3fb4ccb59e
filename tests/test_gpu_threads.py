"""Two host threads drive two shard owners at once, each on a stream of its own: the library keeps
no state between calls, so the rounds must come out as if each owner had run alone - bit for bit
the oracle's rounds."""
import threading

import numpy as np
import pytest

import synth
from parity import OracleSlices, bit_mismatches, bits_of

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _drive(A, w, options, rounds, out, errors):
    try:
        torch.cuda.set_device(0)
        stream = torch.cuda.Stream()                 # default priority
        with torch.cuda.stream(stream):
            h = w.hyper
            owner = A.ShardOwner(w.n, w.workers,
                                 A.make_hyper(h.lr, h.beta1, h.beta2, h.eps, h.weight_decay),
                                 **options)
            tmp = torch.empty(w.n, dtype=torch.float32, device="cuda")
            w.device_theta(tmp)
            owner.set_state("theta", tmp)
            for r in range(rounds):
                for stage in (synth.STAGE_TILDE, synth.STAGE_FULL):
                    rows = []
                    for wk, c in enumerate(w.stage_counts(r, stage)):
                        row = []
                        for mb in range(c):
                            g = torch.empty(w.n, dtype=torch.bfloat16, device="cuda")
                            synth.device_grad_bf16(g, w.grad_spec(r, stage, wk, mb), 0)
                            row.append(g)
                        rows.append(row)
                    owner.add_microbatch_rows(rows)
                    owner.stage1() if stage == synth.STAGE_TILDE else owner.stage2()
            stream.synchronize()
            out["theta"] = owner.get_state("theta").cpu().numpy()
            out["m"] = owner.get_state("m").cpu().numpy()
            out["v"] = owner.get_state("v").cpu().numpy()
            out["theta_bf16"] = bits_of(owner.theta_bf16)
            out["theta_tilde_bf16"] = bits_of(owner.theta_tilde_bf16)
            out["step"] = owner.step.value
    except Exception as e:                            # surfaced by the main thread
        errors.append(e)


def test_two_threads_on_two_streams_do_not_disturb_each_other():
    import paper_2406_02613_amd as A
    A.binding.lib()
    rounds = 3
    jobs = [
        (synth.Workload(name="ta", n=400_037, workers=3, rounds=rounds, grad_std=1e-3,
                        k_range=(2, 5), seed=21),
         dict(fused_publish=True, fused_reduce=True, blocked_state=True, bf16_stash=True,
              batched=True)),
        (synth.Workload(name="tb", n=250_001, workers=4, rounds=rounds, grad_std=1e-4, k_fixed=4,
                        seed=22),
         dict(device_scalars=True, fused_reduce=True)),
    ]
    outs, errors = [{}, {}], []
    threads = [threading.Thread(target=_drive, args=(A, w, opt, rounds, outs[k], errors))
               for k, (w, opt) in enumerate(jobs)]
    for t in threads:
        t.start()
    for t in threads:
        t.join(timeout=100)
        assert not t.is_alive(), "a driver thread did not finish"
    assert not errors, errors
    for (w, _), got in zip(jobs, outs):
        print("threads: checking", w.name, flush=True)
        ref = OracleSlices(w, [(0, w.n)], "f32")
        for r in range(rounds):
            ref.run_stage(r, synth.STAGE_TILDE)
            ref.run_stage(r, synth.STAGE_FULL)
        sh = ref.shards[0]
        assert got["step"] == sh.step == rounds
        for name in ("theta", "m", "v"):
            assert bit_mismatches(got[name], getattr(sh, name)) == 0, (w.name, name)
        for name in ("theta_bf16", "theta_tilde_bf16"):
            assert np.array_equal(got[name], getattr(sh, name)), (w.name, name)

"""The two-stream scheduler of Alg. 1 on one GPU: whatever number of micro-batches each stage
ends up accumulating, the result equals the oracle replaying the same counts."""
import numpy as np
import pytest

import oracle
import synth
from parity import bit_mismatches, bits_of

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def replay(w, theta0, hp, peers_bits, peer_counts, log):
    """Oracle: the same rounds with the realised per-stage micro-batch counts of worker 0."""
    n = theta0.size
    theta, m, v = theta0.copy(), np.zeros(n, np.float32), np.zeros(n, np.float32)
    gsum = np.zeros(n, np.float32)
    step = 0
    # micro-batches accumulated for (round, acc): acc 1 of round t is consumed in round t+1
    counts = {(-1, 1): 1}
    for rec in log.stages:
        other = 2 if rec.stage == 1 else 1
        counts[(rec.round, other)] = rec.microbatches
    last_bf16 = None
    for rec in log.stages:
        src_round = rec.round - 1 if rec.stage == 1 else rec.round
        k = counts[(src_round, rec.stage)]
        acc = np.zeros(n, np.float32)
        for j in range(k):
            oracle.accumulate(acc, synth.host_grad_bf16(spec(w, src_round, rec.stage, j), 0, n),
                              init=(j == 0))
        shards = [oracle.cast(acc), *peers_bits]
        total_here = k + sum(peer_counts)
        if rec.stage == 1:
            oracle.reduce(gsum, shards, accumulate_=False)
            total = total_here
            _, last_bf16 = oracle.estimate(theta, m, v, gsum, hp, step + 1, total, want_f32=False,
                                           precision="f32")
        else:
            oracle.reduce(gsum, shards, accumulate_=True)
            total += total_here
            last_bf16 = oracle.commit(theta, m, v, gsum, hp, step + 1, total, precision="f32")
            step += 1
        assert rec.total_count == total
    return theta, m, v, step, last_bf16


def spec(w, rnd, acc, k):
    return w.grad_spec(rnd + 1, acc, 0, k)          # round -1 is the initialisation gradient


@pytest.mark.parametrize("blocked,placed", [(True, False), (False, False), (True, True)])
def test_two_stream_rounds_equal_the_oracle_replay(blocked, placed):
    import paper_2406_02613_amd as A
    w = synth.Workload(name="ts", n=400_000 + 37, workers=3, rounds=4, grad_std=1e-3, seed=17)
    h = w.hyper
    # placed: every buffer from an arena, by memory class (placement changes no bit)
    arena = A.HbmArena(2 << 30, step_bytes=512 << 20, probe_bytes=256 << 20) if placed else None
    own = A.TwoStreamOwner(w.n, w.workers, A.make_hyper(h.lr, h.beta1, h.beta2, h.eps,
                                                        h.weight_decay), blocked_state=blocked,
                           arena=arena)
    th0 = w.host_theta(0, w.n)
    own.set_theta(torch.from_numpy(th0).cuda())
    peer_counts = [2, 3]
    peers_bits = [synth.host_grad_bf16(w.grad_spec(0, 1, wk, 0), 0, w.n) for wk in (1, 2)]
    peers = []
    for wk, b in zip((1, 2), peers_bits):
        p = own.new_peer_buffer(wk)
        p.copy_(torch.from_numpy(b.view(np.int16).copy()).view(torch.bfloat16))
        peers.append(p)
    buf = own.new_buffer("compute", w.n, torch.bfloat16)

    def grad_source(rnd, acc, k):
        synth.device_grad_bf16(buf, spec(w, rnd, acc, k), 0)     # runs on the computation stream
        return buf

    plan = lambda rnd, acc: 1 + (3 * rnd + acc) % 4            # planned accumulation steps
    log = own.run(w.rounds, grad_source, peers, peer_counts, min_microbatches=plan)
    assert len(log.stages) == 2 * w.rounds and own.step.value == w.rounds
    for rec in log.stages:
        other = 2 if rec.stage == 1 else 1
        assert rec.microbatches >= plan(rec.round, other)
        print("round", rec.round, "stage", rec.stage, "accumulated", rec.microbatches,
              "total", rec.total_count, f"comm {rec.comm_ms:.3f} ms comp {rec.comp_ms:.3f} ms",
              flush=True)
    theta, m, v, step, last = replay(w, th0, oracle.make_hyper(h.lr, h.beta1, h.beta2, h.eps,
                                                               h.weight_decay),
                                     peers_bits, peer_counts, log)
    assert step == w.rounds
    assert bit_mismatches(own.get_state("theta").cpu().numpy(), theta) == 0
    assert bit_mismatches(own.get_state("m").cpu().numpy(), m) == 0
    assert bit_mismatches(own.get_state("v").cpu().numpy(), v) == 0
    assert np.array_equal(bits_of(own.params_bf16), last)

"""The entry points are plain kernel launches with their scalars passed by value, so a stage
whose scalars do not change (the speculative stage: same update index, same counts) can be
recorded into a HIP graph and replayed on new gradient contents.  Host-side counters are
updated when the calls are recorded, not when the graph is replayed."""
import numpy as np
import pytest

import oracle
from parity import bf16_tensor, bits_of

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def test_speculative_stage_recorded_in_a_graph_replays_like_eager_calls():
    import paper_2406_02613_amd as A
    B = A.binding
    n, W, step = 300_037, 3, 5
    rng = np.random.default_rng(77)
    hp = A.make_hyper(6e-4, 0.9, 0.95, 1e-8, 0.1)
    ohp = oracle.make_hyper(6e-4, 0.9, 0.95, 1e-8, 0.1)
    theta_h = (rng.standard_normal(n) * 0.02).astype(np.float32)
    m_h = (rng.standard_normal(n) * 1e-4).astype(np.float32)
    v_h = (rng.standard_normal(n) ** 2 * 1e-8).astype(np.float32)
    theta, m, v = (torch.from_numpy(x).cuda() for x in (theta_h, m_h, v_h))
    before = [t.clone() for t in (theta, m, v)]

    def buffers():
        return dict(stash=[torch.empty(n, dtype=torch.bfloat16, device="cuda") for _ in range(W)],
                    comm=[torch.empty(n, dtype=torch.bfloat16, device="cuda") for _ in range(W)],
                    gsum=torch.empty(n, dtype=torch.float32, device="cuda"),
                    out=torch.empty(n, dtype=torch.bfloat16, device="cuda"))

    grads = [[torch.zeros(n, dtype=torch.bfloat16, device="cuda") for _ in range(2)]
             for _ in range(W)]

    def stage(buf, total):
        for w in range(W):
            B.acco_accumulate_first(buf["stash"][w], grads[w][0], False, A.Counter(0))
            B.acco_accumulate_second(buf["stash"][w], grads[w][1], comm_bf16=buf["comm"][w])
        B.acco_reduce_estimate_step(theta, m, v, buf["gsum"], buf["comm"], [2] * W, total, hp,
                                    step, theta_tilde_bf16=buf["out"], n=n)

    captured, eager = buffers(), buffers()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # a first run outside any capture
        stage(captured, A.Counter(0))
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    graph = torch.cuda.CUDAGraph()
    total = A.Counter(0)
    with torch.cuda.graph(graph):
        stage(captured, total)
    assert total.value == 2 * W                        # bookkeeping happened at record time

    for replay in range(4):
        print("graph replay", replay, flush=True)
        host = [[oracle.cast((rng.standard_normal(n) * 1e-3).astype(np.float32)) for _ in range(2)]
                for _ in range(W)]
        for w in range(W):
            for k in range(2):
                grads[w][k].copy_(bf16_tensor(host[w][k]))          # eager work between replays
        captured["out"].zero_()
        captured["gsum"].zero_()
        graph.replay()
        stage(eager, A.Counter(0))
        torch.cuda.synchronize()
        assert torch.equal(captured["out"].view(torch.int16), eager["out"].view(torch.int16))
        assert torch.equal(captured["gsum"].view(torch.int32), eager["gsum"].view(torch.int32))
        # and against the oracle
        acc = [np.empty(n, np.float32) for _ in range(W)]
        for w in range(W):
            oracle.accumulate(acc[w], host[w][0], init=True)
            oracle.accumulate(acc[w], host[w][1], init=False)
        gsum_h = np.empty(n, np.float32)
        oracle.reduce(gsum_h, [oracle.cast(a) for a in acc], accumulate_=False)
        _, want = oracle.estimate(theta_h, m_h, v_h, gsum_h, ohp, step + 1, 2 * W, want_f32=False,
                                  precision="f32")
        assert np.array_equal(bits_of(captured["out"]), want)
        assert np.array_equal(captured["gsum"].cpu().numpy().view(np.uint32), gsum_h.view(np.uint32))
    for t, b in zip((theta, m, v), before):            # the speculative stage commits nothing
        assert torch.equal(t.view(torch.int32), b.view(torch.int32))


def test_batched_accumulation_launches_replay_from_a_graph():
    """acco_accumulate_batch passes its pointer table by value: a recorded launch keeps working on
    the same buffers with new contents, like the single calls."""
    import paper_2406_02613_amd as A
    B = A.binding
    n, W = 70_001, 5
    rng = np.random.default_rng(78)
    grads = [[torch.zeros(n, dtype=torch.bfloat16, device="cuda") for _ in range(W)] for _ in range(2)]
    stash = [torch.empty(n, dtype=torch.bfloat16, device="cuda") for _ in range(W)]
    comm = [torch.empty(n, dtype=torch.bfloat16, device="cuda") for _ in range(W)]

    def stage():
        B.acco_accumulate_batch(B.BATCH_FIRST, n, out_bf16=stash, grad_bf16=grads[0])
        B.acco_accumulate_batch(B.BATCH_SECOND_PUBLISH, n, out_bf16=comm, stash_bf16=stash,
                                grad_bf16=grads[1])

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        stage()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        stage()
    for replay in range(3):
        print("batched graph replay", replay, flush=True)
        host = [[oracle.cast((rng.standard_normal(n) * 1e-3).astype(np.float32)) for _ in range(W)]
                for _ in range(2)]
        for k in range(2):
            for w in range(W):
                grads[k][w].copy_(bf16_tensor(host[k][w]))              # eager work between replays
        for c in comm:
            c.zero_()
        graph.replay()
        torch.cuda.synchronize()
        for w in range(W):
            acc = np.empty(n, np.float32)
            oracle.accumulate(acc, host[0][w], init=True)
            oracle.accumulate(acc, host[1][w], init=False)
            assert np.array_equal(bits_of(comm[w]), oracle.cast(acc)), (replay, w)

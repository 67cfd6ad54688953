"""A decode step captured once in a HIP graph and replayed: the bit-widths live in device memory,
so one graph has to serve every pattern (Sec. 4.4 / Alg. 1: the precision changes from token to
token).  Every replay is checked against the same calls issued directly, with the program's own
work and synchronizations between the replays."""
import numpy as np
import pytest
import torch

import synth
import paper_2506_12024_amd as fq
from gpu_util import DEV, make_layer, to_dev
from test_gpu_stream import _build

pytestmark = pytest.mark.gpu

V = 4099


def _capture(fn):
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        fn()  # once outside the capture: nothing in the graph is a first call
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            fn()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    return graph


def test_token_loop_graph_matches_direct_calls():
    # linears at M = 1 -> entropy of the token's logits -> scheduler step, which rewrites the
    # bit-width array that the next replay's linears read
    shapes = [(1000, 512), (1536, 1024), (2048, 640), (777, 2048), (4096, 1152), (300, 128), (2500, 896), (1024, 4096)]
    n, T, window = len(shapes), 36, 4
    layers, xs = [], []
    for i, (N, K) in enumerate(shapes):
        w = synth.weight(0, "graph/w%d" % i, N, K, 0.02, outlier_p=0.001)
        layers.append(make_layer(w, (4, 8, 16))[0])
        xs.append(to_dev(synth.activations(0, "graph/x%d" % i, 1, K)))
    base = synth.normal_f32(0, "graph/logits", V, 1.0)
    logits = to_dev((base[None, :] * (2.0 + 3.0 * np.arange(T, dtype=np.float32) / T)[:, None]).astype(np.float32))
    ev_entry = torch.tensor([5, 2, 7, 0, 3, 6, 1, 4, 2, 5], dtype=torch.int32, device=DEV)
    ev_bits = torch.tensor([8, 8, 8, 8, 4, 4, 4, 4, 4, 4], dtype=torch.int32, device=DEV)

    class Side:
        def __init__(self):
            self.ys = [torch.full((1, N), float("nan"), dtype=torch.float16, device=DEV) for N, _ in shapes]
            self.ws = torch.empty(fq.Plan.workspace_bytes(n), dtype=torch.uint8, device=DEV)
            self.plan = fq.Plan(layers, xs, self.ys, 1, self.ws)
            self.bits = torch.full((n,), 16, dtype=torch.int32, device=DEV)
            self.ev_token = torch.full((10,), -1, dtype=torch.int32, device=DEV)
            self.state = torch.zeros(fq.fq_sched_state_bytes(window), dtype=torch.uint8, device=DEV)
            self.cur = torch.zeros(V, dtype=torch.float32, device=DEV)
            self.H = torch.zeros(1, dtype=torch.float32, device=DEV)

        def reset(self):
            self.bits.fill_(16)
            self.ev_token.fill_(-1)
            # a threshold above every PPLE: the scheduler fires whenever its wait is over
            fq.fq_sched_init(self.state, window, 1e30, 2, ev_entry, ev_bits, 10, self.bits, self.ev_token)

        def token(self):
            self.plan.run(self.bits)
            fq.fq_entropy_kl(self.cur, None, 1, V, self.H, None)
            fq.fq_sched_step(self.state, self.H)

    direct, replayed = Side(), Side()
    direct.reset()
    replayed.reset()
    graph = _capture(replayed.token)
    replayed.reset()  # the capture's warm-up call advanced the scheduler
    seen = set()
    for t in range(T):
        for s in (direct, replayed):
            s.cur.copy_(logits[t])
            for y in s.ys:
                y.fill_(float("nan"))
        seen.add(tuple(direct.bits.cpu().tolist()))
        direct.token()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(direct.bits, replayed.bits), t
        assert torch.equal(direct.H, replayed.H), t
        for i in range(n):
            assert torch.equal(direct.ys[i].view(torch.int16), replayed.ys[i].view(torch.int16)), (t, i)
            assert torch.isfinite(direct.ys[i].float()).all(), (t, i)
    assert torch.equal(direct.ev_token, replayed.ev_token)
    assert len(seen) >= 5  # the replays really ran under different patterns
    assert fq.fq_sched_peek(direct.state) == fq.fq_sched_peek(replayed.state)


@pytest.mark.parametrize("widths", [(4, 8, 16), (2, 4, 8, 16)])
def test_streaming_plan_graph_replays(widths):
    # the batched streaming kernel hands out its tiles from a queue in the plan's workspace and
    # leaves it zeroed: replays need no memset node and follow each other directly (with 2-bit
    # copies a launch is three kernels: the entry lists, the streaming kernel, the 2-bit pass)
    M = 16
    shapes, layers, packs, xs_np, xs, ys, plan = _build(
        M, "graph/stream", lambda i, N, K: synth.weight(0, "graph/stream/w%d" % i, N, K, 0.02), widths=widths)
    n = len(layers)
    bits = torch.zeros(n, dtype=torch.int32, device=DEV)
    k = len(widths)
    patterns = [[widths[(i + s) % k] for i in range(n)] for s in range(3)] + [[widths[0]] * n,
                                                                              [0 if i % 2 else 16 for i in range(n)]]
    expect = []
    for p in patterns:
        bits.copy_(torch.tensor(p, dtype=torch.int32))
        for y in ys:
            y.fill_(3.0)
        plan.run(bits)
        torch.cuda.synchronize()
        expect.append([y.clone() for y in ys])
    graph = _capture(lambda: plan.run(bits))
    for rep in range(2):
        for p, want in zip(patterns, expect):
            bits.copy_(torch.tensor(p, dtype=torch.int32))
            for y in ys:
                y.fill_(3.0)
            graph.replay()
            if rep:
                graph.replay()  # twice in a row, nothing in between
            torch.cuda.synchronize()
            for i in range(n):
                assert torch.equal(ys[i].view(torch.int16), want[i].view(torch.int16)), (rep, i, p[i])

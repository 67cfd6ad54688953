"""The stage-ordered plan (one persistent launch for a decode step in dependent order) against the
same stages run as separate launches of stage-ordered plans -- bit for bit: a stage is cut into
workgroup and wavefront shares the same way whether it runs alone or after others --, against the
one-launch plan and fq_linear (same item arithmetic, but a row whose K is shared by two wavefronts
is summed in a different order: compared at the output tolerance) and against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import synth
import paper_2506_12024_amd as fq
import bench
from gpu_util import DEV, make_layer, rel_err, to_dev

pytestmark = pytest.mark.gpu

TOL_Y = 2e-3


def _close(a, b):
    """Two fp16 results of the same linear from kernels that sum in different orders."""
    a, b = a.float(), b.float()
    return float((a - b).abs().max()) <= TOL_Y * float(b.abs().max())


def _staged(layers, xs, ys, stage):
    ws = torch.empty(fq.StagedPlan.workspace_bytes(len(layers), max(stage) + 1), dtype=torch.uint8, device=DEV)
    return fq.StagedPlan(layers, xs, ys, stage, 1, ws)


def test_independent_stages_match_separate_plans_and_oracle():
    # ragged shapes, every bit-width, stages of one to three entries
    shapes = [(100, 1408), (37, 128), (530, 5120), (4096, 4096), (16, 11008), (1000, 2048), (64, 13824),
              (3, 256), (2048, 1024)]
    stage = [0, 0, 0, 1, 2, 2, 3, 3, 4]
    bits = [4, 8, 16, 2, 8, 4, 4, 16, 8]
    layers, xs, refs = [], [], []
    for i, ((N, K), b) in enumerate(zip(shapes, bits)):
        w = synth.weight(3, "stg/ind/w%d" % i, N, K, 0.02, outlier_p=0.001)
        x = synth.activations(3, "stg/ind/x%d" % i, 1, K)
        layer, packed = make_layer(w, (2, 4, 8, 16))
        if b == 16:
            refs.append(oracle.linear(x, w, None, None, 16))
        else:
            c, s, z = (t.cpu().numpy() for t in packed[b])
            refs.append(oracle.linear(x, c, s, z, b))
        layers.append(layer)
        xs.append(to_dev(x))
    bits_dev = torch.tensor(bits, dtype=torch.int32, device=DEV)
    ys = [torch.full((1, l.N), float("nan"), dtype=torch.float16, device=DEV) for l in layers]
    ys_sep = [torch.full((1, l.N), float("nan"), dtype=torch.float16, device=DEV) for l in layers]
    plan = _staged(layers, xs, ys, stage)
    plan.run(bits_dev)
    for s in sorted(set(stage)):
        idx = [i for i, v in enumerate(stage) if v == s]
        sep = _staged([layers[i] for i in idx], [xs[i] for i in idx], [ys_sep[i] for i in idx], [0] * len(idx))
        sep.run(bits_dev[idx[0]:idx[-1] + 1])
    torch.cuda.synchronize()
    assert plan.status() == (0, 0)
    for i, (a, b, r) in enumerate(zip(ys, ys_sep, refs)):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16)), i
        assert rel_err(a.cpu().numpy(), r) <= TOL_Y, i


def test_chained_stages_read_what_the_previous_stage_wrote():
    # x of stage s + 1 IS y of stage s (same buffer); the first input changes on every replay, so a
    # stage that read a stale copy of its input from a cache would be found out
    n, D = 7, 1024
    rng = np.random.default_rng(11)
    bits = [int(b) for b in rng.choice([4, 8, 16], size=n)]
    layers, packs, ws_host = [], [], []
    for i in range(n):
        w = synth.weight(4, "stg/chain/w%d" % i, D, D, 0.03)
        layer, packed = make_layer(w, (4, 8, 16))
        layers.append(layer)
        packs.append(packed)
        ws_host.append(w)
    bufs = [torch.zeros((1, D), dtype=torch.float16, device=DEV) for _ in range(n + 1)]
    plan = _staged(layers, bufs[:-1], bufs[1:], list(range(n)))
    bits_dev = torch.tensor(bits, dtype=torch.int32, device=DEV)
    seq = [torch.zeros((1, D), dtype=torch.float16, device=DEV) for _ in range(n + 1)]
    singles = [_staged([layers[i]], [seq[i]], [seq[i + 1]], [0]) for i in range(n)]
    for rep in range(6):
        x0 = synth.activations(4, "stg/chain/x/%d" % rep, 1, D)
        bufs[0].copy_(to_dev(x0))
        seq[0].copy_(to_dev(x0))
        plan.run(bits_dev)
        for i in range(n):
            singles[i].run(bits_dev[i:i + 1])       # the same stage, a launch of its own
        torch.cuda.synchronize()
        for i in range(1, n + 1):
            assert torch.equal(bufs[i].view(torch.int16), seq[i].view(torch.int16)), (rep, i)
        # the oracle on the chain: every stage from the GPU's own input to it
        for i in (0, n - 1):
            xin = bufs[i].cpu().numpy()
            if bits[i] == 16:
                r = oracle.linear(xin, ws_host[i], None, None, 16)
            else:
                c, s, z = (t.cpu().numpy() for t in packs[i][bits[i]])
                r = oracle.linear(xin, c, s, z, bits[i])
            assert rel_err(bufs[i + 1].cpu().numpy(), r) <= TOL_Y, (rep, i)
    assert plan.status() == (0, 0)


def test_llama7b_step_in_dependent_order_matches_the_single_plan():
    # the benchmark's stack, four stages per decoder layer (q/k/v, o, gate/up, down), changing
    # bit patterns; against the one-launch plan over the same entries, and twice for determinism
    st = bench.Stack("llama7b", M=1, bit_choices=(4, 8))
    st.build_staged_plan()
    ys_single = [y.clone() for y in st.ys]
    for step in (0, 5, 77):
        for y in st.ys:
            y.fill_(float("nan"))
        st.run_linears(step)
        torch.cuda.synchronize()
        ys_single = [y.clone() for y in st.ys]
        for y in st.ys:
            y.fill_(float("nan"))
        st.run_linears_one_launch_staged(step)
        torch.cuda.synchronize()
        first = [y.clone() for y in st.ys]
        for e, (a, b) in enumerate(zip(st.ys, ys_single)):
            assert torch.isfinite(a.float()).all() and _close(a, b), (step, e)
        st.run_linears_one_launch_staged(step)
        torch.cuda.synchronize()
        for e, (a, b) in enumerate(zip(st.ys, first)):
            assert torch.equal(a.view(torch.int16), b.view(torch.int16)), (step, e)
    assert st.staged_plan.status() == (0, 0)


def test_wait_that_runs_out_returns_and_the_next_launch_is_whole():
    # forced from the host: no polls allowed, so a workgroup that finds the others not yet arrived
    # gives up at once; every kernel still returns, and with the limit restored the plan works
    n, D = 5, 2048
    layers, ws_host = [], []
    for i in range(n):
        w = synth.weight(5, "stg/gu/w%d" % i, D, D, 0.02)
        layer, _ = make_layer(w, (8,))
        layers.append(layer)
    bufs = [torch.zeros((1, D), dtype=torch.float16, device=DEV) for _ in range(n + 1)]
    bufs[0].copy_(to_dev(synth.activations(5, "stg/gu/x", 1, D)))
    plan = _staged(layers, bufs[:-1], bufs[1:], list(range(n)))
    bits_dev = torch.full((n,), 8, dtype=torch.int32, device=DEV)
    plan.set_wait_limit(0)
    for _ in range(3):
        plan.run(bits_dev)
    torch.cuda.synchronize()
    gave_up, flags = plan.status()
    assert 0 <= gave_up <= 3 and flags == 0
    plan.set_wait_limit(1 << 21)
    plan.run(bits_dev)
    torch.cuda.synchronize()
    assert plan.status()[0] == gave_up
    for i in range(n):                                   # every stage from the plan's own input to it
        y = torch.zeros((1, D), dtype=torch.float16, device=DEV)
        fq.fq_linear(layers[i], 8, bufs[i], 1, y)
        torch.cuda.synchronize()
        assert _close(bufs[i + 1], y), i


def test_unattached_width_is_reported_and_skipped():
    w = synth.weight(6, "stg/un/w", 256, 512, 0.02)
    layer, _ = make_layer(w, (8,))
    x = to_dev(synth.activations(6, "stg/un/x", 1, 512))
    ys = [torch.full((1, 256), 7.0, dtype=torch.float16, device=DEV) for _ in range(2)]
    plan = _staged([layer, layer], [x, x], ys, [0, 1])
    plan.run(torch.tensor([8, 4], dtype=torch.int32, device=DEV))   # no 4-bit copy attached
    torch.cuda.synchronize()
    assert plan.status() == (0, 1)
    assert torch.all(ys[1] == 7.0) and not torch.all(ys[0] == 7.0)


def test_staged_plan_in_a_hip_graph_under_changing_bits():
    n, D = 6, 1024
    layers = []
    for i in range(n):
        w = synth.weight(7, "stg/graph/w%d" % i, D, D, 0.03)
        layer, _ = make_layer(w, (4, 8))
        layers.append(layer)
    bufs = [torch.zeros((1, D), dtype=torch.float16, device=DEV) for _ in range(n + 1)]
    bufs[0].copy_(to_dev(synth.activations(7, "stg/graph/x", 1, D)))
    plan = _staged(layers, bufs[:-1], bufs[1:], list(range(n)))
    bits_dev = torch.full((n,), 8, dtype=torch.int32, device=DEV)
    plan.run(bits_dev)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            plan.run(bits_dev)
    torch.cuda.synchronize()
    rng = np.random.default_rng(2)
    for rep in range(5):
        pat = rng.choice([4, 8], size=n).astype(np.int32)
        bits_dev.copy_(torch.from_numpy(pat).to(DEV))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        got = [b.clone() for b in bufs]
        plan.run(bits_dev)                               # the same launch issued directly
        torch.cuda.synchronize()
        for i in range(1, n + 1):
            assert torch.equal(got[i].view(torch.int16), bufs[i].view(torch.int16)), (rep, i)
        for i in range(n):
            y = torch.zeros((1, D), dtype=torch.float16, device=DEV)
            fq.fq_linear(layers[i], int(pat[i]), bufs[i], 1, y)
            torch.cuda.synchronize()
            assert _close(bufs[i + 1], y), (rep, i)
    assert plan.status() == (0, 0)

"""fq_linears_static, the entry point that allocates nothing, against fq_plan_create + fq_plan_run
on the same inputs: the two run the same kernels over the same descriptor table, so the outputs must
agree bit for bit; each is also held to the oracle's bar.  Two calls in a row share the library's
static device array, the second with a smaller input."""
import numpy as np
import pytest
import torch

import oracle
import synth
import paper_2506_12024_amd as fq
from gpu_util import DEV, make_layer, rel_err, to_dev

pytestmark = pytest.mark.gpu

TOL_Y = 2e-3


def _case(tag, shapes, M, bit_choices, seed):
    layers, xs, refs = [], [], []
    rng = np.random.default_rng(seed)
    bits = rng.choice(bit_choices, size=len(shapes)).astype(np.int32)
    for i, (N, K) in enumerate(shapes):
        w = synth.weight(seed, "%s/w%d" % (tag, i), N, K, 0.02, outlier_p=0.001)
        x = synth.activations(seed, "%s/x%d" % (tag, i), M, K)
        layer, packed = make_layer(w, tuple(bit_choices))
        b = int(bits[i])
        if b == 16:
            y_ref = oracle.linear(x, w, None, None, 16)
        else:
            c, s, z = (t.cpu().numpy() for t in packed[b])
            y_ref = oracle.linear(x, c, s, z, b)
        layers.append(layer)
        xs.append(to_dev(x))
        refs.append(y_ref)
    return layers, xs, refs, torch.from_numpy(bits).to(DEV)


def _run_both(layers, xs, refs, bits_dev, M):
    ys_plan = [torch.full((M, l.N), float("nan"), dtype=torch.float16, device=DEV) for l in layers]
    ys_stat = [torch.full((M, l.N), float("nan"), dtype=torch.float16, device=DEV) for l in layers]
    ws = torch.empty(fq.Plan.workspace_bytes(len(layers)), dtype=torch.uint8, device=DEV)
    plan = fq.Plan(layers, xs, ys_plan, M, ws)
    plan.run(bits_dev)
    fq.fq_linears_static(layers, xs, ys_stat, M, bits_dev)
    torch.cuda.synchronize()
    for i, (a, b, r) in enumerate(zip(ys_plan, ys_stat, refs)):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16)), i
        assert rel_err(b.cpu().numpy(), r) <= TOL_Y, i


@pytest.mark.parametrize("M", [1, 16])
def test_static_entry_point_matches_plan_twice_in_a_row(M):
    # first call: 70 entries (three batches of descriptors) -- 120 at M = 16, enough 256-row tiles
    # there for the streaming kernel and its queue; second call: 3 small entries, which leaves most
    # of the first call's table behind in the static array
    big = [(4096, 1024), (2048, 2048), (1000, 1408), (4096, 512), (512, 4096)] * (14 if M == 1 else 24)
    small = [(300, 1024), (64, 2048), (1000, 512)]
    for tag, shapes, seed in (("noalloc/big/M%d" % M, big, 1), ("noalloc/small/M%d" % M, small, 2)):
        layers, xs, refs, bits_dev = _case(tag, shapes, M, (4, 8, 16), seed)
        _run_both(layers, xs, refs, bits_dev, M)


def test_static_entry_point_rejects_what_it_cannot_hold():
    w = synth.weight(0, "noalloc/rej/w", 64, 256, 0.02)
    layer, _ = make_layer(w, (8,))
    x = to_dev(synth.activations(0, "noalloc/rej/x", 1, 256))
    y = torch.zeros((1, 64), dtype=torch.float16, device=DEV)
    n = fq.FQ_STATIC_MAX_ENTRIES + 1
    bits = torch.full((n,), 8, dtype=torch.int32, device=DEV)
    with pytest.raises(fq.FlexqError) as ei:
        fq.fq_linears_static([layer] * n, [x] * n, [y] * n, 1, bits)
    assert ei.value.code == -3 and "FQ_STATIC_MAX_ENTRIES" in str(ei.value)

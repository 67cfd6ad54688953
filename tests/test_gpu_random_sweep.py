"""Seeded random sweep of shapes, batch sizes and bit-widths through fq_linear, one-launch plans and
stage-ordered plans, each output compared with the CPU oracle (Sec. 2.2 Eq. (3); Sec. 4.1, 4.3:
any resident width may be selected per call): the fixed parity cases pick their shapes by hand,
this one does not.  Row counts around the tile sizes, K from one group to beyond a 70B FFN width
fraction, batches on both sides of every dispatch boundary (1 | 2 .. 32 | above)."""
import numpy as np
import pytest
import torch

import oracle
import synth
import paper_2506_12024_amd as fq
from gpu_util import DEV, gpu_linear, make_layer, rel_err, to_dev

pytestmark = pytest.mark.gpu

TOL_Y = 2e-3
NS_ = [1, 3, 16, 17, 63, 64, 65, 100, 255, 256, 257, 1000, 2049]
KS_ = [1, 2, 3, 5, 8, 11, 16, 17, 32, 33, 43, 64, 86, 108]
MS_ = [1, 1, 1, 2, 3, 4, 7, 8, 16, 17, 31, 32, 33, 48, 100]


def _ref(x, w, packed, b):
    if b == 16:
        return oracle.linear(x, w, None, None, 16)
    c, s, z = (t.cpu().numpy() for t in packed[b])
    return oracle.linear(x, c, s, z, b)


@pytest.mark.parametrize("seed", [1, 2, 3, 4])
def test_random_single_calls(seed):
    rng = np.random.default_rng(seed)
    for it in range(24):
        N, K, M = int(rng.choice(NS_)), 128 * int(rng.choice(KS_)), int(rng.choice(MS_))
        b = int(rng.choice([2, 3, 4, 8, 16]))
        w = synth.weight(5, "sweep/w/%d/%d/%d/%d" % (seed, it, N, K), N, K, 0.02, outlier_p=0.002)
        x = synth.activations(5, "sweep/x/%d/%d" % (seed, it), M, K)
        layer, packed = make_layer(w, (b,))
        y = gpu_linear(layer, b, x)
        assert not np.isnan(y.astype(np.float32)).any(), (M, N, K, b)
        assert rel_err(y, _ref(x, w, packed, b)) <= TOL_Y, (M, N, K, b)


@pytest.mark.parametrize("seed", [5, 6, 7, 8])
def test_random_plans(seed):
    rng = np.random.default_rng(seed)
    for it in range(5):
        n = int(rng.integers(1, 9))
        M = int(rng.choice([1, 1, 2, 4, 16, 32]))
        widths = (2, 3, 4, 8, 16) if rng.random() < 0.6 else (2, 4, 8, 16)
        layers, xs, ys, xs_np, packs, bits = [], [], [], [], [], []
        for i in range(n):
            N = int(rng.choice([1, 5, 40, 64, 100, 300, 1024, 2050]))
            K = 128 * int(rng.choice([1, 2, 4, 11, 32, 40, 86]))
            w = synth.weight(6, "sweep/pw/%d/%d/%d" % (seed, it, i), N, K, 0.02, outlier_p=0.002)
            x = synth.activations(6, "sweep/px/%d/%d/%d" % (seed, it, i), M, K)
            layer, packed = make_layer(w, widths)
            layers.append(layer), packs.append((w, packed)), xs_np.append(x), xs.append(to_dev(x))
            ys.append(torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV))
            bits.append(int(rng.choice(widths)))
        ws = torch.empty(fq.Plan.workspace_bytes(n), dtype=torch.uint8, device=DEV)
        plan = fq.Plan(layers, xs, ys, M, ws)
        bits_dev = torch.tensor(bits, dtype=torch.int32, device=DEV)
        plan.run(bits_dev)
        torch.cuda.synchronize()
        assert plan.status() == (0, 0)
        refs = [_ref(xs_np[i], packs[i][0], packs[i][1], bits[i]) for i in range(n)]
        for i in range(n):
            assert rel_err(ys[i].cpu().numpy(), refs[i]) <= TOL_Y, ("plan", M, layers[i].N, layers[i].K, bits[i])
        if M != 1:
            continue
        stage = [0]  # stages rise by at most one from entry to entry
        for _ in range(n - 1):
            stage.append(stage[-1] + int(rng.integers(0, 2)))
        ys2 = [torch.full((1, l.N), float("nan"), dtype=torch.float16, device=DEV) for l in layers]
        ws2 = torch.empty(fq.StagedPlan.workspace_bytes(n, stage[-1] + 1), dtype=torch.uint8, device=DEV)
        staged = fq.StagedPlan(layers, xs, ys2, stage, 1, ws2)
        staged.run(bits_dev)
        torch.cuda.synchronize()
        assert staged.status() == (0, 0)
        for i in range(n):
            assert rel_err(ys2[i].cpu().numpy(), refs[i]) <= TOL_Y, ("staged", stage[i], layers[i].N, layers[i].K, bits[i])

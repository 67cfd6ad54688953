"""GPU parity of the packed 3-bit path (Table 1 / Sec. 5.1 run 3-bit models; Sec. 2.2 Eq. (2), (3)
with n = 3; the packing is this library's, blocks of 12 bytes) against the CPU oracle: codes,
scales and zero points bit-exact, decode outputs at M = 1 (single calls, one-launch plans and
stage-ordered plans that mix 2 / 3 / 4 / 8 / 16 bits per entry), in batches of 2 to 32 rows (single
calls and plans) and above (slabs of 32 rows) within 2e-3 max-abs normalised."""
import numpy as np
import pytest
import torch

import oracle
import synth
import paper_2506_12024_amd as fq
from gpu_util import DEV, gpu_linear, gpu_quantize, make_layer, rel_err, to_dev

pytestmark = pytest.mark.gpu

TOL_Y = 2e-3


@pytest.mark.parametrize("sym", [False, True])
@pytest.mark.parametrize("shape,outl", [((4096, 4096), 0.001), ((48, 1408), 0.01), ((1, 128), 0.0), ((333, 11008), 0.0)])
def test_quantize_3bit_bit_exact(shape, outl, sym):
    N, K = shape
    w = synth.weight(0, "par3/q/%dx%d" % shape, N, K, 0.02, outlier_p=outl)
    c_ref, s_ref, z_ref = (oracle.quantize_sym if sym else oracle.quantize)(w, 3)
    sizes = fq.fq_packed_sizes(N, K, 3)
    assert sizes == (N * K * 3 // 8, N * (K // 128) * 4, N * (K // 128))
    c = torch.full((sizes[0],), 0xAA, dtype=torch.uint8, device=DEV)
    s = torch.empty((N, K // 128), dtype=torch.float32, device=DEV)
    z = torch.empty((N, K // 128), dtype=torch.uint8, device=DEV)
    (fq.fq_quantize_sym if sym else fq.fq_quantize)(to_dev(w), N, K, 3, 128, c, s, z)
    torch.cuda.synchronize()
    assert np.array_equal(c.cpu().numpy().reshape(N, K * 3 // 8), c_ref)
    assert np.array_equal(s.cpu().numpy().view(np.uint32), s_ref.view(np.uint32))
    assert np.array_equal(z.cpu().numpy(), z_ref)


def test_quantize_3bit_degenerate_groups():
    w = np.zeros((3, 512), dtype=np.float16)
    w[0, 128:256] = np.linspace(0.01, 2.0, 128)             # all positive
    w[0, 256:384] = -np.linspace(0.01, 2.0, 128)            # all negative
    w[1, :8] = (np.arange(8) - 3) / 64.0                     # on-grid
    w[1, 8:11] = [0.5 / 64, 1.5 / 64, -0.5 / 64]             # ties
    w[2, 0], w[2, 1] = 65504.0, -65504.0
    w[2, 2:128] = np.linspace(-3e4, 3e4, 126)
    c_ref, s_ref, z_ref = oracle.quantize(w, 3)
    c, s, z = gpu_quantize(to_dev(w), 3)
    assert np.array_equal(c.cpu().numpy(), c_ref)
    assert np.array_equal(s.cpu().numpy().view(np.uint32), s_ref.view(np.uint32))
    assert np.array_equal(z.cpu().numpy(), z_ref)


# K: one slice of 2048 exactly, less than one, several with a ragged last one, a single group
@pytest.mark.parametrize("N,K", [(4096, 4096), (100, 1408), (37, 128), (16, 11008), (530, 5120), (64, 2048),
                                 (21, 13824), (9, 28672)])
def test_linear_3bit_m1_matches_oracle(N, K):
    w = synth.weight(0, "par3/lin/%dx%d" % (N, K), N, K, 0.02, outlier_p=0.001)
    x = synth.activations(0, "par3/lin/x/%d" % K, 1, K)
    layer, packed = make_layer(w, (3,))
    y = gpu_linear(layer, 3, x)
    c, s, z = (t.cpu().numpy() for t in packed[3])
    y_ref = oracle.linear(x, c, s, z, 3)
    assert not np.isnan(y.astype(np.float32)).any()
    assert rel_err(y, y_ref) <= TOL_Y


def test_linear_3bit_integer_case_exact():
    # codes equal to the integer weights (s = 1, z = 0), integer x: every product, every partial sum
    # and the offsets that the kernel adds and removes (by bit position, for the low pairs and for
    # the high bits) are integers below 2^24, so the output must be the integer matrix-vector
    # product exactly; every position k % 32 of a block carries its own pattern, so a swapped
    # pair, or a high bit taken from the wrong code, shows
    rng = np.random.default_rng(7)
    N, K = 48, 4096 + 384
    w = rng.integers(0, 8, size=(N, K))
    w[:, 0::128] = 0
    w[:, 1::128] = 7
    x = (rng.integers(-2, 3, size=(1, K)) * (rng.random((1, K)) < 0.25)).astype(np.float16)
    layer, packed = make_layer(w.astype(np.float16), (3,))
    assert torch.all(packed[3][1] == 1.0) and torch.all(packed[3][2] == 0)
    y = gpu_linear(layer, 3, x)
    expect = x.astype(np.float64) @ w.T.astype(np.float64)
    assert np.abs(expect).max() < 2048
    assert np.array_equal(y.astype(np.float64), expect)
    # one-hot x: output n is the code at that k, for every position of a 32-code block and beyond
    for k in list(range(2, 34)) + [63, 64, 2047, 2048, 4095, 4096, K - 1]:
        x1 = np.zeros((1, K), dtype=np.float16)
        x1[0, k] = 1
        assert np.array_equal(gpu_linear(layer, 3, x1)[0].astype(np.int64), w[:, k]), k


# batches of the small-batch kernels (one and two batch tiles; K: a single group, an odd number of
# groups, several chunks of x with a ragged last one; N: ragged tiles) and, above 32 rows and past
# the longest row the decode kernels take, the same kernel in slabs of 32 batch rows
@pytest.mark.parametrize("N,K,M", [(4096, 4096, 16), (100, 1408, 2), (37, 128, 5), (530, 5120, 17), (64, 11008, 32),
                                   (200, 384, 8), (2000, 2048, 4), (16, 13824, 3), (300, 1024, 40),
                                   (256, 4096, 100), (130, 2432, 33), (48, 32768 + 128, 1), (48, 32768 + 128, 3)])
def test_linear_3bit_batched_matches_oracle(N, K, M):
    w = synth.weight(0, "par3/blin/%dx%d" % (N, K), N, K, 0.02, outlier_p=0.001)
    x = synth.activations(0, "par3/blin/x/%dx%d" % (M, K), M, K)
    layer, packed = make_layer(w, (3,))
    y = gpu_linear(layer, 3, x)
    c, s, z = (t.cpu().numpy() for t in packed[3])
    y_ref = oracle.linear(x, c, s, z, 3)
    assert not np.isnan(y.astype(np.float32)).any()
    assert rel_err(y, y_ref) <= TOL_Y


@pytest.mark.parametrize("M", [2, 16, 21, 37])
def test_linear_3bit_batched_integer_case_exact(M):
    # as at M = 1: integer codes (s = 1, z = 0) and small integer x make every product and partial
    # sum an integer below 2^24, so the batched kernels must return the integer matrix product
    # exactly; one-hot rows of x read every position of a 32-code block back
    rng = np.random.default_rng(11 + M)
    N, K = 80, 1024 + 384
    w = rng.integers(0, 8, size=(N, K))
    w[:, 0::128] = 0
    w[:, 1::128] = 7
    x = (rng.integers(-2, 3, size=(M, K)) * (rng.random((M, K)) < 0.25)).astype(np.float16)
    layer, packed = make_layer(w.astype(np.float16), (3,))
    assert torch.all(packed[3][1] == 1.0) and torch.all(packed[3][2] == 0)
    y = gpu_linear(layer, 3, x)
    expect = x.astype(np.float64) @ w.T.astype(np.float64)
    assert np.abs(expect).max() < 2048
    assert np.array_equal(y.astype(np.float64), expect)
    ks = list(range(0, 34)) + [63, 64, 127, 128, 1023, 1024, K - 1]
    for k0 in range(0, len(ks), M):
        part = ks[k0:k0 + M]
        x1 = np.zeros((M, K), dtype=np.float16)
        for m, k in enumerate(part):
            x1[m, k] = 1
        y1 = gpu_linear(layer, 3, x1)
        for m, k in enumerate(part):
            assert np.array_equal(y1[m].astype(np.int64), w[:, k]), k


def _refs(xs_np, packs, pattern):
    out = []
    for i, b in enumerate(pattern):
        w, packed = packs[i]
        if b == 16:
            out.append(oracle.linear(xs_np[i], w, None, None, 16))
        else:
            c, s, z = (t.cpu().numpy() for t in packed[b])
            out.append(oracle.linear(xs_np[i], c, s, z, b))
    return out


def test_plans_with_3bit_entries_match_individual_calls_and_oracle():
    shapes = [(256, 1024), (100, 1408), (512, 4096), (64, 11008), (40, 128), (300, 4096)]
    layers, xs, ys, ys2, xs_np, packs = [], [], [], [], [], []
    for i, (N, K) in enumerate(shapes):
        w = synth.weight(0, "par3/plan/w%d" % i, N, K, 0.02, outlier_p=0.001)
        layer, packed = make_layer(w, (2, 3, 4, 8, 16) if i % 2 == 0 else (3, 8))
        x = synth.activations(0, "par3/plan/x%d" % i, 1, K)
        layers.append(layer)
        packs.append((w, packed))
        xs_np.append(x)
        xs.append(to_dev(x))
        ys.append(torch.zeros((1, N), dtype=torch.float16, device=DEV))
        ys2.append(torch.zeros((1, N), dtype=torch.float16, device=DEV))
    ws = torch.empty(fq.Plan.workspace_bytes(len(layers)), dtype=torch.uint8, device=DEV)
    plan = fq.Plan(layers, xs, ys, 1, ws)
    stage = [0, 0, 1, 1, 1, 2]
    ws2 = torch.empty(fq.StagedPlan.workspace_bytes(len(layers), 3), dtype=torch.uint8, device=DEV)
    staged = fq.StagedPlan(layers, xs, ys2, stage, 1, ws2)
    for trial, pattern in enumerate([[3, 3, 3, 3, 3, 3], [3, 8, 4, 3, 16, 8], [16, 3, 2, 8, 3, 3], [2, 8, 3, 3, 4, 3]]):
        for y in ys + ys2:
            y.fill_(float("nan"))
        bits_dev = torch.tensor(pattern, dtype=torch.int32, device=DEV)
        plan.run(bits_dev)
        staged.run(bits_dev)
        torch.cuda.synchronize()
        assert staged.status() == (0, 0)
        for i, (b, y_ref) in enumerate(zip(pattern, _refs(xs_np, packs, pattern))):
            y = ys[i].cpu().numpy()
            assert rel_err(y, y_ref) <= TOL_Y, (trial, i, b)
            assert np.array_equal(y.view(np.uint16), gpu_linear(layers[i], b, xs_np[i]).view(np.uint16)), (trial, i, b)
            assert rel_err(ys2[i].cpu().numpy(), y_ref) <= TOL_Y, ("staged", trial, i, b)


@pytest.mark.parametrize("M,widths", [(4, (3, 4, 8, 16)), (4, (2, 3, 4, 8, 16)), (20, (3, 4, 8, 16)), (16, (2, 3, 8))])
def test_batched_plans_with_3bit_entries(M, widths):
    # small plans: the kernel whose wavefronts split K (no layer holds a 2-bit copy) or the
    # register-fed kernel in 64-row tiles; within tolerance of the oracle under patterns that move
    # the 3-bit entries around
    shapes = [(256, 1024), (100, 1408), (512, 4096), (64, 11008), (40, 128), (300, 4096)]
    layers, xs, ys, xs_np, packs = [], [], [], [], []
    for i, (N, K) in enumerate(shapes):
        w = synth.weight(0, "par3/bplan/w%d" % i, N, K, 0.02, outlier_p=0.001)
        layer, packed = make_layer(w, widths)
        x = synth.activations(0, "par3/bplan/x%d/%d" % (i, M), M, K)
        layers.append(layer)
        packs.append((w, packed))
        xs_np.append(x)
        xs.append(to_dev(x))
        ys.append(torch.zeros((M, N), dtype=torch.float16, device=DEV))
    ws = torch.empty(fq.Plan.workspace_bytes(len(layers)), dtype=torch.uint8, device=DEV)
    plan = fq.Plan(layers, xs, ys, M, ws)
    rng = np.random.default_rng(M)
    patterns = [[3] * len(shapes)] + [[int(b) for b in rng.choice(widths, size=len(shapes))] for _ in range(3)]
    for trial, pattern in enumerate(patterns):
        for y in ys:
            y.fill_(float("nan"))
        plan.run(torch.tensor(pattern, dtype=torch.int32, device=DEV))
        torch.cuda.synchronize()
        assert plan.status()[1] == 0
        for i, (b, y_ref) in enumerate(zip(pattern, _refs(xs_np, packs, pattern))):
            assert rel_err(ys[i].cpu().numpy(), y_ref) <= TOL_Y, (trial, i, b)


def test_plan_of_layers_that_hold_only_a_3bit_copy():
    N, K = 200, 2432
    w = synth.weight(0, "par3/only/w", N, K, 0.02)
    x = synth.activations(0, "par3/only/x", 1, K)
    layer, packed = make_layer(w, (3,))
    y = torch.full((1, N), float("nan"), dtype=torch.float16, device=DEV)
    ws = torch.empty(fq.Plan.workspace_bytes(1), dtype=torch.uint8, device=DEV)
    plan = fq.Plan([layer], [to_dev(x)], [y], 1, ws)
    plan.run(torch.tensor([3], dtype=torch.int32, device=DEV))
    torch.cuda.synchronize()
    c, s, z = (t.cpu().numpy() for t in packed[3])
    assert rel_err(y.cpu().numpy(), oracle.linear(x, c, s, z, 3)) <= TOL_Y

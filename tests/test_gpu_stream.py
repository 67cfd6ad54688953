"""Parity of the streaming small-batch kernel (2 <= M <= 32, plans with at least a thousand
256-row tiles) with the CPU oracle, element by element.  The plan below is the smallest that
takes that path: many linears of modest K, whose shapes cover a single quantization group
(half a 128-byte line at 4 bits), odd and even group counts, a last chunk of x that is not full,
and row counts that end inside a tile and inside an MFMA row tile."""
import numpy as np
import pytest
import torch

import oracle
import synth
import paper_2506_12024_amd as fq
from gpu_util import DEV, make_layer, rel_err, to_dev

pytestmark = pytest.mark.gpu

TOL_Y = 2e-3
NS = [6656, 6600, 4100, 7000, 5000]
KS = [128, 384, 640, 1152, 256]
MIN_ROWS = 1024 * 256  # what the dispatcher asks for before it uses 256-row tiles


# rows longer than one block of scales (32 units): two and three whole blocks, a block and one
# unit, one and a half, and a chunk count that is odd (the last pair of chunks is a single one)
LONG = [(600, 8192), (300, 12288), (520, 4224), (700, 6144), (280, 4608), (300, 28672), (270, 32768)]


def _build(M, tag, weight_fn, extra=(), widths=(4, 8, 16)):
    shapes, rows, i = list(extra), sum(n for n, _ in extra), 0
    while rows < MIN_ROWS + 256:
        shapes.append((NS[i % 5], KS[(i + i // 5) % 5]))
        rows += shapes[-1][0]
        i += 1
    layers, packs, xs_np, xs, ys = [], [], [], [], []
    for i, (N, K) in enumerate(shapes):
        w = weight_fn(i, N, K)
        layer, packed = make_layer(w, widths)
        x = synth.activations(0, "%s/x%d/%d" % (tag, i, M), M, K)
        layers.append(layer)
        packs.append((w, packed))
        xs_np.append(x)
        xs.append(to_dev(x))
        ys.append(torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV))
    ws = torch.empty(fq.Plan.workspace_bytes(len(layers)), dtype=torch.uint8, device=DEV)
    return shapes, layers, packs, xs_np, xs, ys, fq.Plan(layers, xs, ys, M, ws)


@pytest.mark.parametrize("M,every", [(16, 1), (5, 3), (2, 4), (32, 2), (21, 3)])
def test_streaming_plan_matches_oracle(M, every):
    shapes, layers, packs, xs_np, xs, ys, plan = _build(
        M, "par/stream", lambda i, N, K: synth.weight(0, "par/stream/w%d" % i, N, K, 0.02, outlier_p=0.001))
    for shift in (0, 1):
        pattern = [(4, 8, 16)[(i + shift) % 3] for i in range(len(layers))]
        for y in ys:
            y.fill_(float("nan"))
        plan.run(torch.tensor(pattern, dtype=torch.int32, device=DEV))
        torch.cuda.synchronize()
        for i, b in enumerate(pattern):
            y = ys[i].cpu().numpy()
            assert np.isfinite(y.astype(np.float32)).all(), (M, i, b, shapes[i])
            if (i + shift) % every:
                continue
            w, packed = packs[i]
            if b == 16:
                y_ref = oracle.linear(xs_np[i], w, None, None, 16)
            else:
                c, s, z = (t.cpu().numpy() for t in packed[b])
                y_ref = oracle.linear(xs_np[i], c, s, z, b)
            assert rel_err(y, y_ref) <= TOL_Y, (M, i, b, shapes[i])


@pytest.mark.parametrize("M", [16, 27])
def test_streaming_plan_long_rows(M):
    shapes, layers, packs, xs_np, xs, ys, plan = _build(
        M, "par/stream/long", lambda i, N, K: synth.weight(0, "par/stream/long/w%d" % i, N, K, 0.02, outlier_p=0.001),
        extra=LONG)
    for shift in (0, 1, 2):
        pattern = [(4, 8, 16)[(i + shift) % 3] for i in range(len(layers))]
        plan.run(torch.tensor(pattern, dtype=torch.int32, device=DEV))
        torch.cuda.synchronize()
        for i in list(range(len(LONG))) + [len(LONG) + 3 * shift, len(layers) - 1 - shift]:
            b = pattern[i]
            w, packed = packs[i]
            if b == 16:
                y_ref = oracle.linear(xs_np[i], w, None, None, 16)
            else:
                c, s, z = (t.cpu().numpy() for t in packed[b])
                y_ref = oracle.linear(xs_np[i], c, s, z, b)
            assert rel_err(ys[i].cpu().numpy(), y_ref) <= TOL_Y, (M, i, b, shapes[i])


@pytest.mark.parametrize("M", [16, 32])
def test_streaming_plan_integer_case_exact(M):
    # integer activations, weights on the quantization grid with s = 1 and z = 0 (every group
    # spans 0 .. 2^b - 1): every product and every partial sum is an integer below 2^24, so the
    # kernel's offset trick (x times 1024 + q, then x times -(1024 + z)) must cancel exactly
    rng = np.random.default_rng(3)

    def weights(i, N, K):
        w = rng.integers(0, 16, size=(N, K)).astype(np.float16)
        w[:, 0::128] = 0
        w[:, 1::128] = 15
        return w

    shapes, layers, packs, xs_np, xs, ys, plan = _build(M, "par/stream/int", weights)
    for i, (N, K) in enumerate(shapes):  # integer x in place of the generator's
        xi = (rng.integers(-1, 2, size=(M, K)) * (rng.random((M, K)) < 0.3)).astype(np.float16)
        xs_np[i] = xi
        xs[i].copy_(to_dev(xi))
    pattern = [(4, 16, 8, 16, 4)[i % 5] for i in range(len(layers))]
    plan.run(torch.tensor(pattern, dtype=torch.int32, device=DEV))
    torch.cuda.synchronize()
    for i in range(0, len(layers), 2):
        w, packed = packs[i]
        if pattern[i] == 4:
            assert torch.all(packed[4][1] == 1.0) and torch.all(packed[4][2] == 0)
        if pattern[i] == 8:  # 0 .. 15 on the 8-bit grid: s = 15 / 255 is not exact, skip
            continue
        expect = (xs_np[i].astype(np.float64) @ w.astype(np.float64).T)
        assert np.abs(expect).max() < 2048
        assert np.array_equal(ys[i].cpu().numpy().astype(np.float64), expect), (i, pattern[i], shapes[i])


def test_streaming_plan_skipped_entries_and_repeated_runs():
    # entries whose bit-width is none of the attached ones are passed over (y untouched) and the
    # tiles after them still run; launches follow one another without anything being reset by
    # the host in between (the kernel hands out its tiles from a queue it leaves at zero)
    M = 16
    shapes, layers, packs, xs_np, xs, ys, plan = _build(
        M, "par/stream/skip", lambda i, N, K: synth.weight(0, "par/stream/skip/w%d" % i, N, K, 0.02))
    n = len(layers)
    patterns = [
        [0 if i % 5 == 0 or i == n - 1 else (4, 8, 16)[i % 3] for i in range(n)],
        [0] * n,
        [3 if i % 2 else (16, 4, 8)[i % 3] for i in range(n)],
        [(8, 16, 4)[i % 3] for i in range(n)],
    ]
    for p, pattern in enumerate(patterns):
        for y in ys:
            y.fill_(7.0)
        plan.run(torch.tensor(pattern, dtype=torch.int32, device=DEV))
        torch.cuda.synchronize()
        checked = 0
        for i, b in enumerate(pattern):
            y = ys[i].cpu().numpy()
            if b not in (4, 8, 16):
                assert np.all(y == np.float16(7.0)), (p, i, b)
                continue
            assert np.isfinite(y.astype(np.float32)).all(), (p, i, b)
            if checked >= 6 and i < n - 3:
                continue
            checked += 1
            w, packed = packs[i]
            if b == 16:
                y_ref = oracle.linear(xs_np[i], w, None, None, 16)
            else:
                c, s, z = (t.cpu().numpy() for t in packed[b])
                y_ref = oracle.linear(xs_np[i], c, s, z, b)
            assert rel_err(y, y_ref) <= TOL_Y, (p, i, b, shapes[i])


@pytest.mark.parametrize("M,extra", [(16, tuple(LONG)), (23, ()), (2, ()), (32, tuple(LONG[:3]))])
def test_streaming_plan_with_2bit_copies(M, extra):
    # 2-bit copies run in the same launch as the others: a stage is a whole chunk of x (512 k,
    # four units), and a row may end with 2, 4 or 6 of a line's 8 pieces (K % 512 = 128, 256, 384)
    shapes, layers, packs, xs_np, xs, ys, plan = _build(
        M, "par/stream/w2", lambda i, N, K: synth.weight(0, "par/stream/w2/w%d" % i, N, K, 0.02, outlier_p=0.001),
        extra=list(extra), widths=(2, 4, 8, 16))
    n = len(layers)
    patterns = [[(2, 4, 8, 16)[(i + s) % 4] for i in range(n)] for s in range(2)] + [[2] * n, [(8, 16, 4)[i % 3] for i in range(n)],
                                                                                       [0 if i % 3 == 0 else 2 for i in range(n)]]
    unserved = False
    for p, pattern in enumerate(patterns):
        for y in ys:
            y.fill_(5.0)
        plan.run(torch.tensor(pattern, dtype=torch.int32, device=DEV))
        torch.cuda.synchronize()
        unserved = unserved or 0 in pattern  # (the flag word stays set once set)
        assert plan.status() == (0, int(unserved))
        for i, b in enumerate(pattern):
            y = ys[i].cpu().numpy()
            if b == 0:
                assert np.all(y == np.float16(5.0)), (p, i)
                continue
            assert np.isfinite(y.astype(np.float32)).all(), (p, i, b)
            if (i + p) % 4 and i < n - 2 and i >= len(extra):
                continue
            w, packed = packs[i]
            if b == 16:
                y_ref = oracle.linear(xs_np[i], w, None, None, 16)
            else:
                c, s, z = (t.cpu().numpy() for t in packed[b])
                y_ref = oracle.linear(xs_np[i], c, s, z, b)
            assert rel_err(y, y_ref) <= TOL_Y, (M, p, i, b, shapes[i])


@pytest.mark.parametrize("M", [16, 32])
def test_streaming_plan_2bit_integer_case_exact(M):
    # integer activations, weights 0 .. 3 with every group spanning them (s = 1, z = 0): every
    # product, every partial sum and the four offsets by bit position that the kernel adds and
    # removes (1024, 256, 64, 16) are integers below 2^24, so the output is the integer product
    # exactly; each k % 16 carries its own pattern, so a swapped pair or byte shows
    rng = np.random.default_rng(11)

    def weights(i, N, K):
        w = rng.integers(0, 4, size=(N, K)).astype(np.float16)
        w[:, 0::128] = 0
        w[:, 1::128] = 3
        return w

    shapes, layers, packs, xs_np, xs, ys, plan = _build(M, "par/stream/int2", weights, extra=[(300, 2432), (260, 4096)],
                                                        widths=(2, 4))
    for i, (N, K) in enumerate(shapes):
        xi = (rng.integers(-2, 3, size=(M, K)) * (rng.random((M, K)) < 0.3)).astype(np.float16)
        xs_np[i] = xi
        xs[i].copy_(to_dev(xi))
    pattern = [(2, 2, 4)[i % 3] for i in range(len(layers))]
    plan.run(torch.tensor(pattern, dtype=torch.int32, device=DEV))
    torch.cuda.synchronize()
    for i in list(range(0, len(layers), 3)) + [1]:
        w, packed = packs[i]
        assert pattern[i] == 2
        assert torch.all(packed[2][1] == 1.0) and torch.all(packed[2][2] == 0)
        expect = (xs_np[i].astype(np.float64) @ w.astype(np.float64).T)
        assert np.abs(expect).max() < 2048
        assert np.array_equal(ys[i].cpu().numpy().astype(np.float64), expect), (i, shapes[i])
    # one-hot x on one linear: output n is the code at that k, for every position of a 16-code word
    i = 0
    N, K = shapes[i]
    for k in list(range(0, 33)) + [127, 128, 511, 512, 1023, K - 1]:
        x1 = np.zeros((M, K), dtype=np.float16)
        x1[M - 1, k] = 1
        xs[i].copy_(to_dev(x1))
        plan.run(torch.tensor(pattern, dtype=torch.int32, device=DEV))
        torch.cuda.synchronize()
        assert np.array_equal(ys[i].cpu().numpy()[M - 1].astype(np.int64), packs[i][0][:, k].astype(np.int64)), k


def test_streaming_plan_with_more_than_256_entries():
    # the per-launch entry lists are drawn up 256 entries at a time
    M, n = 16, 330
    rng = np.random.default_rng(7)
    shapes = [(820 + 13 * (i % 9), (128, 256, 384)[i % 3]) for i in range(n)]
    assert sum(N for N, _ in shapes) >= MIN_ROWS + 256
    layers, packs, xs_np, xs, ys = [], [], [], [], []
    for i, (N, K) in enumerate(shapes):
        w = synth.weight(0, "par/stream/many/w%d" % i, N, K, 0.02)
        layer, packed = make_layer(w, (2, 4, 8) if i % 2 else (4, 8, 16))
        layers.append(layer)
        packs.append((w, packed))
        xs_np.append(synth.activations(0, "par/stream/many/x%d" % i, M, K))
        xs.append(to_dev(xs_np[-1]))
        ys.append(torch.empty((M, N), dtype=torch.float16, device=DEV))
    ws = torch.empty(fq.Plan.workspace_bytes(n), dtype=torch.uint8, device=DEV)
    plan = fq.Plan(layers, xs, ys, M, ws)
    for p in range(2):
        # widths that some layers do not hold: those entries are passed over
        pattern = [int(rng.choice((2, 4, 8, 16))) for _ in range(n)]
        for y in ys:
            y.fill_(9.0)
        plan.run(torch.tensor(pattern, dtype=torch.int32, device=DEV))
        torch.cuda.synchronize()
        checked = 0
        for i, b in enumerate(pattern):
            y = ys[i].cpu().numpy()
            w, packed = packs[i]
            if b not in packed:
                assert np.all(y == np.float16(9.0)), (p, i, b)
                continue
            assert np.isfinite(y.astype(np.float32)).all(), (p, i, b)
            if i % 23 and i not in (255, 256, 257, n - 1):
                continue
            checked += 1
            if b == 16:
                y_ref = oracle.linear(xs_np[i], w, None, None, 16)
            else:
                c, s, z = (t.cpu().numpy() for t in packed[b])
                y_ref = oracle.linear(xs_np[i], c, s, z, b)
            assert rel_err(y, y_ref) <= TOL_Y, (p, i, b, shapes[i])
        assert checked >= 8

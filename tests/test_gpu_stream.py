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


@pytest.mark.parametrize("M", [16, 23])
def test_streaming_plan_with_2bit_copies(M):
    # a plan of the streaming kernel's size whose layers also hold 2-bit copies runs in two
    # launches: the streaming kernel passes over the entries that are at 2 bits, the register-fed
    # kernel runs exactly those
    shapes, layers, packs, xs_np, xs, ys, plan = _build(
        M, "par/stream/w2", lambda i, N, K: synth.weight(0, "par/stream/w2/w%d" % i, N, K, 0.02, outlier_p=0.001),
        widths=(2, 4, 8, 16))
    n = len(layers)
    patterns = [[(2, 4, 8, 16)[(i + s) % 4] for i in range(n)] for s in range(2)] + [[2] * n, [(8, 16, 4)[i % 3] for i in range(n)],
                                                                                       [0 if i % 3 == 0 else 2 for i in range(n)]]
    for p, pattern in enumerate(patterns):
        for y in ys:
            y.fill_(5.0)
        plan.run(torch.tensor(pattern, dtype=torch.int32, device=DEV))
        torch.cuda.synchronize()
        for i, b in enumerate(pattern):
            y = ys[i].cpu().numpy()
            if b == 0:
                assert np.all(y == np.float16(5.0)), (p, i)
                continue
            assert np.isfinite(y.astype(np.float32)).all(), (p, i, b)
            if (i + p) % 4 and i < n - 2:
                continue
            w, packed = packs[i]
            if b == 16:
                y_ref = oracle.linear(xs_np[i], w, None, None, 16)
            else:
                c, s, z = (t.cpu().numpy() for t in packed[b])
                y_ref = oracle.linear(xs_np[i], c, s, z, b)
            assert rel_err(y, y_ref) <= TOL_Y, (M, p, i, b, shapes[i])


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

"""GPU parity of the packed 2-bit path (Table 1's lowest width; Sec. 2.2 Eq. (2), (3) with n = 2)
against the CPU oracle: codes, scales and zero points bit-exact, decode outputs (M = 1 and batches
up to 32, single calls and plans that mix 2 / 4 / 8 / 16 bits per entry) within 2e-3 max-abs
normalised; the prefill-shaped GEMM at 2 bits likewise."""
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
def test_quantize_2bit_bit_exact(shape, outl, sym):
    N, K = shape
    w = synth.weight(0, "par2/q/%dx%d" % shape, N, K, 0.02, outlier_p=outl)
    c_ref, s_ref, z_ref = (oracle.quantize_sym if sym else oracle.quantize)(w, 2)
    sizes = fq.fq_packed_sizes(N, K, 2)
    assert sizes == (N * K // 4, N * (K // 128) * 4, N * (K // 128))
    c = torch.full((sizes[0],), 0xAA, dtype=torch.uint8, device=DEV)
    s = torch.empty((N, K // 128), dtype=torch.float32, device=DEV)
    z = torch.empty((N, K // 128), dtype=torch.uint8, device=DEV)
    (fq.fq_quantize_sym if sym else fq.fq_quantize)(to_dev(w), N, K, 2, 128, c, s, z)
    torch.cuda.synchronize()
    assert np.array_equal(c.cpu().numpy().reshape(N, K // 4), c_ref)
    assert np.array_equal(s.cpu().numpy().view(np.uint32), s_ref.view(np.uint32))
    assert np.array_equal(z.cpu().numpy(), z_ref)


def test_quantize_2bit_degenerate_groups():
    w = np.zeros((3, 512), dtype=np.float16)
    w[0, 128:256] = np.linspace(0.01, 2.0, 128)             # all positive
    w[0, 256:384] = -np.linspace(0.01, 2.0, 128)            # all negative
    w[1, :4] = (np.arange(4) - 1) / 64.0                     # on-grid
    w[1, 4:7] = [0.5 / 64, 1.5 / 64, -0.5 / 64]              # ties
    w[2, 0], w[2, 1] = 65504.0, -65504.0
    w[2, 2:128] = np.linspace(-3e4, 3e4, 126)
    c_ref, s_ref, z_ref = oracle.quantize(w, 2)
    c, s, z = gpu_quantize(to_dev(w), 2)
    assert np.array_equal(c.cpu().numpy(), c_ref)
    assert np.array_equal(s.cpu().numpy().view(np.uint32), s_ref.view(np.uint32))
    assert np.array_equal(z.cpu().numpy(), z_ref)


# K: one slice of 4096 exactly, less than one, several with a ragged last one, a single group
@pytest.mark.parametrize("N,K", [(4096, 4096), (100, 1408), (37, 128), (16, 11008), (530, 5120), (64, 8192),
                                 (21, 13824)])
def test_linear_2bit_m1_matches_oracle(N, K):
    w = synth.weight(0, "par2/lin/%dx%d" % (N, K), N, K, 0.02, outlier_p=0.001)
    x = synth.activations(0, "par2/lin/x/%d" % K, 1, K)
    layer, packed = make_layer(w, (2,))
    y = gpu_linear(layer, 2, x)
    c, s, z = (t.cpu().numpy() for t in packed[2])
    y_ref = oracle.linear(x, c, s, z, 2)
    assert not np.isnan(y.astype(np.float32)).any()
    assert rel_err(y, y_ref) <= TOL_Y


def test_linear_2bit_integer_case_exact():
    # codes equal to the integer weights (s = 1, z = 0), integer x: every product, every partial sum
    # and the offsets that the kernel adds and removes (1024 / 256 / 64 / 16 by bit position) are
    # integers below 2^24, so the output must be the integer matrix-vector product exactly; each
    # position k % 16 of a code word carries its own weight pattern, so a swapped pair shows
    rng = np.random.default_rng(7)
    N, K = 48, 8192 + 384
    w = rng.integers(0, 4, size=(N, K))
    w[:, 0::128] = 0
    w[:, 1::128] = 3
    x = (rng.integers(-2, 3, size=(1, K)) * (rng.random((1, K)) < 0.25)).astype(np.float16)
    layer, packed = make_layer(w.astype(np.float16), (2,))
    assert torch.all(packed[2][1] == 1.0) and torch.all(packed[2][2] == 0)
    y = gpu_linear(layer, 2, x)
    expect = x.astype(np.float64) @ w.T.astype(np.float64)
    assert np.abs(expect).max() < 2048
    assert np.array_equal(y.astype(np.float64), expect)
    # one-hot x: output n is the code at that k, for every position of a 16-code word and beyond
    for k in list(range(2, 18)) + [63, 64, 4095, 4096, K - 1]:
        x1 = np.zeros((1, K), dtype=np.float16)
        x1[0, k] = 1
        assert np.array_equal(gpu_linear(layer, 2, x1)[0].astype(np.int64), w[:, k]), k


def test_plan_with_2bit_entries_matches_individual_calls_and_oracle():
    shapes = [(256, 1024), (100, 1408), (512, 4096), (64, 11008), (40, 128), (300, 4096)]
    layers, xs, ys, xs_np, packs = [], [], [], [], []
    for i, (N, K) in enumerate(shapes):
        w = synth.weight(0, "par2/plan/w%d" % i, N, K, 0.02, outlier_p=0.001)
        layer, packed = make_layer(w, (2, 4, 8, 16) if i % 2 == 0 else (2, 8))
        x = synth.activations(0, "par2/plan/x%d" % i, 1, K)
        layers.append(layer)
        packs.append((w, packed))
        xs_np.append(x)
        xs.append(to_dev(x))
        ys.append(torch.zeros((1, N), dtype=torch.float16, device=DEV))
    ws = torch.empty(fq.Plan.workspace_bytes(len(layers)), dtype=torch.uint8, device=DEV)
    plan = fq.Plan(layers, xs, ys, 1, ws)
    for trial, pattern in enumerate([[2, 2, 2, 2, 2, 2], [2, 8, 4, 2, 16, 8], [16, 2, 2, 8, 4, 2], [4, 8, 8, 2, 2, 2]]):
        for y in ys:
            y.fill_(float("nan"))
        plan.run(torch.tensor(pattern, dtype=torch.int32, device=DEV))
        torch.cuda.synchronize()
        for i, b in enumerate(pattern):
            w, packed = packs[i]
            if b == 16:
                y_ref = oracle.linear(xs_np[i], w, None, None, 16)
            else:
                c, s, z = (t.cpu().numpy() for t in packed[b])
                y_ref = oracle.linear(xs_np[i], c, s, z, b)
            y = ys[i].cpu().numpy()
            assert rel_err(y, y_ref) <= TOL_Y, (trial, i, b)
            assert np.array_equal(y.view(np.uint16), gpu_linear(layers[i], b, xs_np[i]).view(np.uint16)), (trial, i, b)


@pytest.mark.parametrize("M,N,K", [(2, 100, 1408), (4, 4096, 4096), (8, 530, 5120), (16, 64, 11008), (17, 300, 2048),
                                   (32, 1000, 4096), (5, 37, 128), (32, 16, 13824), (16, 70, 384)])
def test_linear_2bit_batched_matches_oracle(M, N, K):
    w = synth.weight(0, "par2/b/%dx%d" % (N, K), N, K, 0.02, outlier_p=0.001)
    x = synth.activations(0, "par2/b/x/%d/%d" % (M, K), M, K)
    layer, packed = make_layer(w, (2,))
    y = gpu_linear(layer, 2, x)
    c, s, z = (t.cpu().numpy() for t in packed[2])
    y_ref = oracle.linear(x, c, s, z, 2)
    assert not np.isnan(y.astype(np.float32)).any()
    assert rel_err(y, y_ref) <= TOL_Y


@pytest.mark.parametrize("M", [3, 16, 32])
def test_linear_2bit_batched_integer_case_exact(M):
    # s = 1, z = 0, integer x: the MFMA operands are the exact integers q - z, every sum is below
    # 2^24; K = 128 * 67 ends a row after the first group of a 64-byte load
    rng = np.random.default_rng(8)
    N, K = 80, 128 * 67
    w = rng.integers(0, 4, size=(N, K))
    w[:, 0::128] = 0
    w[:, 1::128] = 3
    x = (rng.integers(-2, 3, size=(M, K)) * (rng.random((M, K)) < 0.25)).astype(np.float16)
    layer, packed = make_layer(w.astype(np.float16), (2,))
    y = gpu_linear(layer, 2, x)
    expect = x.astype(np.float64) @ w.T.astype(np.float64)
    assert np.abs(expect).max() < 2048
    assert np.array_equal(y.astype(np.float64), expect)
    for k in (0, 7, 8, 9, 15, 16, 63, 64, 127, 128, 255, 256, K - 129, K - 1):  # one-hot x in batch row 1
        x1 = np.zeros((M, K), dtype=np.float16)
        x1[1, k] = 1
        y1 = gpu_linear(layer, 2, x1)
        assert np.array_equal(y1[1].astype(np.int64), w[:, k]), k
        assert not y1[0].any() and not y1[2].any()


def test_batched_plan_with_2bit_entries():
    # a plan large enough for the streaming kernel (70 x 4096 rows): every width is served per
    # entry, the 2-bit entries among the others in the one launch
    M = 8
    shapes = [(4096, 1024)] * 70
    layers, xs, ys, xs_np, packs = [], [], [], [], []
    for i, (N, K) in enumerate(shapes):
        w = synth.weight(0, "par2/bplan/w%d" % (i % 5), N, K, 0.02, outlier_p=0.001)
        layer, packed = make_layer(w, (2, 4, 8, 16) if i % 5 == 0 else (2, 4))
        x = synth.activations(0, "par2/bplan/x%d" % (i % 7), M, K)
        layers.append(layer), packs.append((w, packed)), xs_np.append(x), xs.append(to_dev(x))
        ys.append(torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV))
    ws = torch.empty(fq.Plan.workspace_bytes(len(layers)), dtype=torch.uint8, device=DEV)
    plan = fq.Plan(layers, xs, ys, M, ws)
    pattern = [(2, 4, 8, 16, 2)[(i // 5) % 5] if i % 5 == 0 else (2, 4)[i % 2] for i in range(len(layers))]
    plan.run(torch.tensor(pattern, dtype=torch.int32, device=DEV))
    torch.cuda.synchronize()
    assert {pattern[i] for i in range(0, 25, 5)} == {2, 4, 8, 16}
    for i in list(range(0, 25, 5)) + [1, 2, 33, 69]:
        b = pattern[i]
        w, packed = packs[i]
        if b == 16:
            y_ref = oracle.linear(xs_np[i], w, None, None, 16)
        else:
            c, s, z = (t.cpu().numpy() for t in packed[b])
            y_ref = oracle.linear(xs_np[i], c, s, z, b)
        assert rel_err(ys[i].cpu().numpy(), y_ref) <= TOL_Y, (i, b)
    for y in ys:
        assert torch.isfinite(y.float()).all()


# ------------------------------------------------------------------ prefill-shaped (MFMA GEMM) at 2 bits

@pytest.mark.parametrize("M,N,K", [(33, 100, 1408), (128, 256, 1024), (300, 200, 2048), (257, 130, 128),
                                   (64, 129, 4096), (2, 48, 32768 + 128)])
def test_linear_2bit_prefill_matches_oracle(M, N, K):
    w = synth.weight(0, "par2/pre/%dx%d" % (N, K), N, K, 0.015, outlier_p=0.001)
    x = synth.activations(0, "par2/pre/x/%dx%d" % (M, K), M, K)
    layer, packed = make_layer(w, (2,))
    y = gpu_linear(layer, 2, x)
    c, s, z = (t.cpu().numpy() for t in packed[2])
    y_ref = oracle.linear(x, c, s, z, 2)
    assert y.shape == (M, N)
    assert not np.isnan(y.astype(np.float32)).any()
    assert rel_err(y, y_ref) <= TOL_Y
    for m in (0, M // 2, M - 1):
        assert rel_err(y[m:m + 1], y_ref[m:m + 1]) <= TOL_Y, m


def test_linear_2bit_prefill_integer_case_exact():
    # codes = the integer weights (s = 1, z = 0), small integer x: the GEMM's operands
    # half((q - z) * half(s)) and its binary32 sums are exact, so the output is the integer product;
    # one-hot rows of x pick single codes at every position of a 16-byte row of codes
    rng = np.random.default_rng(9)
    M, N, K = 200, 150, 1024
    w = rng.integers(0, 4, size=(N, K))
    w[:, 0::128] = 0
    w[:, 1::128] = 3
    x = rng.integers(-2, 3, size=(M, K))
    for m in range(70):
        x[m] = 0
        x[m, m] = 1
    layer, packed = make_layer(w.astype(np.float16), (2,))
    y = gpu_linear(layer, 2, x.astype(np.float16))
    expect = (x @ w.T).astype(np.float16)
    assert np.array_equal(y.view(np.uint16), expect.view(np.uint16))

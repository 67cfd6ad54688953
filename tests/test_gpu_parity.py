"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on identical
seeded inputs.  Bars: packed codes, scales and zeros bit-exact; fp16 outputs within 2e-3
(max-abs normalised); entropy and KL within 1e-4 relative (absolute floor 1e-7)."""
import math

import numpy as np
import pytest
import torch

import oracle
import synth
import paper_2506_12024_amd as fq
from gpu_util import DEV, gpu_linear, gpu_quantize, make_layer, rel_err, to_dev

pytestmark = pytest.mark.gpu

TOL_Y = 2e-3
TOL_E = 1e-4
FLOOR_E = 1e-7


# ------------------------------------------------------------------ quantize

@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("shape,outl", [((4096, 4096), 0.001), ((48, 1408), 0.01), ((1, 128), 0.0),
                                        ((333, 11008), 0.0)])
def test_quantize_bit_exact(bits, shape, outl):
    N, K = shape
    w = synth.weight(0, "par/q/%dx%d" % shape, N, K, 0.02, outlier_p=outl)
    c_ref, s_ref, z_ref = oracle.quantize(w, bits)
    c, s, z = gpu_quantize(to_dev(w), bits)
    torch.cuda.synchronize()
    assert np.array_equal(c.cpu().numpy(), c_ref)
    assert np.array_equal(s.cpu().numpy().view(np.uint32), s_ref.view(np.uint32))
    assert np.array_equal(z.cpu().numpy(), z_ref)


@pytest.mark.parametrize("bits", [4, 8])
def test_quantize_degenerate_groups(bits):
    # all-zero group, one-signed groups, exact ties, a group holding the fp16 extremes
    w = np.zeros((4, 512), dtype=np.float16)
    w[0, 128:256] = np.linspace(0.01, 2.0, 128)            # all positive
    w[0, 256:384] = -np.linspace(0.01, 2.0, 128)           # all negative
    w[1, :16] = (np.arange(16) - 7) / 64.0                  # on-grid
    w[1, 16:20] = [1.5 / 64, 2.5 / 64, -0.5 / 64, -1.5 / 64]  # ties
    w[2, 0] = 65504.0
    w[2, 1] = -65504.0
    w[2, 2:128] = np.linspace(-3e4, 3e4, 126)
    w[3, :] = synth.normal_f16(1, "par/q/sub", 512, 1e-6)   # subnormal halves
    c_ref, s_ref, z_ref = oracle.quantize(w, bits)
    c, s, z = gpu_quantize(to_dev(w), bits)
    assert np.array_equal(c.cpu().numpy(), c_ref)
    assert np.array_equal(s.cpu().numpy().view(np.uint32), s_ref.view(np.uint32))
    assert np.array_equal(z.cpu().numpy(), z_ref)


# ------------------------------------------------------------------ linear, batch 1

@pytest.mark.parametrize("bits", [4, 8, 16])
@pytest.mark.parametrize("N,K", [(4096, 4096), (100, 1408), (37, 128), (16, 11008), (530, 5120),
                                 # the 13B-shaped stack's long row and its wide FFN, at batch 1
                                 (200, 13824), (13824, 5120)])
def test_linear_m1_matches_oracle(bits, N, K):
    w = synth.weight(0, "par/lin/%dx%d" % (N, K), N, K, 0.02, outlier_p=0.001)
    x = synth.activations(0, "par/lin/x/%d" % K, 1, K)
    layer, packed = make_layer(w, (bits,))
    y = gpu_linear(layer, bits, x)
    if bits == 16:
        y_ref = oracle.linear(x, w, None, None, 16)
    else:
        c, s, z = (t.cpu().numpy() for t in packed[bits])
        y_ref = oracle.linear(x, c, s, z, bits)
    assert not np.isnan(y.astype(np.float32)).any()
    assert rel_err(y, y_ref) <= TOL_Y


def test_linear_switching_uses_resident_copies_without_repacking():
    # One layer, all three copies attached; alternate the bit-width call by call and check
    # (a) each call matches the oracle at its bit-width, (b) the packed buffers are
    # byte-identical afterwards (nothing was rewritten on a switch).
    N, K = 256, 2048
    w = synth.weight(0, "par/sw/w", N, K, 0.02, outlier_p=0.001)
    layer, packed = make_layer(w, (4, 8, 16))
    before = {b: [t.clone() for t in packed[b]] for b in packed}
    refs = {}
    for step, bits in enumerate([4, 8, 16, 8, 4, 4, 16, 8]):
        x = synth.activations(0, "par/sw/x/%d" % step, 1, K)
        y = gpu_linear(layer, bits, x)
        if bits == 16:
            y_ref = oracle.linear(x, w, None, None, 16)
        else:
            c, s, z = (t.cpu().numpy() for t in packed[bits])
            y_ref = oracle.linear(x, c, s, z, bits)
        assert rel_err(y, y_ref) <= TOL_Y, (step, bits)
        refs[step] = y
    for b in packed:
        for t0, t1 in zip(before[b], packed[b]):
            assert torch.equal(t0, t1)


def test_linear_deterministic():
    w = synth.weight(0, "par/det/w", 512, 4096, 0.02)
    x = synth.activations(0, "par/det/x", 1, 4096)
    layer, _ = make_layer(w, (4, 8))
    for bits in (4, 8):
        a = gpu_linear(layer, bits, x)
        b = gpu_linear(layer, bits, x)
        assert np.array_equal(a.view(np.uint16), b.view(np.uint16))


def test_linear_on_grid_weights_exact():
    # Weights j/64, integer x: every product and sum is exact in binary32, so the GPU must
    # reproduce the oracle bit for bit.
    rng = np.random.default_rng(5)
    N, K = 64, 2048
    j = rng.integers(-7, 9, size=(N, K))
    j[:, 0::128] = -7
    j[:, 1::128] = 8
    w = (j / 64.0).astype(np.float16)
    x = rng.integers(-3, 4, size=(1, K)).astype(np.float16)
    layer, packed = make_layer(w, (4,))
    y = gpu_linear(layer, 4, x)
    c, s, z = (t.cpu().numpy() for t in packed[4])
    y_ref = oracle.linear(x, c, s, z, 4)
    assert np.array_equal(y.view(np.uint16), y_ref.view(np.uint16))


# ------------------------------------------------------------------ linear, batch 2..32 (MFMA)

@pytest.mark.parametrize("bits", [4, 8, 16])
@pytest.mark.parametrize("M,N,K", [(2, 100, 1408), (4, 4096, 4096), (8, 530, 5120), (16, 64, 11008),
                                   (17, 300, 2048), (32, 1000, 4096), (5, 37, 128), (32, 16, 13824),
                                   # enough rows for the 64-row tiles (fewer rows take the K-split kernel)
                                   (16, 11008, 1024), (24, 9000, 640)])
def test_linear_batched_matches_oracle(bits, M, N, K):
    w = synth.weight(0, "par/linb/%dx%d" % (N, K), N, K, 0.02, outlier_p=0.001)
    x = synth.activations(0, "par/linb/x/%dx%d" % (M, K), M, K)
    layer, packed = make_layer(w, (bits,))
    y = gpu_linear(layer, bits, x)
    if bits == 16:
        y_ref = oracle.linear(x, w, None, None, 16)
    else:
        c, s, z = (t.cpu().numpy() for t in packed[bits])
        y_ref = oracle.linear(x, c, s, z, bits)
    assert y.shape == (M, N)
    assert not np.isnan(y.astype(np.float32)).any()
    assert rel_err(y, y_ref) <= TOL_Y
    # each batch row on its own must also be right (a row mix-up can hide in the max-abs norm)
    for m in range(M):
        assert rel_err(y[m:m + 1], y_ref[m:m + 1]) <= TOL_Y, m


def test_linear_batched_integer_case_exact():
    # s = 1, z = 0 integer weights and integer x: every operation is exact, the result must
    # equal the integer matrix product bit for bit (catches any operand-layout mistake).
    rng = np.random.default_rng(7)
    for bits, M, N, K in [(4, 16, 48, 1024), (8, 32, 80, 1152), (4, 3, 20, 2048)]:
        qmax = (1 << bits) - 1
        w = rng.integers(0, qmax + 1, size=(N, K))
        w[:, 0::128] = 0
        w[:, 1::128] = qmax
        x = rng.integers(-2, 3, size=(M, K))
        layer, packed = make_layer(w.astype(np.float16), (bits,))
        assert torch.all(packed[bits][1] == 1.0) and torch.all(packed[bits][2] == 0)
        y = gpu_linear(layer, bits, x.astype(np.float16))
        expect = (x @ w.T).astype(np.float16)
        assert np.array_equal(y.view(np.uint16), expect.view(np.uint16)), (bits, M, N, K)


def test_plan_batched_matches_oracle():
    shapes = [(256, 1024), (100, 1408), (512, 4096), (64, 11008)]
    for M in (4, 32):
        layers, xs, ys, xs_np, packs = [], [], [], [], []
        for i, (N, K) in enumerate(shapes):
            w = synth.weight(0, "par/planb/w%d" % i, N, K, 0.02, outlier_p=0.001)
            layer, packed = make_layer(w, (4, 8, 16))
            x = synth.activations(0, "par/planb/x%d/%d" % (i, M), M, K)
            layers.append(layer)
            packs.append((w, packed))
            xs_np.append(x)
            xs.append(to_dev(x))
            ys.append(torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV))
        ws = torch.empty(fq.Plan.workspace_bytes(len(layers)), dtype=torch.uint8, device=DEV)
        plan = fq.Plan(layers, xs, ys, M, ws)
        pattern = [4, 8, 16, 4]
        plan.run(torch.tensor(pattern, dtype=torch.int32, device=DEV))
        torch.cuda.synchronize()
        for i, b in enumerate(pattern):
            w, packed = packs[i]
            if b == 16:
                y_ref = oracle.linear(xs_np[i], w, None, None, 16)
            else:
                c, s, z = (t.cpu().numpy() for t in packed[b])
                y_ref = oracle.linear(xs_np[i], c, s, z, b)
            assert rel_err(ys[i].cpu().numpy(), y_ref) <= TOL_Y, (M, i, b)


# ------------------------------------------------------------------ linear, prefill-shaped (MFMA GEMM)

@pytest.mark.parametrize("bits", [4, 8, 16])
@pytest.mark.parametrize("M,N,K", [(33, 100, 1408), (128, 256, 1024), (300, 200, 2048), (257, 130, 128),
                                   (64, 129, 4096)])
def test_linear_prefill_matches_oracle(bits, M, N, K):
    w = synth.weight(0, "par/pre/%dx%d" % (N, K), N, K, 0.015, outlier_p=0.001)
    x = synth.activations(0, "par/pre/x/%dx%d" % (M, K), M, K)
    layer, packed = make_layer(w, (bits,))
    y = gpu_linear(layer, bits, x)
    if bits == 16:
        y_ref = oracle.linear(x, w, None, None, 16)
    else:
        c, s, z = (t.cpu().numpy() for t in packed[bits])
        y_ref = oracle.linear(x, c, s, z, bits)
    assert y.shape == (M, N)
    assert not np.isnan(y.astype(np.float32)).any()
    assert rel_err(y, y_ref) <= TOL_Y
    for m in (0, M // 2, M - 1):
        assert rel_err(y[m:m + 1], y_ref[m:m + 1]) <= TOL_Y, m


def test_linear_prefill_integer_case_exact():
    rng = np.random.default_rng(8)
    for bits, M, N, K in [(4, 200, 150, 1024), (8, 130, 70, 640), (16, 100, 140, 256)]:
        qmax = 15 if bits == 4 else 255 if bits == 8 else 8
        w = rng.integers(0, qmax + 1, size=(N, K))
        w[:, 0::128] = 0
        w[:, 1::128] = qmax
        x = rng.integers(-2, 3, size=(M, K))
        layer, packed = make_layer(w.astype(np.float16), (bits,))
        y = gpu_linear(layer, bits, x.astype(np.float16))
        expect = (x @ w.T).astype(np.float16)
        assert np.array_equal(y.view(np.uint16), expect.view(np.uint16)), (bits, M, N, K)


@pytest.mark.parametrize("bits", [2, 4, 8, 16])
@pytest.mark.parametrize("M,N,K", [(1, 200, 28672), (1, 70, 32768), (1, 33, 24704), (4, 100, 28672), (16, 300, 32768),
                                   (32, 64, 28672), (16, 4200, 28672)])
def test_linear_wide_rows_match_oracle(bits, M, N, K):
    # the widest rows the decode kernels take (Llama-70B's FFN is 28672 wide; the limit is 32768):
    # at batch 1 the whole row of x sits in LDS, above the default limit of dynamic LDS
    w = synth.weight(0, "par/wide/%dx%d" % (N, K), N, K, 0.015, outlier_p=0.001)
    x = synth.activations(0, "par/wide/x/%dx%d" % (M, K), M, K)
    layer, packed = make_layer(w, (bits,))
    y = gpu_linear(layer, bits, x)
    if bits == 16:
        y_ref = oracle.linear(x, w, None, None, 16)
    else:
        c, s, z = (t.cpu().numpy() for t in packed[bits])
        y_ref = oracle.linear(x, c, s, z, bits)
    assert not np.isnan(y.astype(np.float32)).any()
    for m in range(M):
        assert rel_err(y[m:m + 1], y_ref[m:m + 1]) <= TOL_Y, m


def test_plan_wide_rows_match_oracle():
    shapes = [(300, 28672), (128, 4096), (90, 32768), (520, 28672), (64, 128)]
    pattern = [4, 8, 16, 8, 4]
    for M in (1, 8):
        layers, packs, xs_np, xs, ys = [], [], [], [], []
        for i, (N, K) in enumerate(shapes):
            w = synth.weight(0, "par/wideplan/w%d" % i, N, K, 0.015, outlier_p=0.001)
            layer, packed = make_layer(w, (4, 8, 16))
            layers.append(layer)
            packs.append((w, packed))
            xs_np.append(synth.activations(0, "par/wideplan/x%d/%d" % (i, M), M, K))
            xs.append(to_dev(xs_np[-1]))
            ys.append(torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV))
        ws = torch.empty(fq.Plan.workspace_bytes(len(layers)), dtype=torch.uint8, device=DEV)
        plan = fq.Plan(layers, xs, ys, M, ws)
        for shift in range(3):
            bits = [pattern[(i + shift) % 5] for i in range(5)]
            plan.run(torch.tensor(bits, dtype=torch.int32, device=DEV))
            torch.cuda.synchronize()
            for i, b in enumerate(bits):
                w, packed = packs[i]
                if b == 16:
                    y_ref = oracle.linear(xs_np[i], w, None, None, 16)
                else:
                    c, s, z = (t.cpu().numpy() for t in packed[b])
                    y_ref = oracle.linear(xs_np[i], c, s, z, b)
                assert rel_err(ys[i].cpu().numpy(), y_ref) <= TOL_Y, (M, shift, i, b)


def test_decode_call_with_large_k_takes_the_gemm_path():
    # K beyond what the decode kernels take: batch-1 still works (GEMM path)
    N, K = 48, 32768 + 128
    w = synth.weight(0, "par/bigk/w", N, K, 0.015)
    x = synth.activations(0, "par/bigk/x", 2, K)
    layer, packed = make_layer(w, (4,))
    y = gpu_linear(layer, 4, x)
    c, s, z = (t.cpu().numpy() for t in packed[4])
    assert rel_err(y, oracle.linear(x, c, s, z, 4)) <= TOL_Y


# ------------------------------------------------------------------ plan (one launch, device bits)

def test_plan_matches_individual_calls_and_oracle():
    shapes = [(256, 1024), (100, 1408), (512, 4096), (64, 11008), (40, 128)]
    layers, xs, ys, xs_np, packs = [], [], [], [], []
    for i, (N, K) in enumerate(shapes):
        w = synth.weight(0, "par/plan/w%d" % i, N, K, 0.02, outlier_p=0.001)
        layer, packed = make_layer(w, (4, 8, 16) if i % 2 == 0 else (4, 8))
        x = synth.activations(0, "par/plan/x%d" % i, 1, K)
        layers.append(layer)
        packs.append((w, packed))
        xs_np.append(x)
        xs.append(to_dev(x))
        ys.append(torch.zeros((1, N), dtype=torch.float16, device=DEV))
    ws = torch.empty(fq.Plan.workspace_bytes(len(layers)), dtype=torch.uint8, device=DEV)
    plan = fq.Plan(layers, xs, ys, 1, ws)
    for trial, pattern in enumerate([[4, 8, 16, 8, 4], [8, 8, 4, 4, 16], [4, 4, 4, 4, 4], [16, 8, 16, 4, 8]]):
        pattern = [b if (b != 16 or i % 2 == 0) else 8 for i, b in enumerate(pattern)]
        for y in ys:
            y.fill_(float("nan"))
        bits_dev = torch.tensor(pattern, dtype=torch.int32, device=DEV)
        plan.run(bits_dev)
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
            y1 = gpu_linear(layers[i], b, xs_np[i])
            assert np.array_equal(y.view(np.uint16), y1.view(np.uint16)), (trial, i, b)
    # an entry whose bit-width is not attached (or not 4/8/16) is skipped, y untouched
    for y in ys:
        y.fill_(3.0)
    plan.run(torch.tensor([4, 16, 0, 8, 4], dtype=torch.int32, device=DEV))
    torch.cuda.synchronize()
    assert torch.all(ys[1] == 3.0) and torch.all(ys[2] == 3.0)
    assert not torch.all(ys[0] == 3.0)


# ------------------------------------------------------------------ entropy / KL

def _check_entropy(a, b):
    R, V = a.shape
    H_ref, KL_ref = oracle.entropy_kl(a, b)
    a_dev = to_dev(a)
    b_dev = to_dev(b) if b is not None else None
    H = torch.full((R,), float("nan"), dtype=torch.float32, device=DEV)
    KL = torch.full((R,), float("nan"), dtype=torch.float32, device=DEV) if b is not None else None
    fq.fq_entropy_kl(a_dev, b_dev, R, V, H, KL)
    torch.cuda.synchronize()
    Hn = H.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(Hn - H_ref) <= TOL_E * np.abs(H_ref) + FLOOR_E), np.abs(Hn - H_ref).max()
    if b is not None:
        KLn = KL.cpu().numpy().astype(np.float64)
        assert np.all(np.abs(KLn - KL_ref) <= TOL_E * np.abs(KL_ref) + FLOOR_E), \
            (np.abs(KLn - KL_ref) / np.abs(KL_ref)).max()
    return Hn


@pytest.mark.parametrize("R,V", [(1, 32000), (3, 32000), (2, 128256), (5, 1000), (4, 7), (2, 1), (600, 4096),
                                 (3, 32001), (2, 4099)])
def test_entropy_kl_matches_oracle(R, V):
    a, b = synth.logits_pair(0, "par/ent/%dx%d" % (R, V), R, V)
    _check_entropy(a, b)
    _check_entropy(a, None)


def test_entropy_kl_special_cases():
    V = 32000
    uni = np.full((1, V), 2.5, dtype=np.float32)
    H = _check_entropy(uni, uni.copy())
    assert abs(H[0] - math.log(V)) < 1e-4 * math.log(V)
    # far-apart distributions (large KL), one dominant logit, -inf entries
    a, _ = synth.logits_pair(1, "par/ent/far/a", 2, 4096)
    b, _ = synth.logits_pair(2, "par/ent/far/b", 2, 4096)
    _check_entropy(a, b)
    dom = np.zeros((1, 1024), dtype=np.float32)
    dom[0, 77] = 50.0
    _check_entropy(dom, dom + np.float32(1.0))
    m = synth.logits_pair(3, "par/ent/inf", 1, 2048)[0]
    m[0, ::3] = -np.inf
    _check_entropy(m, m + synth.normal_f32(3, "par/ent/inf/n", 2048, 0.1).reshape(1, -1))
    # unaligned base pointer (row 1 of an odd-V tensor) takes the scalar path
    a3, b3 = synth.logits_pair(4, "par/ent/odd", 2, 1001)
    _check_entropy(a3[1:], b3[1:])


def test_entropy_r0_is_a_no_op():
    H = torch.zeros(1, device=DEV)
    fq.fq_entropy_kl(H, None, 0, 8, H, None)


@pytest.mark.parametrize("M,shapes", [(1, [(256, 1024), (100, 1408)]), (4, [(256, 1024), (100, 1408)]),
                                      (2, [(40, 256), (24, 128)]), (16, [(11008, 512)] * 24)])
def test_plan_status_reports_entries_that_could_not_be_served(M, shapes):
    # M = 1: the batch-1 kernel; 4: the register-fed batch kernel; 2 with few rows: its K-split
    # form; 16 with many rows: the streaming kernel behind plan_order_kernel
    layers, xs, ys = [], [], []
    for i, (N, K) in enumerate(shapes):
        w = synth.weight(0, "par/status/w%d" % (i % 3), N, K, 0.02)
        layer, _ = make_layer(w, (4, 8) if i else (4,))
        layers.append(layer)
        xs.append(to_dev(synth.activations(0, "par/status/x%d" % (i % 3), M, K)))
        ys.append(torch.full((M, N), 3.0, dtype=torch.float16, device=DEV))
    ws = torch.empty(fq.Plan.workspace_bytes(len(layers)), dtype=torch.uint8, device=DEV)
    plan = fq.Plan(layers, xs, ys, M, ws)
    n = len(layers)
    plan.run(torch.tensor([4] * n, dtype=torch.int32, device=DEV))
    assert plan.status() == (0, 0)
    assert not torch.all(ys[0] == 3.0)
    ys[0].fill_(3.0)
    plan.run(torch.tensor([8] + [4] * (n - 1), dtype=torch.int32, device=DEV))   # entry 0 holds no 8-bit copy
    assert plan.status() == (0, 1)
    assert torch.all(ys[0] == 3.0) and not torch.all(ys[1] == 3.0)
    plan.run(torch.tensor([4] * n, dtype=torch.int32, device=DEV))               # the flag stays
    assert plan.status() == (0, 1)
    plan2 = fq.Plan(layers, xs, ys, M, ws)                                        # a new plan starts clean
    plan2.run(torch.tensor([4] + [5] * (n - 1), dtype=torch.int32, device=DEV))  # 5 is no width at all
    assert plan2.status() == (0, 1)


@pytest.mark.parametrize("bits", [2, 4, 8])
def test_linear_prefill_small_and_uneven_magnitudes(bits):
    # the GEMM's operand carries the group's scale as a half: weights of magnitude 2e-4 give 8-bit
    # scales near 5e-6, below the normal range of a half, and rows 2^-20 apart in magnitude share
    # a tile; the result must be as close to the oracle as for weights of ordinary size
    M, N, K = 96, 300, 1024
    w = synth.weight(0, "par/pre/small/%d" % bits, N, K, 2e-4, outlier_p=0.001).astype(np.float32)
    w[100:200] *= 2.0 ** -6                       # some rows far smaller still (halves: down to ~1e-7)
    w[200:] *= 2.0 ** 5
    w[:, 512:] *= 2.0 ** -3                       # and the scales of a row differ from group to group
    w = w.astype(np.float16)
    x = synth.activations(0, "par/pre/small/x", M, K)
    layer, packed = make_layer(w, (bits,))
    c, s, z = (t.cpu().numpy() for t in packed[bits])
    assert s.min() < 2.0 ** -15                   # below the smallest normal half
    y_ref = oracle.linear(x, c, s, z, bits)
    y = gpu_linear(layer, bits, x)
    for lo, hi in ((0, 100), (100, 200), (200, 300)):   # each band against its own magnitude
        assert rel_err(y[:, lo:hi], y_ref[:, lo:hi]) <= TOL_Y, (lo, hi)

"""GPU parity for the W8A8 prefill path (Sec. 4.1 / 4.3 / 4.5), the entropy/KL reduction over
binary16 logits and the ascending-KL replacement order (Sec. 4.3), through the C ABI against
the CPU oracle on identical seeded inputs.  Bars: activation codes, scales, group sums and
the order bit-exact; fp16 outputs within 2e-3 (max-abs normalised); entropy and KL within
1e-4 relative (absolute floor 1e-7)."""
import numpy as np
import pytest
import torch

import oracle
import synth
import paper_2506_12024_amd as fq
from gpu_util import DEV, make_layer, rel_err, to_dev

pytestmark = pytest.mark.gpu

TOL_Y = 2e-3
TOL_E = 1e-4
FLOOR_E = 1e-7


def gpu_quantize_act(x: np.ndarray):
    M, K = x.shape
    x_dev = to_dev(x)
    xq = torch.full((M, K), 99, dtype=torch.int8, device=DEV)
    sx = torch.full((M,), float("nan"), dtype=torch.float32, device=DEV)
    xsum = torch.full((K // 128, M), -7, dtype=torch.int32, device=DEV)
    fq.fq_quantize_act(x_dev, M, K, xq, sx, xsum)
    torch.cuda.synchronize()
    return xq, sx, xsum


# ------------------------------------------------------------------ activation quantizer

@pytest.mark.parametrize("M,K", [(1, 128), (5, 1408), (33, 4096), (300, 2048), (2, 28672)])
def test_quantize_act_bit_exact(M, K):
    x = synth.activations(0, "par/act/%dx%d" % (M, K), M, K)
    if M > 2:
        x[1] *= np.float16(40.0)
        x[2] *= np.float16(0.003)
    xq_ref, sx_ref = oracle.quantize_act(x)
    xq, sx, xsum = gpu_quantize_act(x)
    assert np.array_equal(xq.cpu().numpy(), xq_ref)
    assert np.array_equal(sx.cpu().numpy().view(np.uint32), sx_ref.view(np.uint32))
    sums = xq_ref.astype(np.int32).reshape(M, K // 128, 128).sum(axis=2).T
    assert np.array_equal(xsum.cpu().numpy(), sums)


def test_quantize_act_degenerate_rows():
    x = np.zeros((6, 256), dtype=np.float16)
    x[1, :8] = [127.0, 2.5, 3.5, -2.5, -3.5, 0.5, 1.5, -0.5]      # s = 1: ties to even
    x[2, 5] = -4.0                                                 # one negative entry
    x[3, :] = synth.normal_f16(1, "par/act/sub", 256, 1e-6)        # subnormal halves
    x[4, 0], x[4, 1] = 65504.0, -65504.0                           # fp16 extremes
    x[4, 2:] = np.linspace(-3e4, 3e4, 254)
    x[5, :] = (np.resize(np.arange(-127, 128), 256) / 128.0)       # on the grid
    xq_ref, sx_ref = oracle.quantize_act(x)
    xq, sx, _ = gpu_quantize_act(x)
    assert np.array_equal(xq.cpu().numpy(), xq_ref)
    assert np.array_equal(sx.cpu().numpy().view(np.uint32), sx_ref.view(np.uint32))
    assert sx_ref[0] == 1.0 and not xq_ref[0].any()


# ------------------------------------------------------------------ W8A8 linear

def _w8a8(layer, x: np.ndarray):
    M, K = x.shape
    xq, sx, xsum = gpu_quantize_act(x)
    y = torch.full((M, layer.N), float("nan"), dtype=torch.float16, device=DEV)
    fq.fq_linear_w8a8(layer, xq, sx, xsum, M, y)
    torch.cuda.synchronize()
    return y.cpu().numpy(), xq.cpu().numpy(), sx.cpu().numpy()


@pytest.mark.parametrize("M,N,K", [(33, 100, 1408), (128, 256, 1024), (300, 200, 2048), (257, 130, 128),
                                   (64, 129, 4096), (1, 64, 256), (129, 513, 384)])
def test_linear_w8a8_matches_oracle(M, N, K):
    w = synth.weight(0, "par/w8a8/%dx%d" % (N, K), N, K, 0.015, outlier_p=0.001)
    x = synth.activations(0, "par/w8a8/x/%dx%d" % (M, K), M, K)
    layer, packed = make_layer(w, (8,))
    y, xq, sx = _w8a8(layer, x)
    c, s, z = (t.cpu().numpy() for t in packed[8])
    y_ref = oracle.linear_w8a8(xq, sx, c, s, z)
    assert y.shape == (M, N)
    assert not np.isnan(y.astype(np.float32)).any()
    assert rel_err(y, y_ref) <= TOL_Y
    for m in (0, M // 2, M - 1):
        assert rel_err(y[m:m + 1], y_ref[m:m + 1]) <= TOL_Y, m


def test_linear_w8a8_both_token_tilings_on_a_full_grid():
    # The kernel for groups of 128 exists with 192 and with 128 tokens per workgroup and the launcher
    # takes the one whose rounds (one workgroup per compute unit at a time) cost less.  One round or
    # less always goes to 128 tokens, which is what the shapes above exercise; 1536 x 8192 is 8 x 32 =
    # 256 tiles of 192 tokens (one round on 256 compute units) against 384 tiles of 128 (two), so
    # this launch runs the 192-token kernel.  Weight rows sampled from every part of a tile, all
    # tokens; both launches repeatable bit for bit.
    M, N, K = 1536, 8192, 256
    w = synth.weight(0, "par/w8a8/grid/w", N, K, 0.015, outlier_p=0.001)
    x = synth.activations(0, "par/w8a8/grid/x", M, K)
    layer, packed = make_layer(w, (8,))
    y, xq, sx = _w8a8(layer, x)
    y2, _, _ = _w8a8(layer, x)
    assert np.array_equal(y.view(np.uint16), y2.view(np.uint16))
    assert not np.isnan(y.astype(np.float32)).any()
    c, s, z = (t.cpu().numpy() for t in packed[8])
    for n0 in (0, 31, 63, 64, 127, 255, 256, 4095, 4160, 8190):
        y_ref = oracle.linear_w8a8(xq, sx, c, s, z, row0=n0, rows=2)
        assert rel_err(y[:, n0:n0 + 2], y_ref) <= TOL_Y, n0
    for m in (0, 95, 96, 191, 192, 767, 1535):
        y_ref = oracle.linear_w8a8(xq[m:m + 1], sx[m:m + 1], c, s, z)
        assert rel_err(y[m:m + 1], y_ref) <= TOL_Y, m


def test_linear_w8a8_skewed_zero_points():
    # one-signed groups (z = 0 or 255) make the zero-point term as large as it gets
    rng = np.random.default_rng(21)
    N, K, M = 96, 640, 70
    w = np.abs(synth.weight(0, "par/w8a8/skew", N, K, 0.02)).astype(np.float16)
    w[::2] = -w[::2]
    x = (np.abs(synth.activations(0, "par/w8a8/skew/x", M, K)) * rng.choice([1.0, 0.2], size=(M, 1))).astype(np.float16)
    layer, packed = make_layer(w, (8,))
    c, s, z = (t.cpu().numpy() for t in packed[8])
    assert set(np.unique(z)) <= {0, 255}
    y, xq, sx = _w8a8(layer, x)
    assert rel_err(y, oracle.linear_w8a8(xq, sx, c, s, z)) <= TOL_Y


def test_linear_w8a8_integer_case_exact():
    # integer weights with s = 1 (each group spans 0..255) and integer activations with
    # max 127 (s_x = 1): the result is the integer matrix product, exact in binary16
    rng = np.random.default_rng(9)
    M, N, K = 130, 70, 640
    w = rng.integers(0, 3, size=(N, K))
    w[:, 0::128] = 0
    w[:, 1::128] = 255
    x = rng.integers(-2, 3, size=(M, K))
    x[:, 0] = 127                       # meets the weight 0: adds nothing
    x[:, 1::128] = 0                    # the 255s add nothing either
    layer, packed = make_layer(w.astype(np.float16), (8,))
    y, xq, sx = _w8a8(layer, x.astype(np.float16))
    assert np.all(sx == 1.0) and np.array_equal(xq.astype(np.int64), x)
    expect = x @ w.T
    assert np.abs(expect).max() <= 2048
    assert np.array_equal(y.astype(np.float64), expect.astype(np.float64))


# ------------------------------------------------------------------ one scale per weight row (group = K)

@pytest.mark.parametrize("sym", [False, True])
@pytest.mark.parametrize("N,K", [(300, 1024), (5, 128), (64, 28672), (2049, 384)])
def test_quantize_per_row_bit_exact(N, K, sym):
    w = synth.weight(0, "par/rowq/%dx%d" % (N, K), N, K, 0.02, outlier_p=0.001)
    w[0] = 0                                         # an all-zero row: s = 1
    if N > 2:
        w[1] = np.abs(w[1])                          # a one-signed row: z = 0
    c_ref, s_ref, z_ref = (oracle.quantize_sym if sym else oracle.quantize)(w, 8, group=K)
    assert fq.fq_packed_sizes(N, K, 8, K) == (N * K, N * 4, N)
    c = torch.full((N * K,), 0xAA, dtype=torch.uint8, device=DEV)
    sc = torch.full((N,), float("nan"), dtype=torch.float32, device=DEV)
    z = torch.full((N,), 77, dtype=torch.uint8, device=DEV)
    (fq.fq_quantize_sym if sym else fq.fq_quantize)(to_dev(w), N, K, 8, K, c, sc, z)
    torch.cuda.synchronize()
    assert np.array_equal(c.cpu().numpy().reshape(N, K), c_ref)
    assert np.array_equal(sc.cpu().numpy().view(np.uint32), s_ref.reshape(N).view(np.uint32))
    assert np.array_equal(z.cpu().numpy(), z_ref.reshape(N))


@pytest.mark.parametrize("M,N,K", [(33, 100, 1408), (128, 256, 1024), (300, 200, 2048), (257, 130, 128),
                                   (64, 129, 4096), (1, 64, 256), (129, 513, 384), (200, 300, 28672)])
def test_linear_w8a8_per_row_matches_oracle(M, N, K):
    w = synth.weight(0, "par/w8a8row/%dx%d" % (N, K), N, K, 0.015, outlier_p=0.001)
    x = synth.activations(0, "par/w8a8row/x/%dx%d" % (M, K), M, K)
    layer, packed = make_layer(w, (8,), group=K)
    y, xq, sx = _w8a8(layer, x)
    c, s, z = (t.cpu().numpy() for t in packed[8])
    y_ref = oracle.linear_w8a8(xq, sx, c, s, z, group=K)
    assert y.shape == (M, N)
    assert not np.isnan(y.astype(np.float32)).any()
    assert rel_err(y, y_ref) <= TOL_Y
    for m in (0, M // 2, M - 1):
        assert rel_err(y[m:m + 1], y_ref[m:m + 1]) <= TOL_Y, m


def test_linear_w8a8_per_row_whole_and_half_tiles_on_a_full_grid():
    # 2560 x 8192 is 10 x 32 = 320 tiles of 256 x 256, 40 per XCD: on 32 compute units per XCD one
    # round of whole tiles and a last quarter round, which the launcher runs as half tiles in a second
    # launch -- the small shapes above fit half a round and run as half tiles only.  Weight rows and
    # tokens sampled from both kinds of tile; repeatable bit for bit.
    M, N, K = 2560, 8192, 256
    w = synth.weight(0, "par/w8a8row/grid/w", N, K, 0.015, outlier_p=0.001)
    x = synth.activations(0, "par/w8a8row/grid/x", M, K)
    layer, packed = make_layer(w, (8,), group=K)
    y, xq, sx = _w8a8(layer, x)
    y2, _, _ = _w8a8(layer, x)
    assert np.array_equal(y.view(np.uint16), y2.view(np.uint16))
    assert not np.isnan(y.astype(np.float32)).any()
    c, s, z = (t.cpu().numpy() for t in packed[8])
    for n0 in (0, 63, 64, 255, 256, 1023, 1024, 4095, 6400, 7000, 8190):
        y_ref = oracle.linear_w8a8(xq, sx, c, s, z, group=K, row0=n0, rows=2)
        assert rel_err(y[:, n0:n0 + 2], y_ref) <= TOL_Y, n0
    for m in (0, 127, 128, 255, 256, 1279, 1280, 2559):
        y_ref = oracle.linear_w8a8(xq[m:m + 1], sx[m:m + 1], c, s, z, group=K)
        assert rel_err(y[m:m + 1], y_ref) <= TOL_Y, m


def test_linear_w8a8_per_row_skewed_zero_points_and_integer_case():
    # one-signed rows (z = 0 or 255) make the zero-point term as large as it gets
    N, K, M = 96, 640, 70
    w = np.abs(synth.weight(0, "par/w8a8row/skew", N, K, 0.02)).astype(np.float16)
    w[::2] = -w[::2]
    x = np.abs(synth.activations(0, "par/w8a8row/skew/x", M, K)).astype(np.float16)
    layer, packed = make_layer(w, (8,), group=K)
    c, s, z = (t.cpu().numpy() for t in packed[8])
    assert set(np.unique(z)) <= {0, 255}
    y, xq, sx = _w8a8(layer, x)
    assert rel_err(y, oracle.linear_w8a8(xq, sx, c, s, z, group=K)) <= TOL_Y
    # integer weights with s = 1 (every row spans 0 .. 255), integer activations with max 127 (s_x = 1):
    # the result is the integer matrix product, exact in binary16
    rng = np.random.default_rng(9)
    M, N, K = 130, 70, 640
    w = rng.integers(0, 3, size=(N, K))
    w[:, 0] = 0
    w[:, 1] = 255
    x = rng.integers(-2, 3, size=(M, K))
    x[:, 0] = 127                       # meets the weight 0: adds nothing
    x[:, 1] = 0                         # the 255s add nothing either
    layer, packed = make_layer(w.astype(np.float16), (8,), group=K)
    assert torch.all(packed[8][1] == 1.0) and torch.all(packed[8][2] == 0)
    y, xq, sx = _w8a8(layer, x.astype(np.float16))
    assert np.all(sx == 1.0) and np.array_equal(xq.astype(np.int64), x)
    expect = x @ w.T
    assert np.abs(expect).max() <= 2048
    assert np.array_equal(y.astype(np.float64), expect.astype(np.float64))


def test_per_row_copies_are_served_by_w8a8_only():
    w = synth.weight(0, "par/w8a8row/refuse", 64, 256, 0.02)
    layer, _ = make_layer(w, (8,), group=256)
    x = to_dev(synth.activations(0, "par/w8a8row/refuse/x", 1, 256))
    y = torch.zeros((1, 64), dtype=torch.float16, device=DEV)
    with pytest.raises(fq.FlexqError):
        fq.fq_linear(layer, 8, x, 1, y)
    with pytest.raises(fq.FlexqError):
        ws = torch.empty(fq.Plan.workspace_bytes(1), dtype=torch.uint8, device=DEV)
        fq.Plan([layer], [x], [y], 1, ws)
    with pytest.raises(fq.FlexqError):
        layer.attach(4, x, x, x)


def test_linear_w8a8_close_to_weight_only_result():
    # the activation rounding bound of the oracle pins, on the GPU results
    M, N, K = 64, 128, 1024
    w = synth.weight(0, "par/w8a8/cmp", N, K, 0.015)
    x = synth.activations(0, "par/w8a8/cmp/x", M, K)
    layer, packed = make_layer(w, (8,))
    c, s, z = (t.cpu().numpy() for t in packed[8])
    y88, xq, sx = _w8a8(layer, x)
    y816 = oracle.linear(x, c, s, z, 8).astype(np.float64)
    w_hat = oracle.dequant(c, s, z, 8).astype(np.float64)
    bound = 0.5 * sx[:, None].astype(np.float64) * np.abs(w_hat).sum(axis=1)[None, :]
    slack = TOL_Y * np.abs(y816).max()
    assert np.all(np.abs(y88.astype(np.float64) - y816) <= bound + slack)


# ------------------------------------------------------------------ entropy / KL over fp16 logits

def _check_entropy_f16(a: np.ndarray, b, skip: int = 0):
    """`skip` leading rows are uploaded but not reduced: with an odd V the remaining rows start
    at an address that is only 2-byte aligned."""
    a_dev, b_dev = to_dev(a)[skip:], None if b is None else to_dev(b)[skip:]
    a, b = a[skip:], None if b is None else b[skip:]
    R, V = a.shape
    H_ref, KL_ref = oracle.entropy_kl(a.astype(np.float32), None if b is None else b.astype(np.float32))
    H = torch.full((R,), float("nan"), device=DEV)
    KL = torch.full((R,), float("nan"), device=DEV) if b is not None else None
    fq.fq_entropy_kl_f16(a_dev, b_dev, R, V, H, KL)
    torch.cuda.synchronize()
    Hn = H.cpu().numpy().astype(np.float64)
    assert np.all(np.abs(Hn - H_ref) <= TOL_E * np.abs(H_ref) + FLOOR_E)
    if b is not None:
        KLn = KL.cpu().numpy().astype(np.float64)
        assert np.all(np.abs(KLn - KL_ref) <= TOL_E * np.abs(KL_ref) + FLOOR_E)


@pytest.mark.parametrize("R,V", [(1, 4096), (4, 11008), (16, 4096), (3, 1001), (2, 4099), (700, 1024), (2, 1)])
def test_entropy_kl_f16_matches_oracle(R, V):
    a, b = synth.logits_pair(0, "par/ent16/%dx%d" % (R, V), R, V)
    a16, b16 = a.astype(np.float16), b.astype(np.float16)
    _check_entropy_f16(a16, b16)
    _check_entropy_f16(a16, None)
    if R > 1 and V % 2:
        _check_entropy_f16(a16, b16, skip=1)


def test_entropy_kl_f16_on_linear_outputs():
    # what the layer-ranking analysis reduces: a layer's output at 8 bits against 4 bits
    N, K, M = 4096, 4096, 4
    w = synth.weight(0, "par/ent16/lin/w", N, K, 0.02, outlier_p=0.001)
    x = synth.activations(0, "par/ent16/lin/x", M, K)
    layer, _ = make_layer(w, (4, 8))
    x_dev = to_dev(x)
    y8 = torch.empty((M, N), dtype=torch.float16, device=DEV)
    y4 = torch.empty((M, N), dtype=torch.float16, device=DEV)
    fq.fq_linear(layer, 8, x_dev, M, y8)
    fq.fq_linear(layer, 4, x_dev, M, y4)
    torch.cuda.synchronize()
    _check_entropy_f16(y8.cpu().numpy(), y4.cpu().numpy())


# ------------------------------------------------------------------ replacement order

def _gpu_rank(v: np.ndarray) -> np.ndarray:
    v2 = v if v.ndim == 2 else v[:, None]
    n, m = v2.shape
    order = torch.full((max(n, 1),), -1, dtype=torch.int32, device=DEV)
    fq.fq_rank_ascending(to_dev(np.ascontiguousarray(v2, dtype=np.float32)), n, m, order)
    torch.cuda.synchronize()
    return order.cpu().numpy()[:n]


@pytest.mark.parametrize("n,m", [(1, 1), (7, 1), (224, 1), (224, 16), (256, 3), (257, 1), (1000, 5), (5000, 1)])
def test_rank_matches_oracle(n, m):
    rng = np.random.default_rng(100 + n + m)
    v = (rng.integers(0, max(2, n // 3), size=(n, m)) * 1e-3).astype(np.float32)  # plenty of ties
    assert np.array_equal(_gpu_rank(v), oracle.rank_ascending(v))


def test_rank_nan_and_cancellation():
    v = np.array([2.0, np.nan, 1.0, np.nan, 0.5], dtype=np.float32)
    assert _gpu_rank(v).tolist() == oracle.rank_ascending(v).tolist() == [4, 2, 0, 1, 3]
    w = np.array([[1e8, 1.0, -1e8], [0.5, 0.0, 0.0], [1e8, 2.0, -1e8]], dtype=np.float32)
    assert _gpu_rank(w).tolist() == oracle.rank_ascending(w).tolist()


def test_rank_feeds_the_scheduler():
    # the order written on the device is what fq_sched_init takes as its event list
    n = 12
    kl = synth.normal_f32(0, "par/rank/kl", n, 1.0).astype(np.float32) ** 2
    order = torch.empty(n, dtype=torch.int32, device=DEV)
    fq.fq_rank_ascending(to_dev(kl), n, 1, order)
    bits = torch.full((n,), 8, dtype=torch.int32, device=DEV)
    ev_bits = torch.full((n,), 4, dtype=torch.int32, device=DEV)
    state = torch.zeros(fq.fq_sched_state_bytes(2), dtype=torch.uint8, device=DEV)
    fq.fq_sched_init(state, 2, 100.0, 3, order, ev_bits, n, bits)
    H = torch.zeros(1, dtype=torch.float32, device=DEV)      # PPLE = 1 < 100: triggers when full
    fq.fq_sched_step(state, H)
    fq.fq_sched_step(state, H)
    torch.cuda.synchronize()
    ref_order = oracle.rank_ascending(kl)
    expect = np.full(n, 8, dtype=np.int32)
    expect[ref_order[:3]] = 4
    assert np.array_equal(bits.cpu().numpy(), expect)


def test_prefill_paths_repeatable_on_a_large_tile_grid():
    # Several workgroup tiles per CU and many steps: repeated launches must agree bit for bit
    # (a wavefront reading a buffer another one is already refilling shows up here), and a
    # sample of columns from every part of a workgroup tile must match the oracle.
    M, N, K = 600, 1024, 4096
    w = synth.weight(0, "par/rep/w", N, K, 0.015)
    x = synth.activations(0, "par/rep/x", M, K)
    layer, packed = make_layer(w, (4, 8))
    x_dev = to_dev(x)
    xq = torch.empty((M, K), dtype=torch.int8, device=DEV)
    sx = torch.empty(M, dtype=torch.float32, device=DEV)
    xsum = torch.empty((K // 128, M), dtype=torch.int32, device=DEV)
    fq.fq_quantize_act(x_dev, M, K, xq, sx, xsum)
    runs = {"w4": [], "w8": [], "w8a8": []}
    for _ in range(3):
        for key, fn in (("w4", lambda y: fq.fq_linear(layer, 4, x_dev, M, y)),
                        ("w8", lambda y: fq.fq_linear(layer, 8, x_dev, M, y)),
                        ("w8a8", lambda y: fq.fq_linear_w8a8(layer, xq, sx, xsum, M, y))):
            y = torch.full((M, N), float("nan"), dtype=torch.float16, device=DEV)
            fn(y)
            runs[key].append(y)
    torch.cuda.synchronize()
    for key, ys in runs.items():
        assert torch.equal(ys[0].view(torch.int16), ys[1].view(torch.int16)), key
        assert torch.equal(ys[0].view(torch.int16), ys[2].view(torch.int16)), key
    cols = [0, 31, 32, 63, 64, 127, 128, 129, 191, 192, 255, 256, 511, 700, 1023]
    ms = [0, 95, 96, 191, 192, 255, 256, 599]
    xq_h, sx_h = xq.cpu().numpy(), sx.cpu().numpy()
    for key, bits in (("w4", 4), ("w8", 8), ("w8a8", 8)):
        c, s, z = (t.cpu().numpy() for t in packed[bits])
        y = runs[key][0].cpu().numpy()
        for n in cols:
            if key == "w8a8":
                ref = oracle.linear_w8a8(xq_h[ms], sx_h[ms], c[n:n + 1], s[n:n + 1], z[n:n + 1])
            else:
                ref = oracle.linear(x[ms], c[n:n + 1], s[n:n + 1], z[n:n + 1], bits)
            got = y[ms, n].astype(np.float64)
            assert np.abs(got - ref[:, 0].astype(np.float64)).max() <= TOL_Y * np.abs(y.astype(np.float64)).max(), (key, n)

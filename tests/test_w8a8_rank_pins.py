"""Pins for the oracle's W8A8 prefill routines and its replacement-order routine.

W8A8: Sec. 4.1 / 4.3 / 4.5 (the prefill multiplies 8-bit weights by 8-bit activations on
integer matrix units).  Activations are quantized per token with the symmetric form stated
after Sec. 2.2 Eq. (3): z = 0, Xmax = -Xmin = max |x|, 2^8 - 2 levels.  Replacement order:
Sec. 4.3 (linear layers with smaller KL divergence are replaced first).

Nothing here compares the oracle with itself: closed forms, hand-worked ties, bounds that the
arithmetic fixes, a plain-Python brute force, numpy's integer matmul and numpy's stable sort.
"""
import numpy as np
import pytest

import oracle
import synth

G = 128


# ---------------------------------------------------------------- activation quantizer

def test_act_on_grid_closed_form():
    # x = j / 128 for j in [-127, 127]: max |x| = 127/128, s = (254/128) / 254 = 2^-7 exactly,
    # every quotient is the integer j
    j = np.resize(np.arange(-127, 128), 512).astype(np.int32)
    x = (j / 128.0).astype(np.float16)[None, :]
    xq, sx = oracle.quantize_act(x)
    assert sx[0] == np.float32(2.0 ** -7)
    assert np.array_equal(xq[0].astype(np.int32), j)


def test_act_ties_round_to_even_and_sign():
    # max |x| = 127 gives s = 1; 2.5 -> 2, 3.5 -> 4, -2.5 -> -2, -3.5 -> -4, 0.5 -> 0, 1.5 -> 2
    x = np.zeros((1, 128), dtype=np.float16)
    x[0, :8] = [127.0, 2.5, 3.5, -2.5, -3.5, 0.5, 1.5, -0.5]
    xq, sx = oracle.quantize_act(x)
    assert sx[0] == np.float32(1.0)
    assert xq[0, :8].tolist() == [127, 2, 4, -2, -4, 0, 2, 0]
    assert not xq[0, 8:].any()


def test_act_zero_row_and_per_token_scale():
    x = np.zeros((3, 256), dtype=np.float16)
    x[1, 5] = -4.0          # a single negative entry: max |x| = 4, it must map to -127
    x[2, 7] = 1.0
    x[2, 9] = 0.25
    xq, sx = oracle.quantize_act(x)
    assert sx[0] == np.float32(1.0) and not xq[0].any()
    assert sx[1] == np.float32(8.0) / np.float32(254.0) and xq[1, 5] == -127
    assert sx[2] == np.float32(2.0) / np.float32(254.0)
    assert xq[2, 7] == 127 and xq[2, 9] == 32          # 0.25 * 127 = 31.75 -> 32


def test_act_invariants_random():
    x = synth.activations(0, "pins/act", 16, 1024)
    x[3] *= np.float16(30.0)                           # rows of very different magnitude
    x[7] *= np.float16(0.01)
    xq, sx = oracle.quantize_act(x)
    xf = x.astype(np.float64)
    assert xq.min() >= -127 and xq.max() <= 127
    amax = np.abs(xf).max(axis=1)
    # the scale is the binary32 quotient of 2 max|x| by 254
    assert np.array_equal(sx, ((amax + amax).astype(np.float32) / np.float32(254.0)).astype(np.float32))
    # the largest entry of each row sits on the last level, the error is at most half a step
    for m in range(x.shape[0]):
        k = int(np.argmax(np.abs(xf[m])))
        assert abs(int(xq[m, k])) == 127 and np.sign(xq[m, k]) == np.sign(xf[m, k])
    err = np.abs(xf - xq.astype(np.float64) * sx[:, None].astype(np.float64))
    assert np.all(err <= 0.5 * sx[:, None].astype(np.float64) * (1 + 2.0 ** -12))


def test_act_matches_second_writing_in_numpy_float32():
    x = synth.activations(0, "pins/act2", 8, 512)
    xq, sx = oracle.quantize_act(x)
    xf = x.astype(np.float32)
    amax = np.abs(xf).max(axis=1)
    s = ((amax + amax) / np.float32(254.0)).astype(np.float32)
    q = np.clip(np.rint((xf / s[:, None]).astype(np.float32)), -127, 127).astype(np.int8)
    assert np.array_equal(sx, s) and np.array_equal(xq, q)


def test_act_rejects_non_finite():
    x = np.ones((2, 128), dtype=np.float16)
    x[1, 3] = np.inf
    with pytest.raises(ValueError):
        oracle.quantize_act(x)


# ---------------------------------------------------------------- W8A8 linear

def _small_layer(seed, N, K, outlier_p=0.0):
    w = synth.weight(seed, "pins/w8a8/w", N, K, 0.02, outlier_p=outlier_p)
    return w, oracle.quantize(w, 8)


def test_w8a8_brute_force_python():
    N, K, M = 5, 256, 3
    w, (c, s, z) = _small_layer(3, N, K)
    x = synth.activations(3, "pins/w8a8/x", M, K)
    xq, sx = oracle.quantize_act(x)
    y = oracle.linear_w8a8(xq, sx, c, s, z)
    for m in range(M):
        for n in range(N):
            acc = 0.0
            for k in range(K):
                g = k // G
                wv = np.float32(np.float32(int(c[n, k]) - int(z[n, g])) * s[n, g])
                xv = np.float32(np.float32(int(xq[m, k])) * sx[m])
                acc += float(xv) * float(wv)
            assert y[m, n] == np.float16(acc), (m, n)


def test_w8a8_integer_case_is_an_integer_matmul():
    # s = 1, z = 0 weights (codes are the weights) and integer activations with max 127
    # (sx = 1): y is the plain integer matrix product, exactly representable in binary16
    rng = np.random.default_rng(5)
    N, K, M = 16, 128, 4
    c = rng.integers(0, 3, size=(N, K)).astype(np.uint8)
    s = np.ones((N, 1), dtype=np.float32)
    z = np.zeros((N, 1), dtype=np.uint8)
    xi = rng.integers(-3, 4, size=(M, K)).astype(np.int32)
    xi[:, 0] = 127
    c[:, 0] = 0                                          # keep the sums small
    xq, sx = oracle.quantize_act(xi.astype(np.float16))
    assert np.all(sx == 1.0) and np.array_equal(xq.astype(np.int32), xi)
    y = oracle.linear_w8a8(xq, sx, c, s, z)
    ref = xi @ c.astype(np.int32).T
    assert np.abs(ref).max() < 2048
    assert np.array_equal(y.astype(np.int32), ref)


def test_w8a8_equals_weight_only_linear_when_x_is_on_the_int8_grid():
    # activations that the 8-bit grid represents exactly (sx a power of two) lose nothing, so
    # the W8A8 product is the fp16-activation product of the same INT8 weights
    rng = np.random.default_rng(6)
    N, K, M = 24, 384, 5
    w, (c, s, z) = _small_layer(6, N, K, outlier_p=0.01)
    xi = rng.integers(-127, 128, size=(M, K)).astype(np.int32)
    xi[:, 1] = 127
    x = (xi / 256.0).astype(np.float16)                  # s = 2 * (127/256) / 254 = 2^-8
    xq, sx = oracle.quantize_act(x)
    assert np.all(sx == np.float32(2.0 ** -8)) and np.array_equal(xq.astype(np.int32), xi)
    y88 = oracle.linear_w8a8(xq, sx, c, s, z)
    y816 = oracle.linear(x, c, s, z, 8)
    assert np.array_equal(y88.view(np.uint16), y816.view(np.uint16))


def test_w8a8_within_the_activation_rounding_bound_of_the_weight_only_result():
    # |y_w8a8 - y_w8a16| <= sum_k |w_hat[n][k]| * sx[m] / 2, plus the two binary16 roundings
    N, K, M = 32, 512, 6
    w, (c, s, z) = _small_layer(7, N, K, outlier_p=0.001)
    x = synth.activations(7, "pins/w8a8/xb", M, K)
    xq, sx = oracle.quantize_act(x)
    y88 = oracle.linear_w8a8(xq, sx, c, s, z).astype(np.float64)
    y816 = oracle.linear(x, c, s, z, 8).astype(np.float64)
    w_hat = oracle.dequant(c, s, z, 8).astype(np.float64)
    bound = 0.5 * sx[:, None].astype(np.float64) * np.abs(w_hat).sum(axis=1)[None, :] * (1 + 2.0 ** -12)
    half_ulp = 2.0 ** -11 * (np.abs(y88) + np.abs(y816))
    assert np.all(np.abs(y88 - y816) <= bound + half_ulp)
    # and the two are not the same thing: activation rounding does show
    assert np.abs(y88 - y816).max() > 0


def test_w8a8_row_slice_and_three_groups():
    # distinct scale and zero per group; a wrong group index or a transposed operand shows
    N, K, M = 4, 384, 2
    c = np.zeros((N, K), dtype=np.uint8)
    s = np.array([[0.5, 2.0, 4.0]] * N, dtype=np.float32) * np.arange(1, N + 1, dtype=np.float32)[:, None]
    z = np.array([[1, 2, 3]] * N, dtype=np.uint8)
    c[:, 0], c[:, 128], c[:, 256] = 3, 5, 4          # (3-1)*.5=1, (5-2)*2=6, (4-3)*4=4  (times n+1)
    c[:, 1:128], c[:, 129:256], c[:, 257:] = 1, 2, 3  # zero weight elsewhere
    xq = np.zeros((M, K), dtype=np.int8)
    xq[0, 0], xq[0, 128], xq[0, 256] = 1, 10, 100
    xq[1, 0], xq[1, 128], xq[1, 256] = -2, 0, 7
    sx = np.array([1.0, 0.5], dtype=np.float32)
    y = oracle.linear_w8a8(xq, sx, c, s, z).astype(np.float64)
    ref0 = 1 * 1 + 10 * 6 + 100 * 4
    ref1 = 0.5 * (-2 * 1 + 7 * 4)
    for n in range(N):
        assert y[0, n] == ref0 * (n + 1) and y[1, n] == ref1 * (n + 1)
    part = oracle.linear_w8a8(xq, sx, c, s, z, row0=1, rows=2).astype(np.float64)
    assert np.array_equal(part, y[:, 1:3])


# ---------------------------------------------------------------- replacement order

def test_rank_hand_case():
    v = np.array([0.30, 0.05, 0.20, 0.05, 0.00], dtype=np.float32)
    assert oracle.rank_ascending(v).tolist() == [4, 1, 3, 2, 0]


def test_rank_matches_numpy_stable_sort_with_ties():
    rng = np.random.default_rng(11)
    v = rng.integers(0, 50, size=1000).astype(np.float32) * np.float32(1e-3)
    assert np.array_equal(oracle.rank_ascending(v), np.argsort(v, kind="stable").astype(np.int32))


def test_rank_by_row_sum_in_double():
    rng = np.random.default_rng(12)
    v = rng.random((300, 7)).astype(np.float32)
    key = v.astype(np.float64).sum(axis=1)
    assert np.array_equal(oracle.rank_ascending(v), np.argsort(key, kind="stable").astype(np.int32))
    # an entry whose rows cancel in binary32 but not in double keeps its place
    w = np.array([[1e8, 1.0, -1e8], [0.5, 0.0, 0.0], [1e8, 2.0, -1e8]], dtype=np.float32)
    assert oracle.rank_ascending(w).tolist() == [1, 0, 2]


def test_rank_nan_last_and_is_a_permutation():
    v = np.array([2.0, np.nan, 1.0, np.nan, 0.5], dtype=np.float32)
    assert oracle.rank_ascending(v).tolist() == [4, 2, 0, 1, 3]
    assert oracle.rank_ascending(np.zeros(0, dtype=np.float32)).size == 0


def test_quantize_with_one_group_per_row_closed_form_and_equivalence():
    # group = K: the row is one group.  On-grid row j * 2^-10, j in [-127, 128]: s = 2^-10, z = 127, codes j + 127
    # exactly (Sec. 2.2 Eq. 2 with Xmin / Xmax over the row); and a row quantized as one group of K equals
    # the same values quantized as a 1 x K matrix with group K -- whatever the other rows hold
    K = 256
    j = np.arange(-127, 129)
    w = np.zeros((3, K), dtype=np.float16)
    w[0] = (j * 2.0 ** -10).astype(np.float16)
    w[1] = np.linspace(-0.3, 0.1, K).astype(np.float16)
    w[2] = np.linspace(0.0, 7.0, K).astype(np.float16)
    c, s, z = oracle.quantize(w, 8, group=K)
    assert s.shape == (3, 1) and z.shape == (3, 1)
    assert s[0, 0] == np.float32(2.0 ** -10) and z[0, 0] == 127
    assert np.array_equal(c[0].astype(np.int64), j + 127)
    for r in range(3):
        c1, s1, z1 = oracle.quantize(w[r:r + 1], 8, group=K)
        assert np.array_equal(c1[0], c[r]) and s1[0, 0] == s[r, 0] and z1[0, 0] == z[r, 0]
    assert z[2, 0] == 0 and c[2].max() == 255 and c[2].min() == 0
    # the W8A8 linear with one group per row against the integer definition written out
    rng = np.random.default_rng(3)
    xq = rng.integers(-127, 128, size=(4, K)).astype(np.int8)
    sx = np.array([0.5, 1.0, 0.25, 2.0], dtype=np.float32)
    y = oracle.linear_w8a8(xq, sx, c, s, z, group=K).astype(np.float64)
    ref = (xq.astype(np.int64) @ (c.astype(np.int64) - z.astype(np.int64)).T) * s[:, 0].astype(np.float64) * sx[:, None].astype(np.float64)
    assert np.all(np.abs(y - ref) <= np.abs(ref) * 2.0 ** -10 + 1e-6)

"""Pins for the 2-bit path of the CPU oracle (Table 1 lists 2-, 3- and 4-bit models; Sec. 2.2
Eq. (2) and (3) with n = 2): hand-worked cases, the byte layout (four codes per byte), invariants,
brute force, and agreement with routines of the oracle that are written separately (the
quantize-dequantize routine) or that a library provides (integer matmul)."""
import os

import numpy as np
import pytest

import oracle
import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
G = 128


def _unpack2(codes):
    codes = np.asarray(codes, dtype=np.uint8)
    out = np.empty(codes.shape[:-1] + (codes.shape[-1] * 4,), dtype=np.int64)
    for p in range(4):
        out[..., p::4] = (codes >> (2 * p)) & 3
    return out


def _cases():
    out = []
    with open(os.path.join(GOLDEN, "quant2_hand_cases.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            bits, vals, s, z, codes = [p.strip() for p in line.split(";")]
            out.append((int(bits), [float(v) for v in vals.split()], float(s), int(z), [int(c) for c in codes.split()]))
    return out


@pytest.mark.parametrize("case", _cases())
def test_quantize_2bit_hand_cases(case):
    bits, vals, s_exp, z_exp, codes_exp = case
    assert bits == 2
    w = np.zeros((1, G), dtype=np.float16)
    w[0, :len(vals)] = vals
    assert np.array_equal(w[0, :len(vals)].astype(np.float64), vals), "case values must be exact halves"
    codes, scales, zeros = oracle.quantize(w, 2, G)
    assert codes.shape == (1, G // 4)
    assert scales[0, 0] == np.float32(s_exp) and zeros[0, 0] == z_exp
    q = _unpack2(codes)[0]
    assert list(q[:len(vals)]) == codes_exp
    assert np.all(q[len(vals):] == z_exp)  # the padding zeros sit on the zero point


def test_pack_2bit_bytes_hand_case():
    # codes 1,2,3,0,3,3,0,1 at k = 0..7 (s = 1, z = 0: the code is the value):
    # byte 0 = 1 | 2<<2 | 3<<4 | 0<<6 = 0x39, byte 1 = 3 | 3<<2 | 0<<4 | 1<<6 = 0x4F
    w = np.zeros((1, G), dtype=np.float16)
    w[0, :8] = [1, 2, 3, 0, 3, 3, 0, 1]
    codes, scales, zeros = oracle.quantize(w, 2, G)
    assert scales[0, 0] == 1.0 and zeros[0, 0] == 0
    assert list(codes[0, :3]) == [0x39, 0x4F, 0x00]


def test_pack_2bit_every_code_at_every_position():
    for pos in range(4):
        for c in range(4):
            w = np.zeros((2, G), dtype=np.float16)
            w[:, 100] = 3  # fixes the range: s = 1, z = 0
            k = 20 + pos
            w[1, k] = c
            codes, _, _ = oracle.quantize(w, 2, G)
            byte = int(codes[1, k // 4])
            assert (byte >> (2 * pos)) & 3 == c
            assert byte & ~(3 << (2 * pos)) & 0xFF == 0
            assert codes[0, k // 4] == 0  # the other row is untouched: rows follow each other


def test_quantize_2bit_invariants_random():
    w = synth.weight(3, "pins2/w", 64, 1024, 0.02, outlier_p=0.001)
    codes, scales, zeros = oracle.quantize(w, 2, G)
    q = _unpack2(codes)
    assert q.min() >= 0 and q.max() <= 3 and zeros.max() <= 3
    wf = w.astype(np.float64)
    s = np.repeat(scales.astype(np.float64), G, axis=1)
    z = np.repeat(zeros.astype(np.float64), G, axis=1)
    w_hat = (q - z) * s
    assert np.all(np.abs(w_hat - wf) <= 0.5 * s * (1 + 2.0 ** -12) + 2.0 ** -22 * np.abs(wf))
    assert np.allclose(oracle.dequant(codes, scales, zeros, 2, G).astype(np.float64), w_hat, rtol=1e-7, atol=0)
    wg, qg = wf.reshape(64, -1, G), q.reshape(64, -1, G)
    assert np.all(np.take_along_axis(qg, wg.argmin(-1)[..., None], -1)[..., 0] == 0)
    assert np.all(np.take_along_axis(qg, wg.argmax(-1)[..., None], -1)[..., 0] == 3)
    assert np.allclose(scales, (wg.max(-1) - wg.min(-1)) / 3, rtol=2e-7)
    # the same scales, zero points and codes as the separately written quantize-dequantize routine
    fq = oracle.fake_quantize(w, 2, G)
    assert np.array_equal(fq.view(np.uint16), w_hat.astype(np.float32).astype(np.float16).view(np.uint16))


def test_quantize_2bit_is_nearest_level_brute_force():
    w = synth.weight(4, "pins2/bf", 8, 256, 0.02, outlier_p=0.01)
    codes, scales, zeros = oracle.quantize(w, 2, G)
    q = _unpack2(codes)
    levels = np.arange(4, dtype=np.float64)
    wf = w.astype(np.float64)
    for n in range(8):
        for k in range(256):
            s, z = float(scales[n, k // G]), float(zeros[n, k // G])
            d = np.abs((levels - z) * s - wf[n, k])
            if q[n, k] != int(d.argmin()):
                assert abs(d[q[n, k]] - d.min()) <= 1e-4 * s, (n, k)


def test_quantize_sym_2bit_codes():
    # symmetric variant at n = 2: 2^n - 2 = 2 levels of width s = max|w|, integers -1 .. 1, stored
    # as code = q + 2 with zero point 2
    w = np.zeros((1, G), dtype=np.float16)
    w[0, :6] = [0.5, -0.5, 0.2, 0.3, -0.26, 0.25]  # 0.25 / 0.5 = 0.5 -> 0 (half to even)
    codes, scales, zeros = oracle.quantize_sym(w, 2, G)
    assert scales[0, 0] == np.float32(0.5) and zeros[0, 0] == 2
    assert list(_unpack2(codes)[0, :6]) == [3, 1, 2, 3, 1, 2]
    assert np.all(_unpack2(codes)[0, 6:] == 2)


def test_linear_2bit_integer_case_reduces_to_integer_matvec():
    rng = np.random.default_rng(12)
    N, K, M = 12, 384, 3
    w = rng.integers(0, 4, size=(N, K))
    w[:, 0::G] = 0
    w[:, 1::G] = 3
    x = rng.integers(-2, 3, size=(M, K))
    codes, scales, zeros = oracle.quantize(w.astype(np.float16), 2, G)
    assert np.all(scales == 1.0) and np.all(zeros == 0)
    y = oracle.linear(x.astype(np.float16), codes, scales, zeros, 2, G)
    assert np.array_equal(y.astype(np.float64), (x @ w.T).astype(np.float64))


def test_linear_2bit_matches_double_triple_loop_tiny():
    w = synth.weight(6, "pins2/lin", 3, 384, 0.02)
    w[:, 128:256] *= np.float16(3.0)
    w[:, 256:384] += np.float16(0.05)
    x = synth.activations(6, "pins2/x", 2, 384)
    codes, scales, zeros = oracle.quantize(w, 2, G)
    assert len(set(scales[0])) == 3
    q = _unpack2(codes)
    y = oracle.linear(x, codes, scales, zeros, 2, G)
    for m in range(2):
        for n in range(3):
            acc = 0.0
            for k in range(384):
                g = k // 128
                acc += float(x[m, k]) * float(np.float32(np.float32(q[n, k] - int(zeros[n, g])) * scales[n, g]))
            assert y[m, n] == np.float16(acc)


def test_linear_2bit_representable_weights_agree_at_4_and_8_bits():
    # weights on a 4-level grid: the 2-, 4- and 8-bit copies dequantize to (nearly) the same
    # matrix, so the three outputs agree within the rounding of the wider scales
    rng = np.random.default_rng(22)
    N, K = 16, 512
    j = rng.integers(-1, 3, size=(N, K))
    j[:, 0::G] = -1
    j[:, 1::G] = 2
    w = (j / 64.0).astype(np.float16)
    x = synth.activations(7, "pins2/x248", 1, K)
    y2 = oracle.linear(x, *oracle.quantize(w, 2, G), 2, G).astype(np.float64)
    y4 = oracle.linear(x, *oracle.quantize(w, 4, G), 4, G).astype(np.float64)
    y8 = oracle.linear(x, *oracle.quantize(w, 8, G), 8, G).astype(np.float64)
    exact = (x.astype(np.float64) @ (j / 64.0).T)
    assert np.array_equal(y2, exact.astype(np.float16).astype(np.float64))  # s = 1/64, z = 1: exact
    assert np.abs(y2 - y4).max() <= 2e-3 * np.abs(y2).max()
    assert np.abs(y2 - y8).max() <= 2e-3 * np.abs(y2).max()


def test_2bit_rejects_bad_input():
    with pytest.raises(ValueError):
        oracle.quantize(np.zeros((2, 200), dtype=np.float16), 2, G)
    with pytest.raises(ValueError):
        oracle.quantize(np.zeros((2, 12), dtype=np.float16), 2, 6)  # a group must hold whole bytes

"""Pins for the 3-bit path of the CPU oracle (Table 1 lists 2-, 3- and 4-bit models; Sec. 2.2
Eq. (2) and (3) with n = 3): hand-worked cases, the byte layout (blocks of 12 bytes for 32 codes:
8 bytes of low bit pairs, one 32-bit word of high bits), invariants, brute force, and agreement
with routines of the oracle that are written separately (the quantize-dequantize routine) or that a
library provides (integer matmul).  The unpacking below is written from the statement of the
format, not taken from the oracle."""
import os

import numpy as np
import pytest

import oracle
import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
G = 128


def _high_bit_place(i):
    # codes 0..7, 16..23, 8..15, 24..31 of a block from bit 0 of the word up
    return (i % 8) + 16 * ((i // 8) % 2) + 8 * (i // 16)


def _unpack3(codes):
    codes = np.asarray(codes, dtype=np.uint8)
    rows, nbytes = codes.shape
    K = nbytes * 8 // 3
    out = np.zeros((rows, K), dtype=np.int64)
    blocks = codes.reshape(rows, K // 32, 12)
    words = (blocks[..., 8].astype(np.uint32) | (blocks[..., 9].astype(np.uint32) << 8) |
             (blocks[..., 10].astype(np.uint32) << 16) | (blocks[..., 11].astype(np.uint32) << 24))
    for i in range(32):
        lo = (blocks[..., i // 4] >> (2 * (i % 4))) & 3
        hi = (words >> _high_bit_place(i)) & 1
        out[:, i::32] = lo.astype(np.int64) + 4 * hi.astype(np.int64)
    return out


def _cases():
    out = []
    with open(os.path.join(GOLDEN, "quant3_hand_cases.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            bits, vals, s, z, codes = [p.strip() for p in line.split(";")]
            out.append((int(bits), [float(v) for v in vals.split()], float(s), int(z), [int(c) for c in codes.split()]))
    return out


@pytest.mark.parametrize("case", _cases())
def test_quantize_3bit_hand_cases(case):
    bits, vals, s_exp, z_exp, codes_exp = case
    assert bits == 3
    w = np.zeros((1, G), dtype=np.float16)
    w[0, :len(vals)] = vals
    assert np.array_equal(w[0, :len(vals)].astype(np.float64), vals), "case values must be exact halves"
    codes, scales, zeros = oracle.quantize(w, 3, G)
    assert codes.shape == (1, G * 3 // 8)
    assert scales[0, 0] == np.float32(s_exp) and zeros[0, 0] == z_exp
    q = _unpack3(codes)[0]
    assert list(q[:len(vals)]) == codes_exp
    assert np.all(q[len(vals):] == z_exp)  # the padding zeros sit on the zero point


def test_pack_3bit_bytes_hand_case():
    # s = 1, z = 0 (a 7 elsewhere in the group fixes the range), so the code is the value.
    # Code 4 (low pair 0, high bit 1) at k = 1, 9, 18, 27 and code 3 (low pair 3, high bit 0) at
    # k = 5.  Low plane: only k = 5 has low bits, byte 1 = 3 << 2 = 0x0C.  High word: code 1 ->
    # bit 1 (byte 8 = 0x02); code 9 -> bit 16 + 1 (byte 10 = 0x02); code 18 -> bit 8 + 2 (byte 9 =
    # 0x04); code 27 -> bit 24 + 3 (byte 11 = 0x08).
    w = np.zeros((1, G), dtype=np.float16)
    w[0, [1, 9, 18, 27]] = 4
    w[0, 5] = 3
    w[0, 100] = 7
    codes, scales, zeros = oracle.quantize(w, 3, G)
    assert scales[0, 0] == 1.0 and zeros[0, 0] == 0
    assert list(codes[0, :12]) == [0x00, 0x0C, 0, 0, 0, 0, 0, 0, 0x02, 0x04, 0x02, 0x08]
    # block 3 (k = 96 .. 127) holds the 7 at its place 4: low pair 3 in byte 1, high bit at bit 4
    assert list(codes[0, 36:48]) == [0x00, 0x03, 0, 0, 0, 0, 0, 0, 0x10, 0, 0, 0]
    assert not codes[0, 12:36].any()


def test_pack_3bit_every_code_at_every_position():
    for pos in range(32):
        for c in range(8):
            w = np.zeros((2, G), dtype=np.float16)
            w[:, 100] = 7  # fixes the range: s = 1, z = 0
            k = 32 + pos
            w[1, k] = c
            codes, _, _ = oracle.quantize(w, 3, G)
            blk = codes[1, 12:24].astype(np.int64)
            assert (blk[pos // 4] >> (2 * (pos % 4))) & 3 == c & 3
            word = int(blk[8]) | int(blk[9]) << 8 | int(blk[10]) << 16 | int(blk[11]) << 24
            assert word == (c >> 2) << _high_bit_place(pos)
            assert sum(int(b) for b in blk[:8]) == (c & 3) << (2 * (pos % 4))
            assert not codes[0, 12:24].any()  # the other row is untouched: rows follow each other
    assert sorted(_high_bit_place(i) for i in range(32)) == list(range(32))


def test_quantize_3bit_invariants_random():
    w = synth.weight(3, "pins3/w", 64, 1024, 0.02, outlier_p=0.001)
    codes, scales, zeros = oracle.quantize(w, 3, G)
    q = _unpack3(codes)
    assert q.min() >= 0 and q.max() <= 7 and zeros.max() <= 7
    wf = w.astype(np.float64)
    s = np.repeat(scales.astype(np.float64), G, axis=1)
    z = np.repeat(zeros.astype(np.float64), G, axis=1)
    w_hat = (q - z) * s
    assert np.all(np.abs(w_hat - wf) <= 0.5 * s * (1 + 2.0 ** -12) + 2.0 ** -22 * np.abs(wf))
    assert np.allclose(oracle.dequant(codes, scales, zeros, 3, G).astype(np.float64), w_hat, rtol=1e-7, atol=0)
    wg, qg = wf.reshape(64, -1, G), q.reshape(64, -1, G)
    assert np.all(np.take_along_axis(qg, wg.argmin(-1)[..., None], -1)[..., 0] == 0)
    assert np.all(np.take_along_axis(qg, wg.argmax(-1)[..., None], -1)[..., 0] == 7)
    assert np.allclose(scales, (wg.max(-1) - wg.min(-1)) / 7, rtol=2e-7)
    # the same scales, zero points and codes as the separately written quantize-dequantize routine
    fq = oracle.fake_quantize(w, 3, G)
    assert np.array_equal(fq.view(np.uint16), w_hat.astype(np.float32).astype(np.float16).view(np.uint16))


def test_quantize_3bit_is_nearest_level_brute_force():
    w = synth.weight(4, "pins3/bf", 8, 256, 0.02, outlier_p=0.01)
    codes, scales, zeros = oracle.quantize(w, 3, G)
    q = _unpack3(codes)
    levels = np.arange(8, dtype=np.float64)
    wf = w.astype(np.float64)
    for n in range(8):
        for k in range(256):
            s, z = float(scales[n, k // G]), float(zeros[n, k // G])
            d = np.abs((levels - z) * s - wf[n, k])
            if q[n, k] != int(d.argmin()):
                assert abs(d[q[n, k]] - d.min()) <= 1e-4 * s, (n, k)


def test_quantize_sym_3bit_codes():
    # symmetric variant at n = 3: 2^n - 2 = 6 steps, s = 2 max|w| / 6, integers -3 .. 3, stored as
    # code = q + 4 with zero point 4.  max|w| = 0.75: s = 0.25; 0.125 / 0.25 = 0.5 -> 0 and
    # 0.375 / 0.25 = 1.5 -> 2 (half to even)
    w = np.zeros((1, G), dtype=np.float16)
    w[0, :7] = [0.75, -0.75, 0.25, -0.5, 0.125, 0.375, -0.3]
    codes, scales, zeros = oracle.quantize_sym(w, 3, G)
    assert scales[0, 0] == np.float32(0.25) and zeros[0, 0] == 4
    assert list(_unpack3(codes)[0, :7]) == [7, 1, 5, 2, 4, 6, 3]
    assert np.all(_unpack3(codes)[0, 7:] == 4)


def test_linear_3bit_integer_case_reduces_to_integer_matvec():
    rng = np.random.default_rng(13)
    N, K, M = 12, 384, 3
    w = rng.integers(0, 8, size=(N, K))
    w[:, 0::G] = 0
    w[:, 1::G] = 7
    x = rng.integers(-2, 3, size=(M, K))
    codes, scales, zeros = oracle.quantize(w.astype(np.float16), 3, G)
    assert np.all(scales == 1.0) and np.all(zeros == 0)
    y = oracle.linear(x.astype(np.float16), codes, scales, zeros, 3, G)
    assert np.array_equal(y.astype(np.float64), (x @ w.T).astype(np.float64))


def test_linear_3bit_matches_double_triple_loop_tiny():
    w = synth.weight(6, "pins3/lin", 3, 384, 0.02)
    w[:, 128:256] *= np.float16(3.0)
    w[:, 256:384] += np.float16(0.05)
    x = synth.activations(6, "pins3/x", 2, 384)
    codes, scales, zeros = oracle.quantize(w, 3, G)
    assert len(set(scales[0])) == 3
    q = _unpack3(codes)
    y = oracle.linear(x, codes, scales, zeros, 3, G)
    for m in range(2):
        for n in range(3):
            acc = 0.0
            for k in range(384):
                g = k // 128
                acc += float(x[m, k]) * float(np.float32(np.float32(q[n, k] - int(zeros[n, g])) * scales[n, g]))
            assert y[m, n] == np.float16(acc)


def test_linear_3bit_weights_on_the_grid_are_exact():
    # weights on an 8-level grid: s = 1/64, z = 3, every product and sum exactly representable
    # (unlike at 2 bits the 4- and 8-bit copies cannot hold this grid: 7 divides neither 15 nor 255)
    rng = np.random.default_rng(23)
    N, K = 16, 512
    j = rng.integers(-3, 5, size=(N, K))
    j[:, 0::G] = -3
    j[:, 1::G] = 4
    w = (j / 64.0).astype(np.float16)
    x = rng.integers(-3, 4, size=(1, K)).astype(np.float16)
    codes, scales, zeros = oracle.quantize(w, 3, G)
    assert np.all(scales == np.float32(1 / 64)) and np.all(zeros == 3)
    y3 = oracle.linear(x, codes, scales, zeros, 3, G).astype(np.float64)
    exact = (x.astype(np.float64) @ (j / 64.0).T)
    assert np.array_equal(y3, exact.astype(np.float16).astype(np.float64))


def test_3bit_rejects_bad_input():
    with pytest.raises(ValueError):
        oracle.quantize(np.zeros((2, 200), dtype=np.float16), 3, G)
    with pytest.raises(ValueError):
        oracle.quantize(np.zeros((2, 48), dtype=np.float16), 3, 16)  # a group must hold whole blocks of 32

"""Pins for the 3-bit path of the CPU oracle (Table 1 lists 2-, 3- and 4-bit models; Sec. 2.2
Eq. (2) and (3) with n = 3): hand-worked cases, the byte layout (blocks of 12 bytes for 32 codes:
three little-endian words of ten whole codes each, the two last codes spread over the words' bits
15 and 31), invariants, brute force, and agreement with routines of the oracle that are written
separately (the quantize-dequantize routine) or that a library provides (integer matmul).  The
unpacking below is written from the statement of the format, not taken from the oracle."""
import os

import numpy as np
import pytest

import oracle
import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
G = 128


def _bit_place(i, t):
    """Bit t of code i of a block, counted over the block's 96 bits (byte b holds bits 8 b .. 8 b + 7)."""
    if i < 30:
        word, r = divmod(i, 10)
        half, p = divmod(r, 5)
        return 32 * word + 16 * half + 3 * p + t
    return 32 * t + 15 + 16 * (i - 30)


def _block_int(blk):
    return sum(int(b) << (8 * j) for j, b in enumerate(blk))


def _unpack3(codes):
    codes = np.asarray(codes, dtype=np.uint8)
    rows, nbytes = codes.shape
    K = nbytes * 8 // 3
    out = np.zeros((rows, K), dtype=np.int64)
    blocks = codes.reshape(rows, K // 32, 12).astype(np.int64)
    for i in range(32):
        for t in range(3):
            place = _bit_place(i, t)
            out[:, i::32] += ((blocks[..., place // 8] >> (place % 8)) & 1) << t
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
    # Block 0: code 4 (bit 2 alone) at k = 1, 9, 18, 27 and code 3 (bits 0 and 1) at k = 5.
    #   k = 1:  word 0, low half, place 1: bits 3..5, bit 2 of the code is bit 5       -> byte 0 = 0x20
    #   k = 5:  word 0, high half, place 0: bits 16..18, the code's bits 0, 1          -> byte 2 = 0x03
    #   k = 9:  word 0, high half, place 4: bits 28..30, bit 30                        -> byte 3 = 0x40
    #   k = 18: word 1, high half, place 3: bits 25..27, bit 27                        -> byte 7 = 0x08
    #   k = 27: word 2, high half, place 2: bits 22..24, bit 24                        -> byte 11 = 0x01
    # Block 1: code 5 (bits 0, 2) at its place 30: bit 15 of words 0 and 2 -> bytes 1 and 9 = 0x80;
    #   code 6 (bits 1, 2) at its place 31: bit 31 of words 1 and 2 -> bytes 7 and 11 = 0x80.
    # Block 3: the 7 at its place 4: word 0, low half, place 4: bits 12..14 -> byte 1 = 0x70.
    w = np.zeros((1, G), dtype=np.float16)
    w[0, [1, 9, 18, 27]] = 4
    w[0, 5] = 3
    w[0, 32 + 30] = 5
    w[0, 32 + 31] = 6
    w[0, 100] = 7
    codes, scales, zeros = oracle.quantize(w, 3, G)
    assert scales[0, 0] == 1.0 and zeros[0, 0] == 0
    assert list(codes[0, :12]) == [0x20, 0, 0x03, 0x40, 0, 0, 0, 0x08, 0, 0, 0, 0x01]
    assert list(codes[0, 12:24]) == [0, 0x80, 0, 0, 0, 0, 0, 0x80, 0, 0x80, 0, 0x80]
    assert list(codes[0, 36:48]) == [0, 0x70, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0]
    assert not codes[0, 24:36].any()


def test_pack_3bit_every_code_at_every_position():
    for pos in range(32):
        for c in range(8):
            w = np.zeros((2, G), dtype=np.float16)
            w[:, 100] = 7  # fixes the range: s = 1, z = 0
            k = 32 + pos
            w[1, k] = c
            codes, _, _ = oracle.quantize(w, 3, G)
            expect = sum(((c >> t) & 1) << _bit_place(pos, t) for t in range(3))
            assert _block_int(codes[1, 12:24]) == expect
            assert not codes[0, 12:24].any()  # the other row is untouched: rows follow each other
    # every bit of a block belongs to exactly one (code, bit)
    assert sorted(_bit_place(i, t) for i in range(32) for t in range(3)) == list(range(96))
    # a whole code keeps its three bits together, inside one 16-bit half of one word
    for i in range(30):
        a = _bit_place(i, 0)
        assert [_bit_place(i, t) for t in range(3)] == [a, a + 1, a + 2] and a // 16 == (a + 2) // 16


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

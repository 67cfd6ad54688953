"""Pins for the CPU oracle: every routine of oracle/flexq_oracle.c is checked
against something other than itself -- hand-worked cases (tests/golden/),
closed forms, invariants the mathematics fixes, brute force on tiny inputs and
independent library routines (numpy's float16 conversion, integer matmul).

Citations: quantizer Sec. 2.2 Eq. (2); dequantizer Eq. (3); softmax Sec. 2.3;
entropy inside PPLE Sec. 4.2 Eq. (5); KL of Sec. 3.1 taken between two
next-token distributions.
"""
import math
import os

import numpy as np
import pytest

import oracle
import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
G = 128


# ---------------------------------------------------------------- half conversions

def test_half_to_float_all_patterns_match_numpy():
    bits = np.arange(65536, dtype=np.uint16)
    ref = bits.view(np.float16).astype(np.float32)
    got = np.array([oracle.half_to_float(int(b)) for b in bits], dtype=np.float32)
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), ref[~nan].view(np.uint32))


def test_double_to_half_matches_numpy_rne():
    rng = np.random.default_rng(1)
    vals = np.concatenate([
        rng.normal(0, 1, 4000), rng.normal(0, 1e-5, 2000), rng.normal(0, 3000, 2000),
        # exact ties between neighbouring halves, subnormal edge, overflow edge
        np.array([1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 2.0 ** -25, 3 * 2.0 ** -25, 2.0 ** -24,
                  65504.0, 65519.999, 65520.0, 70000.0, -65520.0, 0.0, -0.0, 5.960464477539063e-08]),
    ])
    with np.errstate(over="ignore"):
        ref = vals.astype(np.float16).view(np.uint16)
    got = np.array([oracle.double_to_half(float(v)) for v in vals], dtype=np.uint16)
    assert np.array_equal(got, ref)


def test_synth_f16_conversion_matches_numpy():
    lib = synth._load()
    rng = np.random.default_rng(2)
    vals = np.concatenate([rng.normal(0, 0.02, 3000), rng.normal(0, 1e-6, 1000), rng.normal(0, 4e4, 500),
                           [2.0 ** -25, 2.0 ** -24, 1 + 2.0 ** -11, 65520.0, 65519.0]]).astype(np.float32)
    with np.errstate(over="ignore"):
        ref = vals.astype(np.float16).view(np.uint16)
    got = np.array([lib.fqs_f32_to_f16(float(v)) for v in vals], dtype=np.uint16)
    assert np.array_equal(got, ref)


# ---------------------------------------------------------------- quantizer, Eq. (2)

def _golden_cases():
    out = []
    with open(os.path.join(GOLDEN, "quant_hand_cases.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            bits, vals, s, z, codes = [p.strip() for p in line.split(";")]
            fill = 0.0
            if vals.startswith("fill="):
                first, vals = vals.split(None, 1)
                fill = float(first[5:])
            out.append((int(bits), [float(v) for v in vals.split()], float(s), int(z),
                        [int(c) for c in codes.split()], fill))
    return out


def _unpack(codes, bits):
    codes = np.asarray(codes, dtype=np.uint8)
    if bits == 8:
        return codes.astype(np.int64)
    out = np.empty(codes.shape[:-1] + (codes.shape[-1] * 2,), dtype=np.int64)
    out[..., 0::2] = codes & 0xF
    out[..., 1::2] = codes >> 4
    return out


@pytest.mark.parametrize("case", _golden_cases())
def test_quantize_hand_cases(case):
    bits, vals, s_exp, z_exp, codes_exp, fill = case
    w = np.full((1, G), fill, dtype=np.float16)
    w[0, :len(vals)] = vals
    assert np.array_equal(w[0, :len(vals)].astype(np.float64), vals), "case values must be exact halves"
    codes, scales, zeros = oracle.quantize(w, bits, G)
    assert scales[0, 0] == np.float32(s_exp)
    assert zeros[0, 0] == z_exp
    q = _unpack(codes, bits)[0]
    assert list(q[:len(vals)]) == codes_exp
    # padding zeros map to the zero point (or 0 for the all-zero group)
    if fill == 0.0:
        assert np.all(q[len(vals):] == z_exp)


def test_pack_bytes_hand_case():
    # Codes 1,2,3,4 at k = 0..3 (4-bit): byte0 = 1 | 2<<4 = 0x21, byte1 = 3 | 4<<4 = 0x43.
    # Obtained with s = 1, z = 0 (all-positive group whose maximum is 15).
    w = np.zeros((1, G), dtype=np.float16)
    w[0, :5] = [1, 2, 3, 4, 15]
    codes, scales, zeros = oracle.quantize(w, 4, G)
    assert scales[0, 0] == 1.0 and zeros[0, 0] == 0
    assert list(codes[0, :3]) == [0x21, 0x43, 0x0F]
    w8 = np.zeros((1, G), dtype=np.float16)
    w8[0, :3] = [7, 200, 255]
    codes8, s8, z8 = oracle.quantize(w8, 8, G)
    assert list(codes8[0, :4]) == [7, 200, 255, 0]


def test_pack_every_code_at_both_parities():
    # s = 1, z = 0: the code equals the (integer) weight; place each of the 16 codes at an
    # even and at an odd index and read it back from the documented nibble.
    for parity in (0, 1):
        for c in range(16):
            w = np.zeros((1, G), dtype=np.float16)
            w[0, 100] = 15  # fixes the range
            pos = 10 + parity
            w[0, pos] = c
            codes, _, _ = oracle.quantize(w, 4, G)
            byte = int(codes[0, pos // 2])
            assert ((byte >> 4) if parity else (byte & 0xF)) == c
            other = (byte & 0xF) if parity else (byte >> 4)
            assert other == 0


@pytest.mark.parametrize("bits", [4, 8])
def test_quantize_invariants_random(bits):
    # codes in [0, 2^n-1]; |dequant - w| <= s/2 up to binary32 rounding of X/s + z;
    # group minimum -> code 0, maximum -> 2^n - 1 when the group straddles 0.
    w = synth.weight(3, "pins/w", 64, 1024, 0.02, outlier_p=0.001)
    codes, scales, zeros = oracle.quantize(w, bits, G)
    q = _unpack(codes, bits)
    qmax = (1 << bits) - 1
    assert q.min() >= 0 and q.max() <= qmax
    assert zeros.min() >= 0 and zeros.max() <= qmax
    wf = w.astype(np.float64)
    s = np.repeat(scales.astype(np.float64), G, axis=1)
    z = np.repeat(zeros.astype(np.float64), G, axis=1)
    w_hat = (q - z) * s
    bound = 0.5 * s * (1 + 2.0 ** -12) + 2.0 ** -22 * np.abs(wf)
    assert np.all(np.abs(w_hat - wf) <= bound)
    deq = oracle.dequant(codes, scales, zeros, bits, G).astype(np.float64)
    assert np.allclose(deq, w_hat, rtol=1e-7, atol=0)
    wg = wf.reshape(64, -1, G)
    qg = q.reshape(64, -1, G)
    straddle = (wg.min(-1) < 0) & (wg.max(-1) > 0)
    assert straddle.all()
    assert np.all(np.take_along_axis(qg, wg.argmin(-1)[..., None], -1)[..., 0] == 0)
    assert np.all(np.take_along_axis(qg, wg.argmax(-1)[..., None], -1)[..., 0] == qmax)
    # scale is (max - min) / (2^n - 1) to binary32 accuracy
    assert np.allclose(scales, (wg.max(-1) - wg.min(-1)) / qmax, rtol=2e-7)


@pytest.mark.parametrize("bits", [4, 8])
def test_quantize_is_nearest_level_brute_force(bits):
    # Each code must be the level (c - z) * s closest to w among all 2^n levels, except
    # where two levels are (nearly) equidistant.
    w = synth.weight(4, "pins/bf", 8, 256, 0.02, outlier_p=0.01)
    codes, scales, zeros = oracle.quantize(w, bits, G)
    q = _unpack(codes, bits)
    levels = np.arange(1 << bits, dtype=np.float64)
    wf = w.astype(np.float64)
    for n in range(8):
        for k in range(256):
            s = float(scales[n, k // G])
            z = float(zeros[n, k // G])
            d = np.abs((levels - z) * s - wf[n, k])
            best = int(d.argmin())
            if q[n, k] != best:
                assert abs(d[q[n, k]] - d[best]) <= 1e-4 * s, (n, k, q[n, k], best)


def test_quantize_groups_are_independent():
    w = synth.weight(5, "pins/ind", 4, 512, 0.02)
    c0, s0, z0 = oracle.quantize(w, 4, G)
    w2 = w.copy()
    w2[2, 128:256] *= 3  # touch row 2, group 1 only
    c1, s1, z1 = oracle.quantize(w2, 4, G)
    mask = np.ones_like(s0, dtype=bool)
    mask[2, 1] = False
    assert np.array_equal(s0[mask], s1[mask]) and np.array_equal(z0[mask], z1[mask])
    cm = np.ones_like(c0, dtype=bool)
    cm[2, 64:128] = False
    assert np.array_equal(c0[cm], c1[cm])
    assert not np.array_equal(c0[2, 64:128], c1[2, 64:128]) or s0[2, 1] != s1[2, 1]
    # permuting rows permutes the outputs
    perm = [3, 1, 0, 2]
    cp, sp, zp = oracle.quantize(w[perm], 4, G)
    assert np.array_equal(cp, c0[perm]) and np.array_equal(sp, s0[perm]) and np.array_equal(zp, z0[perm])


def test_quantize_rejects_bad_input():
    w = np.zeros((2, 256), dtype=np.float16)
    with pytest.raises(ValueError):
        oracle.quantize(w, 5, G)
    with pytest.raises(ValueError):
        oracle.quantize(np.zeros((2, 200), dtype=np.float16), 4, G)
    w[1, 5] = np.inf
    with pytest.raises(ValueError):
        oracle.quantize(w, 4, G)


# ---------------------------------------------------------------- linear

def _int_weights(rng, N, K, bits):
    """Integer weights in [0, 2^n-1] whose every group contains 0 and 2^n-1:
    Eq. (2) then gives s = 1, z = 0, code = weight, and Eq. (3) returns it exactly."""
    qmax = (1 << bits) - 1
    w = rng.integers(0, qmax + 1, size=(N, K))
    w[:, 0::G] = 0
    w[:, 1::G] = qmax
    return w


@pytest.mark.parametrize("bits", [4, 8])
def test_linear_integer_case_reduces_to_integer_matvec(bits):
    rng = np.random.default_rng(10 + bits)
    N, K, M = 12, 384, 3   # N != K, M > 1: a transposed operand or a swapped index fails
    w = _int_weights(rng, N, K, bits)
    x = rng.integers(-2, 3, size=(M, K))
    codes, scales, zeros = oracle.quantize(w.astype(np.float16), bits, G)
    assert np.all(scales == 1.0) and np.all(zeros == 0)
    y = oracle.linear(x.astype(np.float16), codes, scales, zeros, bits, G)
    expect = x @ w.T  # exact integer arithmetic
    assert y.shape == (M, N)
    assert np.array_equal(y.astype(np.float64), expect.astype(np.float16).astype(np.float64))
    assert np.abs(expect).max() < 2048 or bits == 8  # small sums are exact halves


def test_linear_on_grid_weights_exact_rational():
    # Case A grid: w = j/64, j in [-7, 8]: s = 1/64, z = 7, dequant exact.  With integer x the
    # result is an integer multiple of 1/64, known from integer arithmetic.
    rng = np.random.default_rng(20)
    N, K, M = 5, 256, 2
    j = rng.integers(-7, 9, size=(N, K))
    j[:, 0::G] = -7
    j[:, 1::G] = 8
    x = rng.integers(-3, 4, size=(M, K))
    w = (j / 64.0).astype(np.float16)
    codes, scales, zeros = oracle.quantize(w, 4, G)
    y = oracle.linear(x.astype(np.float16), codes, scales, zeros, 4, G)
    expect = (x @ j.T) / 64.0
    assert np.array_equal(y.astype(np.float64), expect.astype(np.float16).astype(np.float64))


def test_linear_matches_double_triple_loop_tiny():
    # three groups per row with visibly different scales and zero points: every k must use
    # the scale and zero of its own group
    w = synth.weight(6, "pins/lin", 3, 384, 0.02)
    w[:, 128:256] *= np.float16(3.0)
    w[:, 256:384] += np.float16(0.05)
    x = synth.activations(6, "pins/x", 2, 384)
    for bits in (4, 8):
        codes, scales, zeros = oracle.quantize(w, bits, G)
        assert len(set(scales[0])) == 3 and len(set(zeros[0])) >= 2
        q = _unpack(codes, bits)
        y = oracle.linear(x, codes, scales, zeros, bits, G)
        for m in range(2):
            for n in range(3):
                acc = 0.0
                for k in range(384):
                    g = k // 128
                    w_hat = np.float32(np.float32(q[n, k] - int(zeros[n, g])) * scales[n, g])
                    acc += float(x[m, k]) * float(w_hat)
                assert y[m, n] == np.float16(acc)


def test_linear_4bit_representable_weights_agree_at_8_bits():
    rng = np.random.default_rng(21)
    N, K = 16, 512
    j = rng.integers(-7, 9, size=(N, K))
    j[:, 0::G] = -7
    j[:, 1::G] = 8
    w = (j / 64.0).astype(np.float16)
    x = synth.activations(7, "pins/x48", 1, K)
    y4 = oracle.linear(x, *oracle.quantize(w, 4, G), 4, G).astype(np.float64)
    y8 = oracle.linear(x, *oracle.quantize(w, 8, G), 8, G).astype(np.float64)
    assert np.abs(y4 - y8).max() <= 2e-3 * np.abs(y4).max()
    assert np.abs(y4 - y8).max() <= 2 * 2.0 ** -11 * np.abs(y4).max() + 1e-6


def test_linear_batch_rows_equal_single_rows_and_row_window():
    w = synth.weight(8, "pins/lb", 24, 256, 0.02)
    x = synth.activations(8, "pins/xb", 4, 256)
    c, s, z = oracle.quantize(w, 8, G)
    y = oracle.linear(x, c, s, z, 8, G)
    for m in range(4):
        assert np.array_equal(y[m], oracle.linear(x[m:m + 1], c, s, z, 8, G)[0])
    assert np.array_equal(oracle.linear(x, c, s, z, 8, G, row0=5, rows=7), y[:, 5:12])


def test_linear_fp16_passthrough_integer_case():
    rng = np.random.default_rng(22)
    w = rng.integers(-8, 9, size=(7, 200)).astype(np.float16)
    x = rng.integers(-4, 5, size=(3, 200)).astype(np.float16)
    y = oracle.linear(x, w, None, None, 16)
    expect = x.astype(np.int64) @ w.astype(np.int64).T
    assert np.array_equal(y.astype(np.float64), expect.astype(np.float16).astype(np.float64))


# ---------------------------------------------------------------- entropy / KL

@pytest.mark.parametrize("V", [2, 7, 32000, 128256])
def test_entropy_uniform_is_ln_V(V):
    for c in (0.0, -3.5, 11.0):
        H, _ = oracle.entropy_kl(np.full((1, V), c, dtype=np.float32))
        assert abs(H[0] - math.log(V)) <= 1e-10 * math.log(V)  # V double additions of p ln p
    if V == 32000:
        assert abs(math.exp(H[0]) - 32000) < 1e-6  # PPLE of a uniform distribution is V (Eq. 5)


def test_entropy_dominant_logit_is_zero():
    a = np.zeros((1, 1000), dtype=np.float32)
    a[0, 17] = 80.0
    H, _ = oracle.entropy_kl(a)
    # closed form: 999 entries of probability e^-80 each: H = 999 e^-80 (80 + 1) to first order
    assert abs(H[0] - 999 * 81 * math.exp(-80.0)) < 3e-32


def test_entropy_and_kl_two_entry_closed_forms():
    for t1, t2 in [(0.3, -0.2), (2.0, 2.5), (-4.0, 1.0), (0.0, 0.0)]:
        a = np.array([[t1, 0.0]], dtype=np.float32)
        b = np.array([[t2, 0.0]], dtype=np.float32)
        t1f, t2f = float(a[0, 0]), float(b[0, 0])
        p = 1 / (1 + math.exp(-t1f))
        q = 1 / (1 + math.exp(-t2f))
        h_ref = -(p * math.log(p) + (1 - p) * math.log(1 - p))
        kl_ref = p * math.log(p / q) + (1 - p) * math.log((1 - p) / (1 - q))
        H, KL = oracle.entropy_kl(a, b)
        assert abs(H[0] - h_ref) < 1e-13
        assert abs(KL[0] - kl_ref) < 1e-13
        # direction: KL(a || b) is not KL(b || a) unless they coincide
        _, KLr = oracle.entropy_kl(b, a)
        kl_rev = q * math.log(q / p) + (1 - q) * math.log((1 - q) / (1 - p))
        assert abs(KLr[0] - kl_rev) < 1e-13


def test_entropy_three_entry_brute_force():
    a = np.array([[1.0, -0.5, 2.25], [0.0, 0.0, -1e9]], dtype=np.float32)
    b = np.array([[0.5, 0.5, 2.0], [1.0, -1.0, 0.0]], dtype=np.float32)
    H, KL = oracle.entropy_kl(a, b)
    for r in range(2):
        ea = [math.exp(float(v)) for v in a[r]]
        eb = [math.exp(float(v)) for v in b[r]]
        p = [e / sum(ea) for e in ea]
        q = [e / sum(eb) for e in eb]
        h = -sum(pi * math.log(pi) for pi in p if pi > 0)
        kl = sum(pi * math.log(pi / qi) for pi, qi in zip(p, q) if pi > 0)
        assert abs(H[r] - h) < 1e-13 and abs(KL[r] - kl) < 1e-13


def test_kl_identity_nonnegativity_shift_invariance():
    a, b = synth.logits_pair(9, "pins/logits", 3, 32000)
    H, KL = oracle.entropy_kl(a, b)
    Hs, KLs = oracle.entropy_kl(a, a)
    assert np.all(KLs == 0.0)
    assert np.all(KL > 0)
    # shifting either argument by a constant (exactly representable shifts) changes nothing
    H2, KL2 = oracle.entropy_kl(a + np.float32(8.0), b - np.float32(4.0))
    a8 = (a + np.float32(8.0))
    exact = (a8 - np.float32(8.0) == a).all(axis=1)  # rows where the shift was exact in binary32
    assert np.allclose(H2, H, rtol=1e-6) and np.allclose(KL2, KL, rtol=1e-4)
    # small-noise expansion: KL ~ Var_p(delta) / 2 (loose sanity bound)
    for r in range(3):
        p = np.exp(a[r].astype(np.float64) - a[r].max())
        p /= p.sum()
        d = (b[r] - a[r]).astype(np.float64)
        var = (p * d * d).sum() - (p * d).sum() ** 2
        assert abs(KL[r] - 0.5 * var) < 0.05 * KL[r]
    assert np.all((H > 0) & (H < math.log(32000)))


def test_entropy_minus_inf_logits_carry_no_mass():
    a = np.array([[0.0, -np.inf, 0.0, -np.inf]], dtype=np.float32)
    b = np.array([[0.0, 5.0, 0.0, -3.0]], dtype=np.float32)
    H, KL = oracle.entropy_kl(a, b)
    assert abs(H[0] - math.log(2)) < 1e-15
    eb = [1.0, math.exp(5.0), 1.0, math.exp(-3.0)]
    kl = 2 * 0.5 * math.log(0.5 / (1.0 / sum(eb)))
    assert abs(KL[0] - kl) < 1e-13


def test_config0_reference_values_are_plausible():
    # The single-layer configuration: logits ~ N(0, 3), second = first + N(0, 0.1).
    # Entropy of softmax of N(0, sigma) logits is about ln V - sigma^2 / 2 for large V;
    # KL is about noise^2 / 2.
    a, b = synth.logits_pair(0, "cfg0/logits", 1, 32000)
    H, KL = oracle.entropy_kl(a, b)
    assert abs(H[0] - (math.log(32000) - 4.5)) < 0.8
    assert 0.6 * 0.005 < KL[0] < 1.4 * 0.005

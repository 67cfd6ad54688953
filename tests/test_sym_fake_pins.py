"""Pins for the oracle's symmetric quantizer and its quantize-dequantize routine.

Symmetric variant: stated after Sec. 2.2 Eq. (3) (z = 0, Xmax = -Xmin = max |X|, 2^n - 2 levels).
Quantize-dequantize at 2 .. 8 bits: how the paper obtained its low-bit accuracy numbers
(Sec. 5.1, Table 1).

Nothing here compares the oracle with itself: closed forms, symmetries, bounds the arithmetic
fixes, a second writing in numpy binary32, a plain-Python brute force, and the asymmetric
routines pinned elsewhere.
"""
import numpy as np
import pytest

import oracle
import synth

G = 128


def _unpack4(c):
    out = np.empty((c.shape[0], c.shape[1] * 2), dtype=np.int32)
    out[:, 0::2] = c & 0xF
    out[:, 1::2] = c >> 4
    return out


# ---------------------------------------------------------------- symmetric quantizer

def test_sym_closed_form_4bit():
    # w = j / 64 for j in -7 .. 7: max |w| = 7/64, s = (14/64) / 14 = 2^-6 exactly, q = j,
    # stored code = j + 8, stored zero point 8
    j = np.resize(np.arange(-7, 8), G).astype(np.int32)
    w = (j / 64.0).astype(np.float16)[None, :]
    c, s, z = oracle.quantize_sym(w, 4)
    assert s[0, 0] == np.float32(2.0 ** -6) and z[0, 0] == 8
    assert np.array_equal(_unpack4(c)[0], j + 8)


def test_sym_closed_form_8bit_and_ties_to_even():
    # max |w| = 127 gives s = 254 / 254 = 1; 2.5 -> 2, 3.5 -> 4, -2.5 -> -2, 0.5 -> 0, 1.5 -> 2
    w = np.zeros((1, G), dtype=np.float16)
    w[0, :7] = [127.0, 2.5, 3.5, -2.5, -3.5, 0.5, 1.5]
    c, s, z = oracle.quantize_sym(w, 8)
    assert s[0, 0] == np.float32(1.0) and z[0, 0] == 128
    assert (c[0, :7].astype(np.int32) - 128).tolist() == [127, 2, 4, -2, -4, 0, 2]
    assert np.all(c[0, 7:] == 128)


@pytest.mark.parametrize("bits", [4, 8])
def test_sym_invariants(bits):
    w = synth.weight(0, "pins/sym/w%d" % bits, 24, 512, 0.02, outlier_p=0.01)
    c, s, z = oracle.quantize_sym(w, bits)
    codes = _unpack4(c) if bits == 4 else c.astype(np.int32)
    off, lim = 1 << (bits - 1), (1 << (bits - 1)) - 1
    assert np.all(z == off)
    assert codes.min() >= off - lim and codes.max() <= off + lim       # 2^n - 1 values: never code 0
    wf = w.astype(np.float64).reshape(24, -1, G)
    amax = np.abs(wf).max(axis=2)
    # the scale is the binary32 quotient of 2 max|w| by 2^n - 2
    assert np.array_equal(s, ((amax + amax).astype(np.float32) / np.float32(2 * lim)).astype(np.float32))
    q = (codes - off).reshape(24, -1, G)
    # the largest entry of each group sits on the last level, with its sign; error <= s / 2
    i = np.abs(wf).argmax(axis=2)
    top = np.take_along_axis(q, i[..., None], axis=2)[..., 0]
    assert np.all(np.abs(top) == lim)
    assert np.all(np.sign(top) == np.sign(np.take_along_axis(wf, i[..., None], axis=2)[..., 0]))
    err = np.abs(wf - q * s[..., None].astype(np.float64))
    assert np.all(err <= 0.5 * s[..., None].astype(np.float64) * (1 + 2.0 ** -12))


@pytest.mark.parametrize("bits", [4, 8])
def test_sym_is_odd(bits):
    # quantizing -w mirrors the codes about the stored zero point
    w = synth.weight(1, "pins/sym/odd%d" % bits, 8, 256, 0.02)
    c1, s1, z1 = oracle.quantize_sym(w, bits)
    c2, s2, z2 = oracle.quantize_sym((-w).astype(np.float16), bits)
    a = _unpack4(c1) if bits == 4 else c1.astype(np.int32)
    b = _unpack4(c2) if bits == 4 else c2.astype(np.int32)
    assert np.array_equal(s1, s2) and np.array_equal(a + b, np.full_like(a, 2 << (bits - 1)))


def test_sym_zero_group_and_second_writing():
    w = synth.weight(2, "pins/sym/np", 4, 384, 0.02, outlier_p=0.01)
    w[1, 128:256] = 0
    c, s, z = oracle.quantize_sym(w, 8)
    assert s[1, 1] == np.float32(1.0) and np.all(c[1, 128:256] == 128)
    wf = w.astype(np.float32).reshape(4, 3, G)
    amax = np.abs(wf).max(axis=2)
    sn = np.where(amax == 0, np.float32(1.0), ((amax + amax) / np.float32(254.0)).astype(np.float32))
    qn = np.clip(np.rint((wf / sn[..., None]).astype(np.float32)), -127, 127).astype(np.int32) + 128
    assert np.array_equal(s, sn) and np.array_equal(c.astype(np.int32), qn.reshape(4, 384))
    # Eq. (3) on the stored form gives s * q: the asymmetric routines apply unchanged
    d = oracle.dequant(c, s, z, 8)
    assert np.array_equal(d, ((qn - 128).astype(np.float32) * sn[..., None]).reshape(4, 384))


def test_sym_rejects_non_finite():
    w = np.ones((1, G), dtype=np.float16)
    w[0, 5] = np.nan
    with pytest.raises(ValueError):
        oracle.quantize_sym(w, 4)
    with pytest.raises(ValueError):
        oracle.fake_quantize(w, 3)


# ---------------------------------------------------------------- quantize-dequantize

@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("sym", [False, True])
def test_fake_equals_dequant_of_quantize(bits, sym):
    w = synth.weight(3, "pins/fake/%d%d" % (bits, sym), 16, 512, 0.02, outlier_p=0.01)
    c, s, z = (oracle.quantize_sym if sym else oracle.quantize)(w, bits)
    ref = oracle.dequant(c, s, z, bits).astype(np.float16)       # binary32 -> binary16, to nearest even
    got = oracle.fake_quantize(w, bits, sym=sym)
    assert np.array_equal(got.view(np.uint16), ref.view(np.uint16))


@pytest.mark.parametrize("bits", [2, 3, 5])
def test_fake_low_bits_second_writing_and_level_count(bits):
    w = synth.weight(4, "pins/fake/low%d" % bits, 8, 384, 0.02, outlier_p=0.01)
    got = oracle.fake_quantize(w, bits).astype(np.float32).reshape(8, 3, G)
    wf = w.astype(np.float32).reshape(8, 3, G)
    lo = np.minimum(wf.min(axis=2), 0).astype(np.float32)
    hi = np.maximum(wf.max(axis=2), 0).astype(np.float32)
    qmax = np.float32((1 << bits) - 1)
    s = ((hi - lo).astype(np.float32) / qmax).astype(np.float32)
    zf = np.clip(np.rint(((-lo).astype(np.float32) / s).astype(np.float32)), 0, qmax)
    q = np.clip(np.rint(((wf / s[..., None]).astype(np.float32) + zf[..., None]).astype(np.float32)), 0, qmax)
    q = q.astype(np.int32).astype(np.float32)        # the stored code is an integer: -0 becomes 0
    ref = (((q - zf[..., None]).astype(np.float32) * s[..., None]).astype(np.float32)).astype(np.float16)
    assert np.array_equal(got.astype(np.float16).view(np.uint16), ref.view(np.uint16))
    for n in range(8):
        for g in range(3):
            assert len(np.unique(got[n, g])) <= (1 << bits)
    # nearest level: error at most half a step (plus the final binary16 rounding)
    err = np.abs(got.astype(np.float64) - wf.astype(np.float64))
    assert np.all(err <= 0.5 * s[..., None] * (1 + 2.0 ** -10) + 2.0 ** -11 * np.abs(got))


def test_fake_two_bit_symmetric_is_ternary():
    # 2^2 - 2 = 2 steps: the levels are -max|w|, 0, +max|w|
    w = synth.weight(5, "pins/fake/tern", 4, 256, 0.02)
    got = oracle.fake_quantize(w, 2, sym=True).astype(np.float64).reshape(4, 2, G)
    amax = np.abs(w.astype(np.float64)).reshape(4, 2, G).max(axis=2)
    for n in range(4):
        for g in range(2):
            assert set(np.unique(got[n, g])) <= {-amax[n, g], 0.0, amax[n, g]}
            big = np.abs(w.astype(np.float64).reshape(4, 2, G)[n, g]) > 0.5 * amax[n, g] * (1 + 1e-3)
            assert np.all(np.abs(got[n, g][big]) == amax[n, g])


def test_fake_on_grid_is_identity_and_brute_force():
    # weights already on a 3-bit grid with a power-of-two step (group range 0 .. 7 * 2^-5)
    rng = np.random.default_rng(6)
    q = rng.integers(0, 8, size=(2, G))
    q[:, 0], q[:, 1] = 0, 7
    w = (q * 2.0 ** -5).astype(np.float16)
    assert np.array_equal(oracle.fake_quantize(w, 3), w)
    # brute force on a tiny case, plain Python floats rounded through numpy scalars
    w = synth.weight(7, "pins/fake/bf", 1, G, 0.02)
    got = oracle.fake_quantize(w, 3)
    vals = [np.float32(v) for v in w[0]]
    lo, hi = min(vals + [np.float32(0)]), max(vals + [np.float32(0)])
    s = np.float32(np.float32(hi - lo) / np.float32(7))
    z = min(max(np.rint(np.float32(np.float32(-lo) / s)), 0), 7)
    for i, v in enumerate(vals):
        qq = min(max(np.rint(np.float32(np.float32(v / s) + np.float32(z))), 0), 7)
        assert got[0, i] == np.float16(np.float32(np.float32(qq - z) * s)), i

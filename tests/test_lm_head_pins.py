"""Pins for the oracle's output layer + entropy + argmax routine (Alg. 1: every decode step takes
the next token and PPLE, Sec. 4.2 Eq. 5, from the same logits)."""
import numpy as np
import scipy.special

import oracle
import synth


def test_identity_weight_reduces_to_the_pinned_entropy():
    # W = I: logits = x, so H is the entropy routine pinned on its own, argmax is argmax x
    V = 512
    x = synth.activations(0, "pins/lm/x", 3, V)
    logits, H, am = oracle.lm_head_entropy(x, np.eye(V, dtype=np.float16))
    assert np.array_equal(logits, x.astype(np.float64))
    H_ref, _ = oracle.entropy_kl(x.astype(np.float32))
    assert np.allclose(H, H_ref, rtol=1e-12, atol=1e-12)
    assert np.array_equal(am, np.argmax(x.astype(np.float64), axis=1))


def test_equal_rows_give_ln_v_and_the_first_index():
    V, K = 1000, 256
    w = np.tile(synth.weight(1, "pins/lm/row", 1, K, 0.02), (V, 1))
    x = synth.activations(1, "pins/lm/x2", 2, K)
    _, H, am = oracle.lm_head_entropy(x, w)
    assert np.allclose(H, np.log(V), rtol=1e-12) and am.tolist() == [0, 0]


def test_one_dominant_row():
    V, K = 300, 128
    w = np.zeros((V, K), dtype=np.float16)
    x = np.ones((1, K), dtype=np.float16)
    w[137] = 1.0                     # logit 128 against 0 everywhere else
    _, H, am = oracle.lm_head_entropy(x, w)
    assert am[0] == 137 and 0 <= H[0] < 1e-50
    w[41] = 1.0                      # two equal maxima: p = 1/2 each, the smaller index wins
    _, H, am = oracle.lm_head_entropy(x, w)
    assert am[0] == 41 and abs(H[0] - np.log(2)) < 1e-12


def test_second_writing_numpy_scipy():
    V, K, M = 2000, 384, 4
    w = synth.weight(2, "pins/lm/w", V, K, 0.05)
    x = synth.activations(2, "pins/lm/x3", M, K)
    logits, H, am = oracle.lm_head_entropy(x, w)
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    assert np.allclose(logits, ref, rtol=1e-12, atol=1e-12)
    lp = ref - scipy.special.logsumexp(ref, axis=1, keepdims=True)
    assert np.allclose(H, -(np.exp(lp) * lp).sum(axis=1), rtol=1e-10)
    assert np.array_equal(am, ref.argmax(axis=1))
    assert np.all(H > 0) and np.all(H <= np.log(V))


def test_transposed_operand_or_wrong_row_shows():
    # logits[m][v] must pair token m with vocabulary row v: distinct values everywhere
    x = np.array([[1, 0, 0, 0], [0, 2, 0, 0]], dtype=np.float16)
    w = np.array([[1, 10, 0, 0], [2, 20, 0, 0], [3, 30, 0, 0]], dtype=np.float16)
    logits, _, am = oracle.lm_head_entropy(x, w)
    assert logits.tolist() == [[1, 2, 3], [20, 40, 60]] and am.tolist() == [2, 2]


def test_brute_force_python():
    V, K = 7, 8
    w = synth.weight(3, "pins/lm/bf", V, K, 0.5)
    x = synth.activations(3, "pins/lm/xbf", 1, K)
    _, H, am = oracle.lm_head_entropy(x, w)
    lg = [sum(float(x[0, k]) * float(w[v, k]) for k in range(K)) for v in range(V)]
    mx = max(lg)
    S = sum(np.exp(l - mx) for l in lg)
    h = -sum((np.exp(l - mx) / S) * (l - mx - np.log(S)) for l in lg)
    assert abs(H[0] - h) < 1e-12 and am[0] == lg.index(mx)

"""GPU parity of the fused output layer + entropy + argmax with the CPU oracle.

Entropy within 1e-4 relative (+1e-7); logits within the rounding of a binary32 sum of K products;
argmax: the kernel decides in binary32, the oracle in double, so the index must agree wherever
the oracle's two largest logits are further apart than that rounding, and must in any case point
at a logit within it of the maximum."""
import numpy as np
import pytest
import torch

import oracle
import synth
import paper_2506_12024_amd as fq
from gpu_util import DEV, to_dev

pytestmark = pytest.mark.gpu


def _run(x, w, want_logits=True):
    M, K = x.shape
    V = w.shape[0]
    H = torch.full((M,), float("nan"), device=DEV)
    am = torch.full((M,), -1, dtype=torch.int32, device=DEV)
    lg = torch.full((M, V), float("nan"), device=DEV) if want_logits else None
    fq.fq_lm_head_entropy(to_dev(x), to_dev(w), M, V, K, lg, H, am)
    torch.cuda.synchronize()
    return (lg.cpu().numpy() if want_logits else None), H.cpu().numpy(), am.cpu().numpy()


def _check(x, w, want_logits=True):
    lg_ref, H_ref, am_ref = oracle.lm_head_entropy(x, w)
    lg, H, am = _run(x, w, want_logits)
    K = x.shape[1]
    mag = (np.abs(x.astype(np.float64)) @ np.abs(w.astype(np.float64)).T)     # sum |x w| per logit
    tol = mag * (K * 2.0 ** -24) + 1e-30
    if want_logits:
        assert np.all(np.abs(lg - lg_ref) <= tol)
    assert np.all(np.abs(H - H_ref) <= 1e-4 * np.abs(H_ref) + 1e-7), (H, H_ref)
    for m in range(x.shape[0]):
        top2 = np.partition(lg_ref[m], -2)[-2:]
        gap = top2[1] - top2[0]
        t = tol[m].max()
        assert lg_ref[m, am[m]] >= top2[1] - 2 * t
        if gap > 2 * t:
            assert am[m] == am_ref[m]


@pytest.mark.parametrize("M", [1, 2, 3, 4])
@pytest.mark.parametrize("V,K", [(32000, 4096), (1000, 512), (7, 1024), (128256, 512), (4099, 5120)])
def test_lm_head_entropy_matches_oracle(M, V, K):
    w = synth.weight(0, "par/lm/w%d_%d" % (V, K), V, K, 0.02, outlier_p=0.001)
    x = synth.activations(0, "par/lm/x%d_%d" % (M, K), M, K)
    _check(x, w, want_logits=(V <= 32000))


def test_lm_head_entropy_special_cases():
    V, K = 3000, 512
    # equal rows: H = ln V, argmax = 0
    w = np.tile(synth.weight(1, "par/lm/row", 1, K, 0.02), (V, 1))
    x = synth.activations(1, "par/lm/xs", 2, K)
    _, H, am = _run(x, w)
    assert np.all(np.abs(H - np.log(V)) <= 1e-4 * np.log(V)) and am.tolist() == [0, 0]
    # one dominant row, then two equal maxima (exact in any precision): the smaller index wins
    w = np.zeros((V, K), dtype=np.float16)
    x = np.ones((1, K), dtype=np.float16)
    w[2137] = 1.0
    _, H, am = _run(x, w)
    assert am[0] == 2137 and abs(H[0]) <= 1e-7
    w[41] = 1.0
    _, H, am = _run(x, w)
    assert am[0] == 41 and abs(H[0] - np.log(2)) <= 1e-4 * np.log(2)


def test_lm_head_entropy_repeated_calls_and_optional_outputs():
    # the arrival ticket is reset by every launch; argmax and logits are optional
    V, K, M = 5000, 1024, 2
    w = synth.weight(2, "par/lm/w2", V, K, 0.05)
    x = synth.activations(2, "par/lm/x2", M, K)
    _, H_ref, _ = oracle.lm_head_entropy(x, w)
    xd, wd = to_dev(x), to_dev(w)
    for _ in range(3):
        H = torch.full((M,), float("nan"), device=DEV)
        fq.fq_lm_head_entropy(xd, wd, M, V, K, None, H, None)
        torch.cuda.synchronize()
        assert np.all(np.abs(H.cpu().numpy() - H_ref) <= 1e-4 * np.abs(H_ref) + 1e-7)

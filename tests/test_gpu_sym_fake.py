"""GPU parity of the symmetric quantizer and of quantize-dequantize with the CPU oracle: codes,
scales, zero points and fp16 results bit for bit; the symmetric copy runs through the same
linears as the asymmetric one."""
import numpy as np
import pytest
import torch

import oracle
import synth
import paper_2506_12024_amd as fq
from gpu_util import DEV, gpu_linear, rel_err, to_dev

pytestmark = pytest.mark.gpu


def _gpu_quantize_sym(w_dev, bits):
    N, K = w_dev.shape
    cb, sb, zb = fq.fq_packed_sizes(N, K, bits, 128)
    codes = torch.empty(cb, dtype=torch.uint8, device=DEV)
    scales = torch.empty(sb // 4, dtype=torch.float32, device=DEV)
    zeros = torch.empty(zb, dtype=torch.uint8, device=DEV)
    fq.fq_quantize_sym(w_dev, N, K, bits, 128, codes, scales, zeros)
    return codes.view(N, -1), scales.view(N, -1), zeros.view(N, -1)


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("shape,outl", [((4096, 4096), 0.001), ((48, 1408), 0.01), ((1, 128), 0.0)])
def test_quantize_sym_bit_exact(bits, shape, outl):
    N, K = shape
    w = synth.weight(0, "par/sym/w", N, K, 0.02, outlier_p=outl)
    w[0, :128] = 0                                    # an all-zero group
    c_ref, s_ref, z_ref = oracle.quantize_sym(w, bits)
    c, s, z = _gpu_quantize_sym(to_dev(w), bits)
    torch.cuda.synchronize()
    assert np.array_equal(c.cpu().numpy(), c_ref)
    assert np.array_equal(s.cpu().numpy().view(np.uint32), s_ref.view(np.uint32))
    assert np.array_equal(z.cpu().numpy(), z_ref)


@pytest.mark.parametrize("bits", [2, 3, 4, 5, 8])
@pytest.mark.parametrize("sym", [False, True])
def test_fake_quantize_bit_exact(bits, sym):
    for (N, K, outl) in [(512, 4096, 0.001), (37, 384, 0.02)]:
        w = synth.weight(1, "par/fake/w", N, K, 0.02, outlier_p=outl)
        w[0, :128] = 0
        ref = oracle.fake_quantize(w, bits, sym=sym)
        w_dev = to_dev(w)
        out = torch.full((N, K), float("nan"), dtype=torch.float16, device=DEV)
        fq.fq_fake_quantize(w_dev, N, K, bits, 128, sym, out)
        torch.cuda.synchronize()
        assert np.array_equal(out.cpu().numpy().view(np.uint16), ref.view(np.uint16)), (bits, sym, N, K)
        # in place
        fq.fq_fake_quantize(w_dev, N, K, bits, 128, sym, w_dev)
        torch.cuda.synchronize()
        assert np.array_equal(w_dev.cpu().numpy().view(np.uint16), ref.view(np.uint16))


@pytest.mark.parametrize("bits", [4, 8])
@pytest.mark.parametrize("M", [1, 8, 40])
def test_symmetric_copy_runs_through_the_same_linears(bits, M):
    N, K = 300, 1408
    w = synth.weight(2, "par/sym/lin", N, K, 0.02, outlier_p=0.001)
    x = synth.activations(2, "par/sym/x%d" % M, M, K)
    c, s, z = _gpu_quantize_sym(to_dev(w), bits)
    layer = fq.Layer(N, K)
    layer.attach(bits, c, s, z)
    y = gpu_linear(layer, bits, x)
    y_ref = oracle.linear(x, c.cpu().numpy(), s.cpu().numpy(), z.cpu().numpy(), bits)
    assert rel_err(y, y_ref) <= 2e-3


def test_two_bit_model_through_the_fp16_path():
    # what Sec. 5.1 does for the widths without a packed kernel: simulate, then run as fp16
    N, K, M = 256, 1024, 4
    w = synth.weight(3, "par/fake/lin", N, K, 0.02)
    x = synth.activations(3, "par/fake/x", M, K)
    w_dev = to_dev(w)
    w_hat = torch.empty_like(w_dev)
    fq.fq_fake_quantize(w_dev, N, K, 2, 128, False, w_hat)
    layer = fq.Layer(N, K)
    layer.attach(16, w_hat)
    y = gpu_linear(layer, 16, x)
    y_ref = oracle.linear(x, oracle.fake_quantize(w, 2), None, None, 16)
    assert rel_err(y, y_ref) <= 2e-3


def test_fake_quantize_in_place():
    # w_hat may be w itself
    w = synth.weight(0, "sym/inplace/w", 64, 1024, 0.02, outlier_p=0.001)
    ref = oracle.fake_quantize(w, 3)
    w_dev = to_dev(w)
    fq.fq_fake_quantize(w_dev, 64, 1024, 3, 128, False, w_dev)
    torch.cuda.synchronize()
    assert np.array_equal(w_dev.cpu().numpy().view(np.uint16), ref.view(np.uint16))

"""Helpers for the GPU parity tests: move seeded host tensors to the device, run the
library through its C ABI binding, bring results back as numpy arrays."""
import numpy as np
import torch

import paper_2506_12024_amd as fq

DEV = "cuda:0"


def to_dev(a: np.ndarray) -> torch.Tensor:
    if a.dtype == np.float16:
        return torch.from_numpy(a.view(np.int16)).to(DEV).view(torch.float16)
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def gpu_quantize(w_dev: torch.Tensor, bits: int, group: int = 128):
    N, K = w_dev.shape
    cb, sb, zb = fq.fq_packed_sizes(N, K, bits, group)
    codes = torch.empty(cb, dtype=torch.uint8, device=DEV)
    scales = torch.empty(sb // 4, dtype=torch.float32, device=DEV)
    zeros = torch.empty(zb, dtype=torch.uint8, device=DEV)
    fq.fq_quantize(w_dev, N, K, bits, group, codes, scales, zeros)
    return codes.view(N, -1), scales.view(N, -1), zeros.view(N, -1)


def make_layer(w: np.ndarray, bits_list=(4, 8), group: int = 128):
    """Quantize w (fp16 [N][K]) on the GPU at each bit-width and attach the copies."""
    N, K = w.shape
    w_dev = to_dev(w)
    layer = fq.Layer(N, K, group)
    packed = {}
    for b in bits_list:
        if b == 16:
            layer.attach(16, w_dev)
            packed[16] = (w_dev,)
        else:
            c, s, z = gpu_quantize(w_dev, b, group)
            layer.attach(b, c, s, z)
            packed[b] = (c, s, z)
    return layer, packed


def gpu_linear(layer, bits: int, x: np.ndarray) -> np.ndarray:
    M, K = x.shape
    x_dev = to_dev(x)
    y = torch.full((M, layer.N), float("nan"), dtype=torch.float16, device=DEV)
    fq.fq_linear(layer, bits, x_dev, M, y)
    torch.cuda.synchronize()
    return y.cpu().numpy()


def rel_err(y_gpu: np.ndarray, y_ref: np.ndarray) -> float:
    """max |y_gpu - y_ref| / max |y_ref| (max-abs normalised)."""
    a = y_gpu.astype(np.float64)
    b = y_ref.astype(np.float64)
    return float(np.abs(a - b).max() / np.abs(b).max())

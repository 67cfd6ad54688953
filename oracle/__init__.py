"""ctypes front end of the CPU oracle (``flexq_oracle.c``).

TEST INFRASTRUCTURE ONLY.  The tests, the smoke check and the benchmark's
``cpu_baseline`` leg call it; the product package never does.  It shares no
code with the GPU library: the C file is compiled with gcc on its own.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "flexq_oracle.c")
_LIB = os.path.join(_HERE, "libflexq_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """gcc -O2, no contraction, no fast-math: every float operation of the
    quantizer is rounded once, as the oracle's header states."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-shared", "-fPIC",
             "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        vp, ci = ctypes.c_void_p, ctypes.c_int
        lib.orc_half_to_float.restype = ctypes.c_float
        lib.orc_half_to_float.argtypes = [ctypes.c_uint16]
        lib.orc_double_to_half.restype = ctypes.c_uint16
        lib.orc_double_to_half.argtypes = [ctypes.c_double]
        lib.orc_quantize.restype = ci
        lib.orc_quantize.argtypes = [vp, ci, ci, ci, ci, vp, vp, vp]
        lib.orc_quantize_sym.restype = ci
        lib.orc_quantize_sym.argtypes = [vp, ci, ci, ci, ci, vp, vp, vp]
        lib.orc_fake_quantize.restype = ci
        lib.orc_fake_quantize.argtypes = [vp, ci, ci, ci, ci, ci, vp]
        lib.orc_lm_head_entropy.restype = ci
        lib.orc_lm_head_entropy.argtypes = [vp, vp, ci, ci, ci, vp, vp, vp]
        lib.orc_dequant.restype = None
        lib.orc_dequant.argtypes = [vp, vp, vp, ci, ci, ci, ci, vp]
        lib.orc_linear.restype = ci
        lib.orc_linear.argtypes = [vp, ci, vp, vp, vp, ci, ci, ci, ci, ci, ci, vp]
        lib.orc_entropy_kl.restype = ci
        lib.orc_entropy_kl.argtypes = [vp, vp, ci, ci, vp, vp]
        lib.orc_rank_ascending.restype = ci
        lib.orc_rank_ascending.argtypes = [vp, ci, ci, vp]
        lib.orc_quantize_act.restype = ci
        lib.orc_quantize_act.argtypes = [vp, ci, ci, vp, vp]
        lib.orc_linear_w8a8.restype = ci
        lib.orc_linear_w8a8.argtypes = [vp, vp, ci, vp, vp, vp, ci, ci, ci, ci, ci, vp]
        _lib = lib
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def half_to_float(bits: int) -> float:
    return float(_load().orc_half_to_float(bits))


def double_to_half(d: float) -> int:
    return int(_load().orc_double_to_half(d))


def quantize(w: np.ndarray, bits: int, group: int = 128):
    """w: fp16 [N][K].  Returns (codes u8 [N][K*bits/8], scales f32 [N][K/group],
    zeros u8 [N][K/group]) in the canonical packed layout (Sec. 2.2 Eq. 2)."""
    w = np.ascontiguousarray(w, dtype=np.float16)
    N, K = w.shape
    if bits not in (2, 3, 4, 8) or group <= 0 or K % group:
        raise ValueError("bad bits/group")
    codes = np.zeros((N, K * bits // 8), dtype=np.uint8)
    scales = np.zeros((N, K // group), dtype=np.float32)
    zeros = np.zeros((N, K // group), dtype=np.uint8)
    rc = _load().orc_quantize(_p(w), N, K, bits, group, _p(codes), _p(scales), _p(zeros))
    if rc != 0:
        raise ValueError("orc_quantize rejected its input (non-finite weight or bad shape)")
    return codes, scales, zeros


def quantize_sym(w: np.ndarray, bits: int, group: int = 128):
    """Symmetric variant stated after Sec. 2.2 Eq. 3 (z = 0, Xmax = -Xmin = max |X|, 2^n - 2
    levels), written in the layout of quantize(): stored code = q + 2^(n-1), stored zero point
    = 2^(n-1), so that dequant() and linear() apply unchanged."""
    w = np.ascontiguousarray(w, dtype=np.float16)
    N, K = w.shape
    if bits not in (2, 3, 4, 8) or group <= 0 or K % group:
        raise ValueError("bad bits/group")
    codes = np.zeros((N, K * bits // 8), dtype=np.uint8)
    scales = np.zeros((N, K // group), dtype=np.float32)
    zeros = np.zeros((N, K // group), dtype=np.uint8)
    rc = _load().orc_quantize_sym(_p(w), N, K, bits, group, _p(codes), _p(scales), _p(zeros))
    if rc != 0:
        raise ValueError("orc_quantize_sym rejected its input (non-finite weight or bad shape)")
    return codes, scales, zeros


def fake_quantize(w: np.ndarray, bits: int, group: int = 128, sym: bool = False) -> np.ndarray:
    """Quantize and dequantize (Sec. 2.2 Eq. 2 then Eq. 3) at 2 .. 8 bits, rounded to fp16: how the
    paper simulated its 2- to 4-bit models (Sec. 5.1, Table 1).  fp16 [N][K]."""
    w = np.ascontiguousarray(w, dtype=np.float16)
    N, K = w.shape
    if not 2 <= bits <= 8 or group <= 0 or K % group:
        raise ValueError("bad bits/group")
    out = np.zeros((N, K), dtype=np.float16)
    rc = _load().orc_fake_quantize(_p(w), N, K, bits, group, 1 if sym else 0, _p(out))
    if rc != 0:
        raise ValueError("orc_fake_quantize rejected its input (non-finite weight or bad shape)")
    return out


def dequant(codes, scales, zeros, bits: int, group: int = 128) -> np.ndarray:
    """Sec. 2.2 Eq. 3: float32 [N][K]."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scales = np.ascontiguousarray(scales, dtype=np.float32)
    zeros = np.ascontiguousarray(zeros, dtype=np.uint8)
    N = codes.shape[0]
    K = codes.shape[1] * 8 // bits
    out = np.empty((N, K), dtype=np.float32)
    _load().orc_dequant(_p(codes), _p(scales), _p(zeros), N, K, bits, group, _p(out))
    return out


def linear(x: np.ndarray, codes, scales, zeros, bits: int, group: int = 128,
           row0: int = 0, rows: int | None = None) -> np.ndarray:
    """y[m][n] for n in [row0, row0+rows): fp16 [M][rows].  bits=16: ``codes`` is
    the fp16 weight matrix itself."""
    x = np.ascontiguousarray(x, dtype=np.float16)
    M, K = x.shape
    if bits == 16:
        wt = np.ascontiguousarray(codes, dtype=np.float16)
        N = wt.shape[0]
        assert wt.shape[1] == K
        cp, sp, zp = _p(wt), None, None
    else:
        codes = np.ascontiguousarray(codes, dtype=np.uint8)
        scales = np.ascontiguousarray(scales, dtype=np.float32)
        zeros = np.ascontiguousarray(zeros, dtype=np.uint8)
        N = codes.shape[0]
        assert codes.shape[1] * 8 // bits == K
        cp, sp, zp = _p(codes), _p(scales), _p(zeros)
    rows = N - row0 if rows is None else rows
    y = np.empty((M, rows), dtype=np.float16)
    rc = _load().orc_linear(_p(x), M, cp, sp, zp, N, K, bits, group, row0, rows, _p(y))
    if rc != 0:
        raise ValueError("orc_linear rejected its arguments")
    return y


def entropy_kl(a: np.ndarray, b: np.ndarray | None = None):
    """Per-row entropy of softmax(a) (nats, float64 [R]) and, when ``b`` is given,
    KL(softmax(a) || softmax(b)).  PPLE of Sec. 4.2 Eq. 5 is exp(entropy)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    if a.ndim == 1:
        a = a[None, :]
    R, V = a.shape
    if b is not None:
        b = np.ascontiguousarray(b, dtype=np.float32).reshape(R, V)
    H = np.empty(R, dtype=np.float64)
    KL = np.empty(R, dtype=np.float64) if b is not None else None
    rc = _load().orc_entropy_kl(_p(a), _p(b), R, V, _p(H), _p(KL))
    if rc != 0:
        raise ValueError("orc_entropy_kl rejected its arguments")
    return (H, KL) if b is not None else (H, None)


def lm_head_entropy(x: np.ndarray, w: np.ndarray):
    """Output layer + what Alg. 1 takes from its logits: x fp16 [M][K], w fp16 [V][K] ->
    (logits f64 [M][V], H f64 [M], argmax int32 [M]); entropy as in Sec. 4.2 Eq. 5."""
    x = np.ascontiguousarray(x, dtype=np.float16)
    w = np.ascontiguousarray(w, dtype=np.float16)
    M, K = x.shape
    V, K2 = w.shape
    if K != K2:
        raise ValueError("x and w disagree on K")
    logits = np.zeros((M, V), dtype=np.float64)
    H = np.zeros(M, dtype=np.float64)
    am = np.zeros(M, dtype=np.int32)
    if _load().orc_lm_head_entropy(_p(x), _p(w), M, V, K, _p(logits), _p(H), _p(am)) != 0:
        raise ValueError("orc_lm_head_entropy rejected its input")
    return logits, H, am


def rank_ascending(values: np.ndarray) -> np.ndarray:
    """Replacement order of Sec. 4.3: entries sorted by ascending KL.  values: float32 [n] or
    [n][m] (m calibration rows per entry, ranked by their sum); returns int32 [n]."""
    v = np.ascontiguousarray(values, dtype=np.float32)
    if v.ndim == 1:
        v = v[:, None]
    n, m = v.shape
    order = np.zeros(n, dtype=np.int32)
    if _load().orc_rank_ascending(_p(v), n, m, _p(order)) != 0:
        raise ValueError("orc_rank_ascending rejected its arguments")
    return order


def quantize_act(x: np.ndarray):
    """Per-token symmetric 8-bit activation quantization (W8A8 prefill, Sec. 4.3; the
    symmetric form stated after Eq. 3).  x: fp16 [M][K]; returns (xq int8 [M][K], sx f32 [M])."""
    x = np.ascontiguousarray(x, dtype=np.float16)
    M, K = x.shape
    xq = np.zeros((M, K), dtype=np.int8)
    sx = np.zeros(M, dtype=np.float32)
    if _load().orc_quantize_act(_p(x), M, K, _p(xq), _p(sx)) != 0:
        raise ValueError("orc_quantize_act rejected its input (non-finite activation or bad shape)")
    return xq, sx


def linear_w8a8(xq: np.ndarray, sx: np.ndarray, codes, scales, zeros, group: int = 128,
                row0: int = 0, rows: int | None = None) -> np.ndarray:
    """y = dequant(xq, sx) . dequant(W8)^T, fp16 [M][rows]."""
    xq = np.ascontiguousarray(xq, dtype=np.int8)
    sx = np.ascontiguousarray(sx, dtype=np.float32)
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scales = np.ascontiguousarray(scales, dtype=np.float32)
    zeros = np.ascontiguousarray(zeros, dtype=np.uint8)
    M, K = xq.shape
    N = codes.shape[0]
    assert codes.shape[1] == K and sx.shape == (M,)
    rows = N - row0 if rows is None else rows
    y = np.empty((M, rows), dtype=np.float16)
    rc = _load().orc_linear_w8a8(_p(xq), _p(sx), M, _p(codes), _p(scales), _p(zeros), N, K, group,
                                 row0, rows, _p(y))
    if rc != 0:
        raise ValueError("orc_linear_w8a8 rejected its arguments")
    return y


class Scheduler:
    """Token-wise precision switching of Sec. 4.4 / Alg. 1 (oracle).  ``bits`` is an int32
    array updated in place; ``events`` is the replacement order as (entry, new_bits) pairs."""

    def __init__(self, bits: np.ndarray, events, window: int = 20, thre: float = 0.0,
                 per_trigger: int = 1):
        lib = _load()
        lib.orc_sched_size.restype = ctypes.c_int
        lib.orc_sched_init.restype = ctypes.c_int
        lib.orc_sched_init.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_double, ctypes.c_int,
                                       ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p,
                                       ctypes.c_void_p]
        lib.orc_sched_step.restype = ctypes.c_int
        lib.orc_sched_step.argtypes = [ctypes.c_void_p, ctypes.c_float]
        lib.orc_sched_threshold_from_prefill.restype = None
        lib.orc_sched_threshold_from_prefill.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int,
                                                         ctypes.c_int]
        lib.orc_sched_thre.restype = ctypes.c_double
        lib.orc_sched_thre.argtypes = [ctypes.c_void_p]
        lib.orc_sched_last_mean.restype = ctypes.c_double
        lib.orc_sched_last_mean.argtypes = [ctypes.c_void_p]
        lib.orc_sched_next_event.restype = ctypes.c_int
        lib.orc_sched_next_event.argtypes = [ctypes.c_void_p]
        self._lib = lib
        assert bits.dtype == np.int32 and bits.flags.c_contiguous
        self.bits = bits
        ev = np.asarray(events, dtype=np.int32).reshape(-1, 2)
        self._entry = np.ascontiguousarray(ev[:, 0])
        self._to = np.ascontiguousarray(ev[:, 1])
        self.ev_token = np.full(len(ev), -1, dtype=np.int32)
        self._state = ctypes.create_string_buffer(lib.orc_sched_size())
        rc = lib.orc_sched_init(self._state, window, thre, per_trigger, _p(self._entry), _p(self._to),
                                len(ev), _p(self.bits), _p(self.ev_token))
        if rc != 0:
            raise ValueError("orc_sched_init rejected its arguments")

    def threshold_from_prefill(self, entropy: np.ndarray, last_n: int):
        e = np.ascontiguousarray(entropy, dtype=np.float32)
        self._lib.orc_sched_threshold_from_prefill(self._state, _p(e), e.size, last_n)

    def step(self, entropy: float) -> int:
        return int(self._lib.orc_sched_step(self._state, float(np.float32(entropy))))

    @property
    def thre(self) -> float:
        return float(self._lib.orc_sched_thre(self._state))

    @property
    def last_mean(self) -> float:
        return float(self._lib.orc_sched_last_mean(self._state))

    @property
    def next_event(self) -> int:
        return int(self._lib.orc_sched_next_event(self._state))

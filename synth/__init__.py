"""Seeded synthetic inputs for the tests and the benchmark.

The tensors stand in for the trained weights, activations and logits of the
paper's workloads (Sec. 5.1 uses real checkpoints and datasets, which are not
available): Llama-shaped linears with weights ~ N(0, std), optionally with a
fraction of entries scaled up as outliers, fp16 activations ~ N(0, 1), fp32
logits ~ N(0, 3) plus a small perturbation, and per-layer bit-width patterns.

Nothing here belongs to the method: the module only maps (seed, name, element
index) to reproducible numbers through ``gen.c`` (splitmix64 counters and
Box-Muller in double).  Both the CPU oracle's callers and the GPU library's
callers take their inputs from here, so the two sides see identical bytes.
Any slice of a tensor can be regenerated alone via ``first``/``count``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gen.c")
_LIB = os.path.join(_HERE, "libfqsynth.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile gen.c with gcc (needs no GPU).  Returns the library path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        u64, dbl, vp = ctypes.c_uint64, ctypes.c_double, ctypes.c_void_p
        lib.fqs_hash64.restype = u64
        lib.fqs_hash64.argtypes = [u64]
        lib.fqs_f32_to_f16.restype = ctypes.c_uint16
        lib.fqs_f32_to_f16.argtypes = [ctypes.c_float]
        lib.fqs_normal_f16.restype = None
        lib.fqs_normal_f16.argtypes = [u64, u64, u64, u64, dbl, dbl, dbl, dbl, vp]
        lib.fqs_normal_f32.restype = None
        lib.fqs_normal_f32.argtypes = [u64, u64, u64, dbl, dbl, vp, vp]
        lib.fqs_choice_i32.restype = None
        lib.fqs_choice_i32.argtypes = [u64, u64, u64, vp, ctypes.c_int32, vp]
        _lib = lib
    return _lib


def stream_key(seed: int, name: str) -> int:
    """64-bit stream key from an integer seed and a tensor name (FNV-1a over the
    name, mixed with the seed through the generator's own hash)."""
    h = 0xCBF29CE484222325
    for ch in name.encode():
        h = ((h ^ ch) * 0x100000001B3) & 0xFFFFFFFFFFFFFFFF
    lib = _load()
    return int(lib.fqs_hash64((h ^ lib.fqs_hash64(seed & 0xFFFFFFFFFFFFFFFF)) & 0xFFFFFFFFFFFFFFFF))


def normal_f16(seed: int, name: str, count: int, std: float, *, mean: float = 0.0,
               outlier_p: float = 0.0, outlier_mul: float = 20.0, first: int = 0) -> np.ndarray:
    """fp16 vector of N(mean, std) values; each entry is multiplied by
    ``outlier_mul`` with probability ``outlier_p``."""
    out = np.empty(count, dtype=np.float16)
    _load().fqs_normal_f16(stream_key(seed, name), stream_key(seed, name + "/outlier"),
                           first, count, mean, std, outlier_p, outlier_mul,
                           out.ctypes.data_as(ctypes.c_void_p))
    return out


def normal_f32(seed: int, name: str, count: int, std: float, *, mean: float = 0.0,
               base: np.ndarray | None = None, first: int = 0) -> np.ndarray:
    """fp32 vector of N(mean, std) values, added to ``base`` when given."""
    out = np.empty(count, dtype=np.float32)
    bp = None
    if base is not None:
        base = np.ascontiguousarray(base, dtype=np.float32)
        assert base.size == count
        bp = base.ctypes.data_as(ctypes.c_void_p)
    _load().fqs_normal_f32(stream_key(seed, name), first, count, mean, std, bp,
                           out.ctypes.data_as(ctypes.c_void_p))
    return out


def choice(seed: int, name: str, count: int, choices, *, first: int = 0) -> np.ndarray:
    """int32 vector drawn uniformly from ``choices`` (e.g. bit-widths (4, 8))."""
    ch = np.ascontiguousarray(choices, dtype=np.int32)
    out = np.empty(count, dtype=np.int32)
    _load().fqs_choice_i32(stream_key(seed, name), first, count,
                           ch.ctypes.data_as(ctypes.c_void_p), ch.size,
                           out.ctypes.data_as(ctypes.c_void_p))
    return out


# ---------------------------------------------------------------------------
# Workload recipes (shapes only; no arithmetic of the method).
# ---------------------------------------------------------------------------

def llama_linears(hidden: int, ffn: int, kv: int | None = None):
    """(name, K, N) of the seven linears of one Llama-style decoder layer; `kv`: width of the key
    and value projections where it is smaller than the hidden size (grouped-query attention)."""
    kv = hidden if kv is None else kv
    return [("q", hidden, hidden), ("k", hidden, kv), ("v", hidden, kv),
            ("o", hidden, hidden), ("gate", hidden, ffn), ("up", hidden, ffn),
            ("down", ffn, hidden)]


STACKS = {
    # name: (layers, hidden, ffn, weight std, outlier probability)
    "llama7b": (32, 4096, 11008, 0.02, 0.0),
    "llama13b": (40, 5120, 13824, 0.02, 0.001),
    "llama70b": (80, 8192, 28672, 0.015, 0.0),
}
KV_WIDTH = {"llama70b": 1024}  # grouped-query attention: 8 key/value heads of 128


def weight(seed: int, name: str, N: int, K: int, std: float, outlier_p: float = 0.0,
           row0: int = 0, rows: int | None = None) -> np.ndarray:
    """fp16 weight matrix [N][K] (rows row0 .. row0+rows of it)."""
    rows = N - row0 if rows is None else rows
    return normal_f16(seed, name, rows * K, std, outlier_p=outlier_p, first=row0 * K).reshape(rows, K)


def activations(seed: int, name: str, M: int, K: int) -> np.ndarray:
    """fp16 activations [M][K] ~ N(0, 1)."""
    return normal_f16(seed, name, M * K, 1.0).reshape(M, K)


def logits_pair(seed: int, name: str, R: int, V: int, std: float = 3.0, noise: float = 0.1):
    """fp32 logits [R][V] ~ N(0, std) and a second tensor = first + N(0, noise)."""
    a = normal_f32(seed, name + "/a", R * V, std)
    b = normal_f32(seed, name + "/noise", R * V, noise, base=a)
    return a.reshape(R, V), b.reshape(R, V)

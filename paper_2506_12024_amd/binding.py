"""ctypes binding of the C ABI in ``include/flexq.h`` -- argument marshalling only.

Function names and argument order follow the header.  Tensor arguments are
``torch`` CUDA(HIP) tensors (or raw integer device pointers); the stream is
torch's current stream unless given.  No arithmetic happens here.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libflexq.so")

FQ_GROUP = 128
FQ_MAX_DECODE_M = 32
FQ_MAX_LM_HEAD_M = 4
FQ_STATIC_MAX_ENTRIES = 512
FQ_SCRATCH_BANKS = 16
FQ_OK, FQ_ERR_NULL, FQ_ERR_BITS, FQ_ERR_SHAPE, FQ_ERR_NOT_ATTACHED, FQ_ERR_ALIGN, FQ_ERR_HIP = \
    0, -1, -2, -3, -4, -5, -6

EXPORTS = [
    "fq_last_error", "fq_packed_sizes", "fq_quantize", "fq_layer_create", "fq_layer_attach",
    "fq_layer_destroy", "fq_linear", "fq_plan_workspace_bytes", "fq_plan_create", "fq_plan_run",
    "fq_plan_destroy", "fq_entropy_kl", "fq_sched_state_bytes", "fq_sched_init",
    "fq_sched_threshold_from_prefill", "fq_sched_step", "fq_sched_peek",
    "fq_entropy_kl_f16", "fq_rank_ascending", "fq_quantize_act", "fq_linear_w8a8",
    "fq_quantize_sym", "fq_fake_quantize", "fq_lm_head_entropy", "fq_linears_static",
    "fq_plan_staged_workspace_bytes", "fq_plan_create_staged", "fq_plan_set_wait_limit", "fq_plan_status",
    "fq_stream_read",
]


class FlexqError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__("flexq error %d: %s" % (code, message))
        self.code = code


def lib_path() -> str:
    return _LIB_PATH


def _load() -> ctypes.CDLL:
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            "libflexq.so is not built: run `python -m paper_2506_12024_amd.build` "
            "(there is no fallback path)")
    try:
        # PyTorch-ROCm carries its own HIP runtime; loaded first, the library binds to that one
        # instead of bringing a second runtime (with no devices set up) into the process
        import torch  # noqa: F401
    except ImportError:
        pass
    L = ctypes.CDLL(_LIB_PATH)
    vp, ci, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
    L.fq_last_error.restype = ctypes.c_char_p
    L.fq_last_error.argtypes = []
    L.fq_packed_sizes.restype = ci
    L.fq_packed_sizes.argtypes = [ci, ci, ci, ci, ctypes.POINTER(sz), ctypes.POINTER(sz), ctypes.POINTER(sz)]
    L.fq_quantize.restype = ci
    L.fq_quantize.argtypes = [vp, ci, ci, ci, ci, vp, vp, vp, vp]
    L.fq_layer_create.restype = ci
    L.fq_layer_create.argtypes = [ctypes.POINTER(vp), ci, ci, ci]
    L.fq_layer_attach.restype = ci
    L.fq_layer_attach.argtypes = [vp, ci, vp, vp, vp]
    L.fq_layer_destroy.restype = ci
    L.fq_layer_destroy.argtypes = [vp]
    L.fq_linear.restype = ci
    L.fq_linear.argtypes = [vp, ci, vp, ci, vp, vp]
    L.fq_plan_workspace_bytes.restype = sz
    L.fq_plan_workspace_bytes.argtypes = [ci]
    L.fq_plan_create.restype = ci
    L.fq_plan_create.argtypes = [ctypes.POINTER(vp), ci, ctypes.POINTER(vp), ctypes.POINTER(vp),
                                 ctypes.POINTER(vp), ci, vp, sz, vp]
    L.fq_plan_run.restype = ci
    L.fq_plan_run.argtypes = [vp, vp, vp]
    L.fq_plan_destroy.restype = ci
    L.fq_plan_destroy.argtypes = [vp]
    L.fq_plan_staged_workspace_bytes.restype = sz
    L.fq_plan_staged_workspace_bytes.argtypes = [ci, ci]
    L.fq_plan_create_staged.restype = ci
    L.fq_plan_create_staged.argtypes = [ctypes.POINTER(vp), ci, ctypes.POINTER(vp), ctypes.POINTER(vp),
                                        ctypes.POINTER(vp), ctypes.POINTER(ctypes.c_int32), ci, vp, sz, vp]
    L.fq_plan_set_wait_limit.restype = ci
    L.fq_plan_set_wait_limit.argtypes = [vp, ctypes.c_longlong]
    L.fq_plan_status.restype = ci
    L.fq_plan_status.argtypes = [vp, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32), vp]
    L.fq_stream_read.restype = ci
    L.fq_stream_read.argtypes = [vp, sz, vp, vp]
    L.fq_linears_static.restype = ci
    L.fq_linears_static.argtypes = [ci, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp), ci, vp, vp]
    L.fq_entropy_kl.restype = ci
    L.fq_entropy_kl.argtypes = [vp, vp, ci, ci, vp, vp, vp]
    L.fq_entropy_kl_f16.restype = ci
    L.fq_entropy_kl_f16.argtypes = [vp, vp, ci, ci, vp, vp, vp]
    L.fq_rank_ascending.restype = ci
    L.fq_rank_ascending.argtypes = [vp, ci, ci, vp, vp]
    L.fq_quantize_sym.restype = ci
    L.fq_quantize_sym.argtypes = [vp, ci, ci, ci, ci, vp, vp, vp, vp]
    L.fq_fake_quantize.restype = ci
    L.fq_fake_quantize.argtypes = [vp, ci, ci, ci, ci, ci, vp, vp]
    L.fq_lm_head_entropy.restype = ci
    L.fq_lm_head_entropy.argtypes = [vp, vp, ci, ci, ci, vp, vp, vp, vp]
    L.fq_quantize_act.restype = ci
    L.fq_quantize_act.argtypes = [vp, ci, ci, vp, vp, vp, vp]
    L.fq_linear_w8a8.restype = ci
    L.fq_linear_w8a8.argtypes = [vp, vp, vp, vp, ci, vp, vp]
    L.fq_sched_state_bytes.restype = sz
    L.fq_sched_state_bytes.argtypes = [ci]
    L.fq_sched_init.restype = ci
    L.fq_sched_init.argtypes = [vp, ci, ctypes.c_double, ci, vp, vp, ci, vp, ci, vp, vp]
    L.fq_sched_threshold_from_prefill.restype = ci
    L.fq_sched_threshold_from_prefill.argtypes = [vp, vp, ci, ci, vp]
    L.fq_sched_step.restype = ci
    L.fq_sched_step.argtypes = [vp, vp, vp]
    L.fq_sched_peek.restype = ci
    L.fq_sched_peek.argtypes = [vp, ctypes.POINTER(ci), ctypes.POINTER(ci), ctypes.POINTER(ctypes.c_double),
                                ctypes.POINTER(ctypes.c_double), vp]
    return L


lib = _load()


def fq_last_error() -> str:
    return lib.fq_last_error().decode()


def _check(rc: int) -> None:
    if rc != FQ_OK:
        raise FlexqError(rc, fq_last_error())


def _ptr(t):
    """Device pointer of a torch tensor (must be contiguous), an int, or None."""
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_contiguous():
        raise ValueError("tensor must be contiguous")
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def fq_packed_sizes(N: int, K: int, bits: int, group: int = FQ_GROUP):
    c, s, z = ctypes.c_size_t(), ctypes.c_size_t(), ctypes.c_size_t()
    _check(lib.fq_packed_sizes(N, K, bits, group, ctypes.byref(c), ctypes.byref(s), ctypes.byref(z)))
    return c.value, s.value, z.value


def fq_quantize(w_fp16, N: int, K: int, bits: int, group: int, codes, scales, zeros, stream=None):
    _check(lib.fq_quantize(_ptr(w_fp16), N, K, bits, group, _ptr(codes), _ptr(scales), _ptr(zeros),
                           _stream(stream)))


def fq_quantize_sym(w_fp16, N: int, K: int, bits: int, group: int, codes, scales, zeros, stream=None):
    _check(lib.fq_quantize_sym(_ptr(w_fp16), N, K, bits, group, _ptr(codes), _ptr(scales), _ptr(zeros),
                               _stream(stream)))


def fq_fake_quantize(w_fp16, N: int, K: int, bits: int, group: int, symmetric: bool, w_hat_fp16, stream=None):
    _check(lib.fq_fake_quantize(_ptr(w_fp16), N, K, bits, group, 1 if symmetric else 0, _ptr(w_hat_fp16),
                                _stream(stream)))


class Layer:
    """Owns an ``fq_layer`` handle and keeps the attached tensors alive."""

    def __init__(self, N: int, K: int, group: int = FQ_GROUP):
        h = ctypes.c_void_p()
        _check(lib.fq_layer_create(ctypes.byref(h), N, K, group))
        self.handle = h
        self.N, self.K, self.group = N, K, group
        self._keep = {}

    def attach(self, bits: int, codes, scales=None, zeros=None):
        _check(lib.fq_layer_attach(self.handle, bits, _ptr(codes), _ptr(scales), _ptr(zeros)))
        self._keep[bits] = (codes, scales, zeros)
        return self

    def destroy(self):
        if self.handle is not None:
            _check(lib.fq_layer_destroy(self.handle))
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def fq_linear(layer: Layer, bits: int, x_fp16, M: int, y_fp16, stream=None):
    _check(lib.fq_linear(layer.handle, bits, _ptr(x_fp16), M, _ptr(y_fp16), _stream(stream)))


class Plan:
    """Owns an ``fq_plan``: ``count`` independent linears run by one launch, the
    bit-width of each read from a device int32 array at run time."""

    def __init__(self, layers, xs, ys, M: int, workspace, stream=None):
        n = len(layers)
        arr = ctypes.c_void_p * max(n, 1)
        self._keep = (list(layers), list(xs), list(ys), workspace)
        h = ctypes.c_void_p()
        ws_bytes = workspace.numel() * workspace.element_size() if hasattr(workspace, "numel") else 0
        _check(lib.fq_plan_create(
            ctypes.byref(h), n, arr(*[l.handle for l in layers]), arr(*[_ptr(x) for x in xs]),
            arr(*[_ptr(y) for y in ys]), M, _ptr(workspace), ws_bytes, _stream(stream)))
        self.handle = h
        self.count = n

    @staticmethod
    def workspace_bytes(count: int) -> int:
        return int(lib.fq_plan_workspace_bytes(count))

    def run(self, bits_dev, stream=None):
        _check(lib.fq_plan_run(self.handle, _ptr(bits_dev), _stream(stream)))

    def status(self, stream=None):
        """Waits for ``stream``; returns (launches that gave up, flags) -- flags bit 0: in some run an
        entry's bit-width could not be served (not attached, or no kernel for it at this M)."""
        g, f = ctypes.c_int32(0), ctypes.c_int32(0)
        _check(lib.fq_plan_status(self.handle, ctypes.byref(g), ctypes.byref(f), _stream(stream)))
        return int(g.value), int(f.value)

    def destroy(self):
        if self.handle is not None:
            _check(lib.fq_plan_destroy(self.handle))
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


class StagedPlan(Plan):
    """Owns a stage-ordered ``fq_plan``: entry i belongs to stage ``stage[i]`` (host ints, never
    decreasing); one launch runs the stages in order."""

    def __init__(self, layers, xs, ys, stage, M: int, workspace, stream=None):
        n = len(layers)
        arr = ctypes.c_void_p * max(n, 1)
        st = (ctypes.c_int32 * max(n, 1))(*[int(v) for v in stage])
        self._keep = (list(layers), list(xs), list(ys), workspace)
        h = ctypes.c_void_p()
        ws_bytes = workspace.numel() * workspace.element_size() if hasattr(workspace, "numel") else 0
        _check(lib.fq_plan_create_staged(
            ctypes.byref(h), n, arr(*[l.handle for l in layers]), arr(*[_ptr(x) for x in xs]),
            arr(*[_ptr(y) for y in ys]), st, M, _ptr(workspace), ws_bytes, _stream(stream)))
        self.handle = h
        self.count = n

    @staticmethod
    def workspace_bytes(count: int, n_stages: int) -> int:
        return int(lib.fq_plan_staged_workspace_bytes(count, n_stages))

    def set_wait_limit(self, polls: int):
        _check(lib.fq_plan_set_wait_limit(self.handle, polls))


def fq_stream_read(src, nbytes: int, sink, stream=None):
    _check(lib.fq_stream_read(_ptr(src), nbytes, _ptr(sink), _stream(stream)))


def fq_linears_static(layers, xs, ys, M: int, bits_dev, stream=None):
    n = len(layers)
    arr = ctypes.c_void_p * max(n, 1)
    _check(lib.fq_linears_static(n, arr(*[l.handle for l in layers]), arr(*[_ptr(x) for x in xs]),
                                 arr(*[_ptr(y) for y in ys]), M, _ptr(bits_dev), _stream(stream)))


def fq_entropy_kl(logits_p, logits_q, R: int, V: int, entropy_out, kl_out, stream=None):
    _check(lib.fq_entropy_kl(_ptr(logits_p), _ptr(logits_q), R, V, _ptr(entropy_out), _ptr(kl_out),
                             _stream(stream)))


def fq_entropy_kl_f16(logits_p, logits_q, R: int, V: int, entropy_out, kl_out, stream=None):
    _check(lib.fq_entropy_kl_f16(_ptr(logits_p), _ptr(logits_q), R, V, _ptr(entropy_out), _ptr(kl_out),
                                 _stream(stream)))


def fq_rank_ascending(values, n: int, m: int, order, stream=None):
    _check(lib.fq_rank_ascending(_ptr(values), n, m, _ptr(order), _stream(stream)))


def fq_lm_head_entropy(x, w, M: int, V: int, K: int, logits, H, argmax=None, stream=None):
    _check(lib.fq_lm_head_entropy(_ptr(x), _ptr(w), M, V, K, _ptr(logits), _ptr(H), _ptr(argmax), _stream(stream)))


def fq_quantize_act(x, M: int, K: int, xq, sx, xsum, stream=None):
    _check(lib.fq_quantize_act(_ptr(x), M, K, _ptr(xq), _ptr(sx), _ptr(xsum), _stream(stream)))


def fq_linear_w8a8(layer, xq, sx, xsum, M: int, y, stream=None):
    _check(lib.fq_linear_w8a8(layer.handle, _ptr(xq), _ptr(sx), _ptr(xsum), M, _ptr(y), _stream(stream)))


def fq_sched_state_bytes(window: int) -> int:
    return int(lib.fq_sched_state_bytes(window))


def fq_sched_init(state, window: int, thre: float, per_trigger: int, ev_entry, ev_bits, n_events: int,
                  bits, ev_token=None, stream=None, entries: int | None = None):
    """`entries` defaults to the length of the `bits` tensor."""
    if entries is None:
        entries = bits.numel()
    _check(lib.fq_sched_init(_ptr(state), window, thre, per_trigger, _ptr(ev_entry), _ptr(ev_bits),
                             n_events, _ptr(bits), entries, _ptr(ev_token), _stream(stream)))


def fq_sched_threshold_from_prefill(state, entropy, R: int, last_n: int, stream=None):
    _check(lib.fq_sched_threshold_from_prefill(_ptr(state), _ptr(entropy), R, last_n, _stream(stream)))


def fq_sched_step(state, entropy, stream=None):
    _check(lib.fq_sched_step(_ptr(state), _ptr(entropy), _stream(stream)))


def fq_sched_peek(state, stream=None):
    """Returns (next_event, tokens, thre, last_mean) after waiting for the stream."""
    ne, tk = ctypes.c_int(), ctypes.c_int()
    th, lm = ctypes.c_double(), ctypes.c_double()
    _check(lib.fq_sched_peek(_ptr(state), ctypes.byref(ne), ctypes.byref(tk), ctypes.byref(th),
                             ctypes.byref(lm), _stream(stream)))
    return ne.value, tk.value, th.value, lm.value

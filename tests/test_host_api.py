"""Host-side logic of the C ABI, checked without a GPU: the library loads, exports every
symbol include/flexq.h declares, and rejects bad arguments before launching anything."""
import ctypes
import os
import re

import pytest

import paper_2506_12024_amd as fq
from paper_2506_12024_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "flexq.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fq_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_functions()
    assert set(names) == set(B.EXPORTS), "binding.EXPORTS and include/flexq.h disagree"
    for n in names:
        assert hasattr(fq.lib, n), n


def test_packed_sizes():
    assert fq.fq_packed_sizes(4096, 4096, 4) == (4096 * 4096 // 2, 4096 * 32 * 4, 4096 * 32)
    assert fq.fq_packed_sizes(11008, 4096, 8) == (11008 * 4096, 11008 * 32 * 4, 11008 * 32)
    assert fq.fq_packed_sizes(256, 4096, 3) == (256 * 4096 * 3 // 8, 256 * 32 * 4, 256 * 32)
    for args, code in [((4096, 4096, 5, 128), B.FQ_ERR_BITS), ((4096, 4000, 4, 128), B.FQ_ERR_SHAPE),
                       ((0, 4096, 4, 128), B.FQ_ERR_SHAPE), ((16, 256, 4, 64), B.FQ_ERR_SHAPE)]:
        with pytest.raises(fq.FlexqError) as ei:
            fq.fq_packed_sizes(*args)
        assert ei.value.code == code
        assert fq.fq_last_error()


FAKE = 0x1000  # a non-NULL, 16-byte aligned value; never dereferenced: validation fails first


def test_quantize_validation():
    L = fq.lib
    assert L.fq_quantize(None, 16, 256, 4, 128, FAKE, FAKE, FAKE, None) == B.FQ_ERR_NULL
    assert L.fq_quantize(FAKE, 16, 256, 5, 128, FAKE, FAKE, FAKE, None) == B.FQ_ERR_BITS
    assert L.fq_quantize(FAKE, 16, 200, 4, 128, FAKE, FAKE, FAKE, None) == B.FQ_ERR_SHAPE
    assert L.fq_quantize(FAKE + 2, 16, 256, 4, 128, FAKE, FAKE, FAKE, None) == B.FQ_ERR_ALIGN
    assert b"alignment" in L.fq_last_error()


def test_layer_and_linear_validation():
    L = fq.lib
    h = ctypes.c_void_p()
    assert L.fq_layer_create(ctypes.byref(h), 16, 200, 128) == B.FQ_ERR_SHAPE
    assert L.fq_layer_create(None, 16, 256, 128) == B.FQ_ERR_NULL
    assert L.fq_layer_create(ctypes.byref(h), 16, 256, 128) == B.FQ_OK
    assert L.fq_layer_attach(h, 5, FAKE, FAKE, FAKE) == B.FQ_ERR_BITS
    assert L.fq_layer_attach(h, 4, None, FAKE, FAKE) == B.FQ_ERR_NULL
    assert L.fq_layer_attach(h, 4, FAKE, None, FAKE) == B.FQ_ERR_NULL
    assert L.fq_layer_attach(h, 4, FAKE + 8, FAKE, FAKE) == B.FQ_ERR_ALIGN
    assert L.fq_layer_attach(h, 4, FAKE, FAKE, FAKE) == B.FQ_OK
    assert L.fq_layer_attach(None, 4, FAKE, FAKE, FAKE) == B.FQ_ERR_NULL
    # linear: every rejection happens before a launch
    assert L.fq_linear(h, 8, FAKE, 1, FAKE, None) == B.FQ_ERR_NOT_ATTACHED
    assert L.fq_linear(h, 16, FAKE, 1, FAKE, None) == B.FQ_ERR_NOT_ATTACHED
    assert L.fq_linear(h, 5, FAKE, 1, FAKE, None) == B.FQ_ERR_BITS
    assert L.fq_linear(h, 4, None, 1, FAKE, None) == B.FQ_ERR_NULL
    assert L.fq_linear(h, 4, FAKE, 0, FAKE, None) == B.FQ_ERR_SHAPE
    assert L.fq_linear(h, 4, FAKE + 4, 1, FAKE, None) == B.FQ_ERR_ALIGN
    assert L.fq_linear(None, 4, FAKE, 1, FAKE, None) == B.FQ_ERR_NULL
    # plan validation
    p = ctypes.c_void_p()
    arr = (ctypes.c_void_p * 1)
    assert L.fq_plan_workspace_bytes(0) == 0
    ws = L.fq_plan_workspace_bytes(3)
    assert ws >= 3 * 64 and ws % 256 == 0
    assert L.fq_plan_create(ctypes.byref(p), 0, arr(h), arr(FAKE), arr(FAKE), 1, FAKE, 4096, None) == B.FQ_ERR_SHAPE
    assert L.fq_plan_create(ctypes.byref(p), 1, arr(h), arr(FAKE), arr(FAKE), 33, 0x1000, 4096, None) == B.FQ_ERR_SHAPE
    assert L.fq_plan_create(ctypes.byref(p), 1, arr(h), arr(FAKE), arr(FAKE), 1, 0x1000, 8, None) == B.FQ_ERR_SHAPE
    assert L.fq_plan_create(ctypes.byref(p), 1, arr(h), arr(FAKE), arr(FAKE), 1, 0x1010, 4096, None) == B.FQ_ERR_ALIGN
    assert L.fq_plan_create(ctypes.byref(p), 1, arr(h), arr(None), arr(FAKE), 1, 0x1000, 4096, None) == B.FQ_ERR_NULL
    assert L.fq_plan_run(None, FAKE, None) == B.FQ_ERR_NULL
    assert L.fq_plan_destroy(None) == B.FQ_ERR_NULL
    assert L.fq_layer_destroy(h) == B.FQ_OK
    assert L.fq_layer_destroy(None) == B.FQ_ERR_NULL


def test_plan_refuses_rows_beyond_the_decode_limit():
    text = open(os.path.join(ROOT, "include", "flexq.h")).read()
    limit = int(re.search(r"#define\s+FQ_MAX_DECODE_K\s+(\d+)", text).group(1))
    assert limit == 32768
    L, FAKE = fq.lib, 0x1000
    arr = (ctypes.c_void_p * 1)
    for K, want in ((limit, B.FQ_OK), (limit + 128, B.FQ_ERR_SHAPE)):
        h, p = ctypes.c_void_p(), ctypes.c_void_p()
        assert L.fq_layer_create(ctypes.byref(h), 64, K, 128) == B.FQ_OK
        assert L.fq_layer_attach(h, 4, FAKE, FAKE, FAKE) == B.FQ_OK
        if want == B.FQ_OK:  # creating the plan would copy its table to the device
            assert L.fq_layer_destroy(h) == B.FQ_OK
            continue
        assert L.fq_plan_create(ctypes.byref(p), 1, arr(h), arr(FAKE), arr(FAKE), 1, 0x1000, 4096, None) == want
        assert "decode limit" in fq.fq_last_error()
        assert L.fq_layer_destroy(h) == B.FQ_OK


def test_entropy_validation():
    L = fq.lib
    assert L.fq_entropy_kl(FAKE, None, 1, 0, FAKE, None, None) == B.FQ_ERR_SHAPE
    assert L.fq_entropy_kl(FAKE, None, -1, 8, FAKE, None, None) == B.FQ_ERR_SHAPE
    assert L.fq_entropy_kl(None, None, 1, 8, FAKE, None, None) == B.FQ_ERR_NULL
    assert L.fq_entropy_kl(FAKE, FAKE, 1, 8, FAKE, None, None) == B.FQ_ERR_NULL
    assert L.fq_entropy_kl(FAKE, None, 1, 8, FAKE, FAKE, None) == B.FQ_ERR_NULL
    assert L.fq_entropy_kl(FAKE + 2, None, 1, 8, FAKE, None, None) == B.FQ_ERR_ALIGN
    # R = 0 is valid and launches nothing
    assert L.fq_entropy_kl(FAKE, None, 0, 8, FAKE, None, None) == B.FQ_OK


def test_package_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2506_12024_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.replace("no oracle", ""), os.path.join(dirpath, f)


def test_sched_validation():
    L = fq.lib
    assert L.fq_sched_state_bytes(0) == 0 and L.fq_sched_state_bytes(1025) == 0
    assert L.fq_sched_state_bytes(20) >= 64 + 20 * 8 and L.fq_sched_state_bytes(20) % 256 == 0
    assert L.fq_sched_init(None, 20, 2.0, 1, FAKE, FAKE, 4, FAKE, 8, None, None) == B.FQ_ERR_NULL
    assert L.fq_sched_init(FAKE, 20, 2.0, 1, FAKE, FAKE, 4, None, 8, None, None) == B.FQ_ERR_NULL
    assert L.fq_sched_init(FAKE, 0, 2.0, 1, FAKE, FAKE, 4, FAKE, 8, None, None) == B.FQ_ERR_SHAPE
    assert L.fq_sched_init(FAKE, 20, 2.0, 0, FAKE, FAKE, 4, FAKE, 8, None, None) == B.FQ_ERR_SHAPE
    assert L.fq_sched_init(FAKE, 20, 2.0, 1, None, FAKE, 4, FAKE, 8, None, None) == B.FQ_ERR_NULL
    assert L.fq_sched_init(FAKE + 4, 20, 2.0, 1, FAKE, FAKE, 4, FAKE, 8, None, None) == B.FQ_ERR_ALIGN
    assert L.fq_sched_init(FAKE, 20, 2.0, 1, FAKE, FAKE, 4, FAKE, 0, None, None) == B.FQ_ERR_SHAPE
    assert L.fq_sched_step(None, FAKE, None) == B.FQ_ERR_NULL
    assert L.fq_sched_step(FAKE, None, None) == B.FQ_ERR_NULL
    assert L.fq_sched_threshold_from_prefill(FAKE, FAKE, 0, 3, None) == B.FQ_ERR_SHAPE
    assert L.fq_sched_peek(None, None, None, None, None, None) == B.FQ_ERR_NULL


def test_entropy_f16_and_rank_validation():
    L = fq.lib
    assert L.fq_entropy_kl_f16(FAKE, None, 1, 0, FAKE, None, None) == B.FQ_ERR_SHAPE
    assert L.fq_entropy_kl_f16(None, None, 1, 8, FAKE, None, None) == B.FQ_ERR_NULL
    assert L.fq_entropy_kl_f16(FAKE, FAKE, 1, 8, FAKE, None, None) == B.FQ_ERR_NULL
    assert L.fq_entropy_kl_f16(FAKE + 1, None, 1, 8, FAKE, None, None) == B.FQ_ERR_ALIGN
    assert L.fq_entropy_kl_f16(FAKE, None, 0, 8, FAKE, None, None) == B.FQ_OK
    assert L.fq_rank_ascending(FAKE, -1, 1, FAKE, None) == B.FQ_ERR_SHAPE
    assert L.fq_rank_ascending(FAKE, 4, 0, FAKE, None) == B.FQ_ERR_SHAPE
    assert L.fq_rank_ascending(FAKE, 1 << 20, 1, FAKE, None) == B.FQ_ERR_SHAPE
    assert L.fq_rank_ascending(None, 4, 1, FAKE, None) == B.FQ_ERR_NULL
    assert L.fq_rank_ascending(FAKE, 4, 1, None, None) == B.FQ_ERR_NULL
    assert L.fq_rank_ascending(FAKE + 2, 4, 1, FAKE, None) == B.FQ_ERR_ALIGN
    assert L.fq_rank_ascending(FAKE, 0, 1, FAKE, None) == B.FQ_OK


def test_w8a8_validation():
    L = fq.lib
    assert L.fq_quantize_act(FAKE, -1, 256, FAKE, FAKE, FAKE, None) == B.FQ_ERR_SHAPE
    assert L.fq_quantize_act(FAKE, 4, 200, FAKE, FAKE, FAKE, None) == B.FQ_ERR_SHAPE
    assert L.fq_quantize_act(FAKE, 4, 0, FAKE, FAKE, FAKE, None) == B.FQ_ERR_SHAPE
    assert L.fq_quantize_act(None, 4, 256, FAKE, FAKE, FAKE, None) == B.FQ_ERR_NULL
    assert L.fq_quantize_act(FAKE, 4, 256, FAKE, FAKE, None, None) == B.FQ_ERR_NULL
    assert L.fq_quantize_act(FAKE, 4, 256, FAKE + 8, FAKE, FAKE, None) == B.FQ_ERR_ALIGN
    assert L.fq_quantize_act(FAKE, 0, 256, FAKE, FAKE, FAKE, None) == B.FQ_OK
    h = ctypes.c_void_p()
    assert L.fq_layer_create(ctypes.byref(h), 16, 256, 128) == B.FQ_OK
    assert L.fq_linear_w8a8(None, FAKE, FAKE, FAKE, 4, FAKE, None) == B.FQ_ERR_NULL
    assert L.fq_linear_w8a8(h, FAKE, FAKE, FAKE, 4, FAKE, None) == B.FQ_ERR_NOT_ATTACHED
    assert L.fq_layer_attach(h, 4, FAKE, FAKE, FAKE) == B.FQ_OK
    assert L.fq_linear_w8a8(h, FAKE, FAKE, FAKE, 4, FAKE, None) == B.FQ_ERR_NOT_ATTACHED
    assert L.fq_layer_attach(h, 8, FAKE, FAKE, FAKE) == B.FQ_OK
    assert L.fq_linear_w8a8(h, None, FAKE, FAKE, 4, FAKE, None) == B.FQ_ERR_NULL
    assert L.fq_linear_w8a8(h, FAKE, FAKE, None, 4, FAKE, None) == B.FQ_ERR_NULL
    assert L.fq_linear_w8a8(h, FAKE, FAKE, FAKE, 0, FAKE, None) == B.FQ_ERR_SHAPE
    assert L.fq_linear_w8a8(h, FAKE + 4, FAKE, FAKE, 4, FAKE, None) == B.FQ_ERR_ALIGN
    assert L.fq_linear_w8a8(h, FAKE, FAKE, FAKE, 4, FAKE + 1, None) == B.FQ_ERR_ALIGN
    assert L.fq_layer_destroy(h) == B.FQ_OK


def test_one_scale_per_row_is_an_8_bit_copy_for_w8a8_only():
    L = fq.lib
    assert fq.fq_packed_sizes(64, 1024, 8, 1024) == (64 * 1024, 64 * 4, 64)
    with pytest.raises(fq.FlexqError):
        fq.fq_packed_sizes(64, 1024, 4, 1024)               # 8 bits only
    with pytest.raises(fq.FlexqError):
        fq.fq_packed_sizes(64, 1000, 8, 1000)               # K a multiple of 128
    with pytest.raises(fq.FlexqError):
        fq.fq_packed_sizes(64, 131072, 8, 131072)           # int32 sums over the row: K <= 65536
    with pytest.raises(fq.FlexqError):
        fq.fq_packed_sizes(64, 1024, 8, 256)                # no other group size
    assert L.fq_quantize(FAKE, 64, 1024, 4, 1024, FAKE, FAKE, FAKE, None) == B.FQ_ERR_SHAPE
    h = ctypes.c_void_p()
    assert L.fq_layer_create(ctypes.byref(h), 64, 1024, 1024) == B.FQ_OK
    assert L.fq_layer_attach(h, 4, FAKE, FAKE, FAKE) == B.FQ_ERR_BITS
    assert L.fq_layer_attach(h, 16, FAKE, None, None) == B.FQ_ERR_BITS
    assert L.fq_layer_attach(h, 8, FAKE, FAKE, FAKE) == B.FQ_OK
    assert L.fq_linear(h, 8, FAKE, 1, FAKE, None) == B.FQ_ERR_SHAPE
    assert "fq_linear_w8a8" in fq.fq_last_error()
    assert L.fq_linear_w8a8(h, FAKE, None, FAKE, 4, FAKE, None) == B.FQ_ERR_NULL   # (validated like the others)
    assert L.fq_layer_destroy(h) == B.FQ_OK


def test_2bit_copy_limits():
    L = fq.lib
    vp_odd = ctypes.c_void_p(FAKE + 1)
    assert fq.fq_packed_sizes(4096, 4096, 2) == (4096 * 4096 // 4, 4096 * 32 * 4, 4096 * 32)
    h = ctypes.c_void_p()
    assert L.fq_layer_create(ctypes.byref(h), 64, 256, 128) == B.FQ_OK
    assert L.fq_layer_attach(h, 2, FAKE, FAKE, FAKE) == B.FQ_OK
    assert L.fq_layer_attach(h, 2, FAKE, None, FAKE) == B.FQ_ERR_NULL
    assert L.fq_layer_attach(h, 3, FAKE, FAKE, FAKE) == B.FQ_OK
    assert L.fq_linear(h, 3, FAKE, 2, vp_odd, None) == B.FQ_ERR_ALIGN  # 3 bits at any batch: checked like the others
    assert L.fq_linear(h, 4, FAKE, 1, FAKE, None) == B.FQ_ERR_NOT_ATTACHED
    assert L.fq_layer_destroy(h) == B.FQ_OK


def test_sym_and_fake_quantize_validation():
    L, vp = fq.lib, ctypes.c_void_p
    ok = vp(FAKE)
    assert L.fq_quantize_sym(None, 4, 128, 4, 128, ok, ok, ok, None) == B.FQ_ERR_NULL
    assert L.fq_quantize_sym(ok, 4, 128, 5, 128, ok, ok, ok, None) == B.FQ_ERR_BITS
    assert L.fq_quantize_sym(ok, 4, 100, 4, 128, ok, ok, ok, None) == B.FQ_ERR_SHAPE
    assert L.fq_quantize_sym(vp(FAKE + 8), 4, 128, 4, 128, ok, ok, ok, None) == B.FQ_ERR_ALIGN
    assert L.fq_fake_quantize(ok, 4, 128, 1, 128, 0, ok, None) == B.FQ_ERR_BITS
    assert L.fq_fake_quantize(ok, 4, 128, 9, 128, 0, ok, None) == B.FQ_ERR_BITS
    assert L.fq_fake_quantize(ok, 4, 128, 3, 128, 0, None, None) == B.FQ_ERR_NULL
    assert L.fq_fake_quantize(ok, 4, 128, 3, 64, 0, ok, None) == B.FQ_ERR_SHAPE
    assert L.fq_fake_quantize(ok, 4, 128, 3, 128, 1, vp(FAKE + 8), None) == B.FQ_ERR_ALIGN
    assert "fq_fake_quantize" in fq.fq_last_error()


def test_lm_head_entropy_validation():
    L, vp = fq.lib, ctypes.c_void_p
    ok = vp(FAKE)
    assert L.fq_lm_head_entropy(ok, ok, 0, 100, 512, None, ok, None, None) == B.FQ_ERR_SHAPE
    assert L.fq_lm_head_entropy(ok, ok, 5, 100, 512, None, ok, None, None) == B.FQ_ERR_SHAPE
    assert L.fq_lm_head_entropy(ok, ok, 1, 100, 500, None, ok, None, None) == B.FQ_ERR_SHAPE
    assert L.fq_lm_head_entropy(ok, ok, 4, 100, 16384, None, ok, None, None) == B.FQ_ERR_SHAPE
    assert L.fq_lm_head_entropy(ok, ok, 1, 0, 512, None, ok, None, None) == B.FQ_ERR_SHAPE
    assert L.fq_lm_head_entropy(ok, None, 1, 100, 512, None, ok, None, None) == B.FQ_ERR_NULL
    assert L.fq_lm_head_entropy(ok, ok, 1, 100, 512, None, None, None, None) == B.FQ_ERR_NULL
    assert L.fq_lm_head_entropy(vp(FAKE + 8), ok, 1, 100, 512, None, ok, None, None) == B.FQ_ERR_ALIGN
    assert "fq_lm_head_entropy" in fq.fq_last_error()


def test_linears_static_validation():
    # the entry point that allocates nothing rejects bad arguments, and sizes beyond its static
    # workspace, before any HIP call
    L = fq.lib
    h = ctypes.c_void_p()
    assert L.fq_layer_create(ctypes.byref(h), 16, 256, 128) == B.FQ_OK
    assert L.fq_layer_attach(h, 4, FAKE, FAKE, FAKE) == B.FQ_OK
    arr = (ctypes.c_void_p * 1)
    assert L.fq_linears_static(1, arr(h), arr(FAKE), arr(FAKE), 1, None, None) == B.FQ_ERR_NULL
    assert L.fq_linears_static(1, arr(h), arr(FAKE), arr(FAKE), 1, FAKE + 2, None) == B.FQ_ERR_ALIGN
    assert L.fq_linears_static(0, arr(h), arr(FAKE), arr(FAKE), 1, FAKE, None) == B.FQ_ERR_SHAPE
    assert L.fq_linears_static(1, arr(h), arr(FAKE), arr(FAKE), 33, FAKE, None) == B.FQ_ERR_SHAPE
    assert L.fq_linears_static(1, None, arr(FAKE), arr(FAKE), 1, FAKE, None) == B.FQ_ERR_NULL
    assert L.fq_linears_static(1, arr(h), arr(None), arr(FAKE), 1, FAKE, None) == B.FQ_ERR_NULL
    assert L.fq_linears_static(1, arr(h), arr(FAKE + 4), arr(FAKE), 1, FAKE, None) == B.FQ_ERR_ALIGN
    n = B.FQ_STATIC_MAX_ENTRIES + 1
    many = (ctypes.c_void_p * n)
    assert L.fq_linears_static(n, many(*[h.value] * n), many(*[FAKE] * n), many(*[FAKE] * n), 1, FAKE,
                               None) == B.FQ_ERR_SHAPE
    assert b"FQ_STATIC_MAX_ENTRIES" in L.fq_last_error()
    assert L.fq_layer_destroy(h) == B.FQ_OK


def test_staged_plan_validation():
    # every rejection of a stage-ordered plan happens before a HIP call
    L = fq.lib
    h = ctypes.c_void_p()
    assert L.fq_layer_create(ctypes.byref(h), 16, 256, 128) == B.FQ_OK
    assert L.fq_layer_attach(h, 4, FAKE, FAKE, FAKE) == B.FQ_OK
    p = ctypes.c_void_p()
    arr3 = (ctypes.c_void_p * 3)
    st = (ctypes.c_int32 * 3)
    hs = arr3(h.value, h.value, h.value)
    xs, ys = arr3(FAKE, FAKE, FAKE), arr3(FAKE + 0x100, FAKE + 0x200, FAKE + 0x300)
    assert L.fq_plan_staged_workspace_bytes(0, 1) == 0 and L.fq_plan_staged_workspace_bytes(3, 4) == 0
    ws = L.fq_plan_staged_workspace_bytes(3, 2)
    assert ws % 256 == 0 and ws >= 3 * 64 + 12 + 1156

    def create(stage, M=1, workspace=0x10000, bytes_=1 << 20, xs_=xs, ys_=ys):
        return L.fq_plan_create_staged(ctypes.byref(p), 3, hs, xs_, ys_, st(*stage), M, workspace, bytes_, None)

    assert create([1, 1, 2]) == B.FQ_ERR_SHAPE             # must start at 0
    assert create([0, 2, 2]) == B.FQ_ERR_SHAPE             # rises by more than one
    assert create([0, 1, 0]) == B.FQ_ERR_SHAPE             # decreases
    assert create([0, 0, 1], M=2) == B.FQ_ERR_SHAPE        # batch 1 only
    assert create([0, 0, 1], bytes_=64) == B.FQ_ERR_SHAPE  # workspace too small
    assert create([0, 0, 1], workspace=0x10010) == B.FQ_ERR_ALIGN
    assert L.fq_plan_create_staged(ctypes.byref(p), 3, hs, xs, ys, None, 1, 0x10000, 1 << 20, None) == B.FQ_ERR_NULL
    # an entry may read what an EARLIER stage wrote, not what its own or a later stage writes
    assert create([0, 0, 1], xs_=arr3(FAKE, FAKE + 0x100, FAKE)) == B.FQ_ERR_SHAPE   # x1 = y0, same stage
    assert create([0, 1, 1], xs_=arr3(FAKE + 0x300, FAKE, FAKE)) == B.FQ_ERR_SHAPE   # x0 = y2, later stage
    assert b"stage" in L.fq_last_error()
    assert L.fq_plan_set_wait_limit(None, 5) == B.FQ_ERR_NULL
    assert L.fq_plan_status(None, None, None, None) == B.FQ_ERR_NULL
    assert L.fq_layer_destroy(h) == B.FQ_OK

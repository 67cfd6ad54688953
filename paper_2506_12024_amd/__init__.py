"""MI355X (gfx950) implementation of FlexQuant's decode hot path (arXiv 2506.12024).

The package is a thin ctypes binding over ``libflexq.so`` (C ABI: ``include/flexq.h``);
every step of the path runs in the library's HIP kernels.  There is no CPU fallback: the
first use of any name below loads the library and raises if it has not been built
(``python -m paper_2506_12024_amd.build``).
"""
_EXPORTS = (
    "FQ_GROUP", "FQ_MAX_DECODE_M", "FlexqError", "Layer", "Plan", "StagedPlan", "fq_entropy_kl", "fq_entropy_kl_f16",
    "fq_last_error", "fq_linear", "fq_linear_w8a8", "fq_packed_sizes", "fq_quantize", "fq_quantize_act",
    "fq_quantize_sym", "fq_fake_quantize", "fq_lm_head_entropy", "FQ_MAX_LM_HEAD_M",
    "fq_linears_static", "fq_stream_read", "FQ_STATIC_MAX_ENTRIES", "FQ_SCRATCH_BANKS",
    "fq_rank_ascending", "fq_sched_init", "fq_sched_peek",
    "fq_sched_state_bytes", "fq_sched_step", "fq_sched_threshold_from_prefill", "lib", "lib_path",
)


def __getattr__(name):
    # Loaded on first use so that the build module can run while the library is stale or absent.
    if name in _EXPORTS:
        from . import binding
        return getattr(binding, name)
    raise AttributeError("module %r has no attribute %r" % (__name__, name))


def __dir__():
    return sorted(list(globals()) + list(_EXPORTS))

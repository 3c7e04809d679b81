"""Partitioned decode attention for AMD MI355X (gfx950): hand-written HIP kernels behind a
C ABI (``include/hg_attn.h``) plus this thin Python binding.

``hg_attn_partial`` / ``hg_attn_merge`` / ``hg_attn_full`` are resolved lazily so that importing
the package (for example to reach ``workloads``) does not require the built library.
"""

_API = (
    "hg_attn_partial",
    "hg_attn_partial_static",
    "hg_attn_partial_merge",
    "hg_attn_profile_times",
    "hg_attn_build_id",
    "hg_attn_merge",
    "hg_attn_merge2",
    "hg_attn_full",
    "hg_attn_logits",
    "hg_attn_concat",
    "hg_attn_select",
    "hg_attn_gather",
    "hg_attn_topk",
    "hg_sched_init",
    "hg_sched_step",
    "HgSchedState",
    "hg_attn_plan",
    "hg_attn_set_span_tokens",
    "hg_attn_set_topk_mode",
    "hg_attn_profile_start",
    "hg_attn_profile_stop",
    "hg_attn_calibration_copy",
    "hg_attn_calibration_stream",
    "pack_ranges",
    "make_desc",
    "hg_strerror",
    "HgError",
    "load_library",
)


def __getattr__(name):
    if name in _API:
        from . import hg_attn as _binding

        return getattr(_binding, name)
    raise AttributeError(name)

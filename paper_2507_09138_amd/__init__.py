"""MI355X-native batched IVF-Flat search: thin Python binding over the C ABI of ``hr_ivf.h``.

Argument marshalling only; every step of the search runs in the HIP kernels of
``libhr_ivf.so``.  PyTorch supplies device memory and streams.

The names of ``binding`` are resolved on first use (so that ``python -m
paper_2507_09138_amd.build`` can run before the library exists); using any of them
without a built library raises ImportError.
"""
_NAMES = ["IvfIndex", "HrError", "hr_ivf_load", "hr_ivf_free", "hr_ivf_workspace_bytes",
          "hr_ivf_search", "hr_ivf_search_static", "HR_STATIC_SCRATCH_BYTES", "hr_ivf_coarse", "hr_ivf_scan", "hr_ivf_scan_step", "hr_ivf_scan_step_rows", "hr_ivf_rescore", "hr_ivf_lists_of_rows",
          "hr_ivf_reorder_probes", "reorder_probes", "hr_ivf_list_hits", "hr_ivf_hot_lists", "hr_ivf_refresh_rows", "hr_ivf_set_resident", "hr_ivf_split_probes", "hr_ivf_stats", "hr_ivf_workspace_layout", "hr_ivf_profile_begin",
          "hr_ivf_profile_end", "hr_last_error", "hr_version", "lib", "lib_path", "HR_METRIC_IP",
          "HR_METRIC_L2", "HR_F32", "HR_F16", "HR_BF16", "HR_K_MAX", "HR_NPROBE_MAX", "HR_LOAD_ROW_TABLES"]
__all__ = list(_NAMES)


def __getattr__(name):
    if name in _NAMES:
        from . import binding
        return getattr(binding, name)
    raise AttributeError(name)

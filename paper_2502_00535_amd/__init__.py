"""MI355X-native data-parallel non-maximum suppression (the map/reduce NMS of
"Work-Efficient Parallel Non-Maximum Suppression Kernels").

The computation lives in ``libnms_mi355x.so`` (HIP, gfx950) behind the C ABI of
``include/nms.h``; :mod:`paper_2502_00535_amd.binding` is a thin ctypes binding with
the same entry-point names that marshals torch tensors (device memory) and the
current HIP stream.  There is no CPU fallback: touching any entry point without the
built library raises ImportError.  ``python -m paper_2502_00535_amd.build`` compiles it.
"""
import importlib

_BINDING_NAMES = (
    "NmsError", "RunPlan", "library_path", "lib", "EXPORTS",
    "nms_status_string", "nms_version", "nms_last_launch_error", "nms_padded_n", "nms_mask_words",
    "nms_sort_workspace_bytes", "nms_workspace_bytes", "nms_host_pair_test",
    "nms_sort", "nms_sort_batched", "nms_overlap_mask", "nms_overlap_mask_batched",
    "nms_reduce", "nms_reduce_batched", "nms_run_ws", "nms_run_batched", "nms_run_ranked_batched", "nms_run_direct_batched",
    "nms_run_batched_profiled", "nms_reduce_greedy", "nms_reduce_greedy_batched",
    "nms_greedy_workspace_bytes", "nms_run_greedy_batched", "nms_run_greedy_fused_batched", "nms_run_early_exit_batched", "nms_map_matrix", "nms_reduce_matrix", "nms_ex_workspace_bytes", "nms_run_ex_batched", "NmsOptions",
    "nms_init", "nms_shutdown", "nms_run", "nms_run_static_batched", "NMS_STATIC_SCRATCH_BYTES",
)

__all__ = list(_BINDING_NAMES)


def __getattr__(name):
    # the binding (and with it the shared library) is loaded on first use, so that
    # `python -m paper_2502_00535_amd.build` can run before the library exists
    if name in _BINDING_NAMES:
        binding = importlib.import_module(".binding", __name__)
        return getattr(binding, name)
    raise AttributeError(f"module {__name__!r} has no attribute {name!r}")

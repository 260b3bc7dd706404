"""ESPO per-generation-step hot path for AMD MI355X (gfx950): Python binding of the C ABI.

`espo_step` and `espo_advantages` are thin argument-marshalling wrappers around the
shared library built from `csrc/`; nothing is computed in Python and there is no CPU
fallback.  Importing the package does not load the library; the first call does.
"""
__all__ = ["espo_step", "espo_advantages", "espo_advantages_terminal", "espo_advantages_packed", "espo_whiten", "espo_whiten_workspace_bytes", "espo_advantages_ws", "espo_advantages_terminal_ws", "espo_advantages_ws_bytes", "espo_whiten_from_ws", "espo_length_order", "espo_step_workspace_bytes", "EspoParams", "EspoError",
           "load_library", "library_path", "espo_debug_step_workspace_bytes", "espo_debug_math_errors", "espo_debug_read", "espo_debug_sweep", "espo_debug_sweep_padded",
           "espo_debug_copy", "espo_batch_stats", "espo_batch_stats_workspace_bytes", "espo_batch_stats_static", "read_batch_result",
           "BATCH_RESULT_BYTES"]


def __getattr__(name):
    if name in __all__:
        from . import binding
        return getattr(binding, name)
    raise AttributeError(name)

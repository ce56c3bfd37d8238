"""MI355X-native resharding of parallelizable tensor collections: Python face of libtpx.

The binding (and with it libtpx.so) is loaded on first use of any name below, so that
`python -m paper_2312_05181_amd.build` can run in a tree where the library does not exist yet.  There is
no fallback: without the library that first use raises ImportError."""

__all__ = ["EXPORTS", "LIB_PATH", "Plan", "TpxError", "tpx_execute", "tpx_execute_static", "tpx_free", "tpx_param_name", "tpx_plan",
           "tpx_plan_dataset", "tpx_plan_ptc", "tpx_plan_query", "tpx_probe_copy", "tpx_probe_fill", "tpx_probe_read", "tpx_set_option", "tpx_workspace_forget"]


def __getattr__(name):
    if name in __all__ or name == "binding":
        import importlib
        binding = importlib.import_module(".binding", __name__)
        return binding if name == "binding" else getattr(binding, name)
    raise AttributeError(f"module {__name__!r} has no attribute {name!r}")


def __dir__():
    return sorted(__all__ + ["binding"])

"""MI355X-native resharding of parallelizable tensor collections: Python face of libtpx."""
from .binding import (EXPORTS, LIB_PATH, Plan, TpxError, tpx_execute, tpx_free, tpx_param_name, tpx_plan,
                      tpx_plan_dataset, tpx_plan_ptc, tpx_probe_copy, tpx_set_option)

__all__ = ["EXPORTS", "LIB_PATH", "Plan", "TpxError", "tpx_execute", "tpx_free", "tpx_param_name", "tpx_plan",
           "tpx_plan_dataset", "tpx_plan_ptc", "tpx_probe_copy", "tpx_set_option"]

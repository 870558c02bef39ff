"""MI355X-native batched evaluation of GPU-memory footprint timelines for
candidate swap/recompute plans (the data-parallel core of TENSILE's plan
generation, arXiv 2105.13336).  See ``include/tensile.h`` for the C ABI."""
from .binding import (DevicePlans, tensile_apply_intervals, TasHandle, TensileError, tas_load, tensile_eval_link, tensile_eval_plans, tensile_eval_plans_per_job, tensile_greedy_plan,  # noqa: F401
                      tensile_score_candidates, tensile_score_recompute, tensile_tas_base_timeline, tensile_tas_free, tensile_tas_info, tensile_tas_update_latencies,
                      tensile_tas_load, tensile_validate_plans, tensile_version, tensile_eval_plans_static, tensile_eval_score_plans, tensile_tuning_set,
                      tensile_tuning_reset)

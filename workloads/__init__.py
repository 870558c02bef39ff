"""Seeded synthetic inputs (tensor access sequences and candidate plans).

Shared by the oracle's tests and the GPU path; holds none of the method's
arithmetic.
"""
from .tas import TAS, Trace, tas_from_lists, tas_hash  # noqa: F401
from .plans import Plans, make_plans, make_plans_numpy, plans_from_lists, plans_hash, eligible_gaps  # noqa: F401
from .configs import CONFIGS, make_tas, make_config_plans, small_random_tas  # noqa: F401

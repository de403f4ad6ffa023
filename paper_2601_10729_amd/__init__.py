"""MI355X-native decode attention over an HBM/host-split paged KV cache (liborbit + binding)."""
from .binding import (  # noqa: F401
    EXPORTS,
    ORBIT_E_CAPACITY,
    ORBIT_E_HIP,
    ORBIT_E_HOST_CAPACITY,
    ORBIT_E_INVAL,
    ORBIT_E_NOT_FOUND,
    ORBIT_E_STATE,
    OrbitContext,
    OrbitError,
    lib,
    orbit_distance_options,
    orbit_distance_pattern,
    orbit_model_latency,
    orbit_plan_check,
    orbit_plan_search,
)

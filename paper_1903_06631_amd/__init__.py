"""liblap: lifetime-aware memory-pool planning on MI355X (hand-written HIP, gfx950).

Thin Python binding over the C-ABI library declared in include/lap.h.  PyTorch
is used for device memory and streams only; every step of the planner runs in
the library's kernels.  There is no CPU fallback: if liblap.so is missing or a
call fails, an exception is raised.
"""
from .binding import (  # noqa: F401
    OPT_SEG_MIN_VARS,
    OPT_SEG_TRIAL_PERCENT,
    SEG_MIN_VARS_DEFAULT,
    SEG_TRIAL_PERCENT_DEFAULT,
    DeviceTrace,
    LapError,
    detect_iteration,
    evaluate_weights,
    lib_path,
    load_library,
    load_profile,
    load_profile_static,
    plan_pool,
    profile_enable,
    profile_last_ms,
    profile_ordering_ms,
    plan_pool_orders,
    schedule_swaps,
    score_swaps,
    select_swaps,
    set_option,
    simulate_swaps,
    status_string,
    validate_trace,
    workspace_bytes,
)

ORD_SIZE_DESC, ORD_LIFE_DESC, ORD_AREA_DESC, ORD_ALLOC_ASC, ORD_SEEDED, ORD_EXPLICIT, ORD_CLASS_SEEDED = range(7)
WS_LOAD_PROFILE, WS_PLAN_POOL, WS_SCORE_SWAPS, WS_VALIDATE, WS_SELECT_SWAPS, WS_DETECT_ITERATION = range(6)
K_LOAD_SCATTER, K_PLACE, K_SCORE, K_SORT, K_SELECT = range(5)
FIT_FIRST, FIT_BEST = range(2)
PS_DOA, PS_AOA, PS_WDOA, PS_SWDOA, PS_PEAK_CUT = range(5)

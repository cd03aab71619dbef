"""MI355X-native constrained-decoding masks (token mask cache build, batched
mask fill, -inf apply) behind the C ABI declared in include/xgm.h."""

from .binding import (  # noqa: F401
    XgmError,
    Vocab,
    Grammar,
    Cache,
    Matcher,
    fill_next_token_bitmask,
    fill_overflow_fixup,
    debug_fill_count_steps,
    fill_and_apply,
    debug_fill_timed,
    debug_plan_workgroups,
    debug_set_fill_pair_threshold,
    debug_set_fill_budget,
    debug_plan_slot,
    debug_lds_lookup_rate,
    MatcherBatch,
    DeviceBatch,
    overflow_total,
    apply_token_bitmask_inplace,
    bitmask_words,
    load_library,
    DTYPE_F32,
    DTYPE_BF16,
    DTYPE_F16,
)

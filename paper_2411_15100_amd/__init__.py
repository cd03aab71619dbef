"""MI355X-native constrained-decoding masks (token mask cache build, batched
mask fill, -inf apply) behind the C ABI declared in include/xgm.h."""

from .binding import (  # noqa: F401
    XgmError,
    Vocab,
    Grammar,
    schema_to_grammar,
    Cache,
    Matcher,
    fill_next_token_bitmask,
    fill_next_token_bitmask_static,
    STATIC_STAGING_BYTES,
    fill_overflow_fixup,
    fill_overflow_count_device,
    debug_fill_count_steps,
    fill_and_apply,
    debug_fill_timed,
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

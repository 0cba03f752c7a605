"""MI355X-native decode-step attention over a paged KV cache with shared-prefix
branches (the step whose latency the TAPER admission controller budgets).

The work is done by hand-written gfx950 kernels in libtaper_attn.so (C ABI in
include/taper_attn.h); this package only marshals arguments.
"""
from .binding import (  # noqa: F401
    Context,
    EXPORTED,
    LIB_PATH,
    Plan,
    Window,
    admit_step,
    append_slots,
    branch_blocks,
    predictor_eval,
    predictor_fit,
    predictor_mape,
    TaperError,
    load_library,
    taper_plan_options,
    taper_probe_result,
    TAPER_OK, TAPER_EINVAL, TAPER_EBLOCK, TAPER_EGROUP, TAPER_ELEN, TAPER_EHIP, TAPER_ENOMEM,
)

"""MI355X-native LightVLM token-reduction path: HIP kernels behind a C ABI
(include/lvlm.h) and a thin ctypes binding with the same call names."""
from .binding import (  # noqa: F401
    BF16, F32, I32, KIND_GENERATED, KIND_IMAGE, KIND_PROTECTED, KV_BUDGET, KV_THRESHOLD, MERGE_LINEAR_RANK,
    MERGE_LINEAR_RAW, MERGE_PAIRWISE, ORDER_FILL, ORDER_STABLE, RULE_TOP, RULE_WEIGHTED, Context, LvlmError,
    merge_weights, schedule,
)

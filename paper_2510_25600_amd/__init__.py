"""PureKV hot path for AMD MI355X: HIP kernels behind a C ABI (csrc/, include/purekv.h) and a thin binding."""
from .binding import (  # noqa: F401
    BK, BLOCK, KIND_CAUSAL, KIND_FULL, KIND_GENERAL, KIND_PREV, WAVES, EHIP, EINVAL, ENOMEM, EUNSUPPORTED, EWORKSPACE, EXPORTS, LIB_PATH, OK, OP_COMPACT, OP_DECODE,
    OP_IMPORTANCE, OP_PREFILL, OP_TOPK, PATTERN_DENSE, PATTERN_SPATIAL, PATTERN_ST, PATTERN_TEMPORAL, Plan,
    PureKVError, Shape, Stack, purekv_budget, purekv_calib_mfma, purekv_calib_tile_step, purekv_decode_attn, purekv_decode_step, purekv_kv_append, purekv_kv_compact, purekv_spearman,
    purekv_lowlayer_importance, purekv_st_spattn_prefill, purekv_stack_layer, purekv_stack_select_compact, purekv_strerror, purekv_topk_select, purekv_topk_select_static, purekv_topk_select_vnorm, raw,
)

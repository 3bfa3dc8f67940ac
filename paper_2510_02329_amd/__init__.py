"""MI355X-native verification step of judge-assisted speculative decoding (thin binding over libsj.so)."""
from .binding import (  # noqa: F401
    SJError, SJConfig, TENSOR_IDS, lib_path, load_library,
    sj_model_load, sj_model_free, sj_model_weight_bytes,
    sj_kv_create, sj_kv_free, sj_kv_set, sj_kv_set_layer, sj_kv_set_state, sj_kv_read, sj_kv_state,
    sj_prefill, sj_verify_step, sj_verify_head, sj_verify_head_static, sj_draft_block, sj_score_block, sj_judge_train, sj_set_mode, sj_set_topk, sj_set_temperature, sj_set_operand_planes, sj_kv_rewind, sj_set_kernel_timing, sj_get_kernel_timing, sj_kernel_class_shape, sj_time_kernel_class, sj_debug_fetch, sj_last_error, sj_version,
    SJ_MODE_TWO_STAGE, SJ_MODE_ALIGNMENT, SJ_MODE_JUDGE, SJ_MODE_TOPK,
    SJ_DBG_LOGITS, SJ_DBG_HIDDEN, SJ_DBG_JUDGE_SCORES, SJ_DBG_P_AT_DRAFT, SJ_DBG_ACCEPT_BITS,
)

"""MI355X-native hot path of WINDQuant's allocation method: a ctypes binding over
libwindq.so (hand-written HIP for gfx950) plus seeded synthetic input generators."""
from .binding import (  # noqa: F401
    CALL_FEATURES_FIT_SCORE, windq_kernel_timer, windq_kernel_timer_read, windq_features_fit_score, windq_features_fit_score_batch, CALL_APPLY_PLAN, CALL_CALIB_STATS, CALL_DEQUANT, CALL_FIT_SCORE, CALL_REFINE, CALL_SALIENT, CALL_UNIT_FEATURES, CALL_UNIT_SALIENCY, EXPORTS, LIB_PATH, MAX_BATCH, MAX_CHUNK, MAX_CLIP,
    N_ACTIONS, N_ERR, N_FEAT, WINDQ_BF16, WINDQ_EDTYPE, WINDQ_EHIP, WINDQ_EINVAL, WINDQ_ESHAPE, WINDQ_EWORKSPACE,
    WINDQ_F32, WINDQ_OK, WindqError, as_mat, lib, load, n_units, windq_apply_plan, windq_bytes_per_group,
    windq_apply_plan_batch, windq_calib_stats, windq_calib_stats_batch, windq_dequant_plan, windq_effective_bits, windq_fit_score_all_bits, windq_fit_score_all_bits_batch, windq_fit_score_rescored_units, windq_fit_score_all_bits_static, STATIC_SCRATCH_BYTES, windq_mat, windq_plan_layout, windq_refine_plan,
    windq_fallback_promote, windq_heuristic_plan, windq_n_protected, windq_salient_encode, windq_unit_saliency, windq_salient_select, windq_unit_features, windq_unit_features_batch, workspace_bytes,
    windq_salient_select_batch, windq_salient_encode_batch, windq_refine_plan_batch, windq_dequant_plan_batch, windq_unit_features_exact_units,
    CALL_DEQUANT_GEMV, windq_dequant_gemv, windq_dequant_gemv_batch,
)
from . import synth  # noqa: F401

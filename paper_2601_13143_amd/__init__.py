"""MI355X-native FastAV pruned prefill: HIP kernels behind a C ABI (include/fastav.h) + a ctypes binding."""
from .binding import (  # noqa: F401
    AUDIO, BF16, EPI_RESADD, EPI_STORE, EPI_SWIGLU, F32, FINE, GLOBAL, TEXT, VIDEO, Decoder, FastavError, Model,
    fastav_attention, fastav_attention_map, fastav_rollout_cutoff, fastav_keep_count, fastav_profile_collect, fastav_profile_enable, fastav_profile_reset, fastav_linear, fastav_rmsnorm, fastav_rope, fastav_schedule, fastav_schedule_lens, fastav_score, fastav_score_static,
    fastav_select_gather, fastav_set_option, OPT_FUSED_SCORE_SELECT, OPT_FUSED_ROPE, OPT_FUSED_SPLITK_NORM, OPT_FUSED_GATHER_OPROJ, fastav_probe_mfma, fastav_probe_read, lib, make_model, PROF_KINDS,
    SEL_DEFAULT, SEL_LOW_ATTENTIVE, SEL_TOP_ATTENTIVE, SEL_LOW_INFORMATIVE, SEL_TOP_INFORMATIVE, SEL_RANDOM,
)

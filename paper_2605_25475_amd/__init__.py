"""MI355X-native bounded-budget KV step of IndexMem: HIP kernels behind libindexmem's C ABI
(include/indexmem.h) and a thin ctypes binding with the same call names."""
from .binding import (  # noqa: F401
    Config, Params, State, Handle, IndexMemError, load_library, EXPORTS,
    im_set_max_live, im_query_status, im_append_kv, im_append_kv_hidden, im_index_score, im_topb_select,
    im_memory_update, im_compact_kv, im_gather_kept, im_decode_attn_with_readout, im_decode_attn_with_readout_static, im_decode_step, im_attend_step, im_attend_step_hidden, im_decode_step_shared, im_decode_step_shared_hidden, im_stream_read, im_profile_start, im_profile_stop,
    IM_PROFILE_MAIN, IM_PROFILE_PREP, IM_PROFILE_PREP_AND_MAIN,
    IM_OK, IM_ERR_INVALID_ARG, IM_ERR_UNSUPPORTED, IM_ERR_LAUNCH,
    IM_STATUS_APPEND_OVERFLOW, IM_STATUS_LIVE_EXCEEDED, IM_STATUS_OVER_BUDGET, IM_STATIC_SCRATCH_BYTES,
)
from .layer import Layer  # noqa: F401

"""MI355X (gfx950) multi-query-attention decode: HIP kernels behind a C ABI
(include/mqa.h) and a thin ctypes binding with the same names."""
from .binding import (  # noqa: F401
    MQA_BF16, MQA_F32, MQA_PROJ_KV, MQA_PROJ_KV_MH, MQA_PROJ_LINEAR, MQA_PROJ_O, MQA_PROJ_Q, MqaError,
    load_library, mha_decode_step, mha_decode_step_window, mqa_decode_step_window, mha_decode_workspace_bytes, mqa_append_kv, mqa_append_kv_rows, mqa_prefill_attention, mha_prefill_attention, mqa_decode_combine,
    mqa_decode_step_beams, mqa_decode_beams_workspace_bytes, mqa_beam_reorder_kv,
    mqa_decode_num_splits, mqa_decode_partials, mqa_decode_step, mqa_decode_workspace_bytes,
    mqa_decode_workspace_bytes_default, mqa_decode_plan, mqa_decode_step_noalloc,
    mqa_project_memory_kv, mqa_memory_decode_step,
    mqa_project_qkvo, mqa_project_qkvo_ex, mqa_project_append_qkv, MQA_EPI_STORE, MQA_EPI_RELU, MQA_EPI_ADD, mqa_stack_add, mqa_stack_argmax, mqa_stack_embed, mqa_stack_layernorm, mqa_stack_relu,
    mqa_stream_copy, mqa_stream_read, mqa_tuning, status_string,
)

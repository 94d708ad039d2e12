"""MI355X-native batched VLA policy inference: thin Python binding over the C-ABI HIP library.

Importing this package does not load the library; `binding.lib()` does, and raises if
libvla.so has not been built (there is no CPU fallback).
"""
from .binding import (  # noqa: F401
    VLA_F32, VLA_BF16, VlaError, VlaPolicy, Batcher, lib, library_path,
    vla_create, vla_destroy, vla_last_error, vla_query_sizes, vla_bind_buffers, vla_load_weights,
    vla_prefill, vla_decode_step, vla_policy_step, vla_select, vla_load_value_head, vla_policy_step_value,
    vla_policy_step_parallel, vla_score_tokens, vla_prefill_slots, vla_decode_slots, vla_release_slots,
    vla_get_state, vla_drain_begin, vla_update_begin, vla_update_tensors, vla_update_commit,
    VLA_ACCEPTING, VLA_DRAINING, VLA_UPDATING, VLA_E_STATE, VLA_E_DRAINING,
    vla_prof_enable, vla_prof_count, vla_prof_read, vla_probe,
)
from .serving import ContinuousWorker, InferenceWorker  # noqa: F401,E402

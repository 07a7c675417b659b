"""rollout_attn: MI355X (gfx950) decode attention over a paged KV cache for GRPO-shaped rollout batches.

The compute lives in ``librollout_attn.so`` (hand-written HIP, C ABI declared in ``include/rollout_attn.h``);
this package is the thin ctypes binding.  PyTorch is used by callers only to own device memory and streams.
"""
from .binding import (RA_ERR_DEVICE, RA_ERR_INVALID_ARG, RA_ERR_OUT_OF_RANGE, RA_ERR_UNSUPPORTED,
                      RA_ERR_WORKSPACE_TOO_SMALL, RA_FLAG_NO_PREFIX_SHARING, RA_FLAG_REUSE_SCHEDULE, RA_FLAG_VALIDATE, RA_KV_BF16,
                      RA_KV_FP8_E4M3, RA_OK, Decoder, RolloutAttnError, library_path, load_library, prefill_from_tensors, problem_from_tensors,
                      ra_prefill, ra_problem, ra_schedule_info, rollout_attn_abi_version, rollout_attn_append, rollout_attn_balance, rollout_attn_check_prefill, rollout_attn_check_problem, rollout_attn_create,
                      rollout_attn_debug_gather, rollout_attn_debug_schedule, rollout_attn_debug_stream, rollout_attn_debug_stream_tail, rollout_attn_decode, rollout_attn_decode_static, rollout_attn_destroy, rollout_attn_get_timing, rollout_attn_last_error, rollout_attn_prefill,
                      rollout_attn_set_timing, rollout_attn_set_wave_weights, rollout_attn_wave_count,
                      rollout_attn_workspace_size)

__all__ = [n for n in dir() if n.startswith(("RA_", "rollout_attn_", "ra_")) or n in
           ("Decoder", "RolloutAttnError", "library_path", "load_library", "problem_from_tensors", "prefill_from_tensors")]

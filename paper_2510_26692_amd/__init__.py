"""MI355X-native Kimi Delta Attention (KDA), forward and backward: thin binding over libkda.so.

The package holds the HIP sources (``csrc/``), the in-tree build script and a
ctypes binding whose functions carry the names of the C entry points in
``include/kda.h``.  Every step of the computation runs in the HIP kernels; the
binding only marshals pointers and sizes.  There is no CPU fallback: calling
any entry point without the built library raises.
"""
from .kda import (KdaDims, KdaError, KdaEpilogue, KdaPrologue, kda_chunk_fwd, kda_chunk_fwd_check, kda_chunk_fwd_fused,
                  kda_recurrent_steps_fused, kda_debug_set_time_split, kda_debug_set_producers,  # noqa: F401
                  kda_debug_set_wait_limit, kda_debug_chunk_fwd_plan, kda_debug_chunk_fwd_status, kda_debug_stream_probe, kda_debug_mfma_probe, kda_debug_prefill_traffic_probe, kda_chunk_fwd_min_workspace_size, kda_chunk_fwd_workspace_size, kda_last_error, kda_recurrent_step, kda_recurrent_steps_pooled,
                  kda_chunk_fwd_scalar_gate, kda_recurrent_steps_pooled_scalar_gate, kda_chunk_bwd,
                  kda_chunk_bwd_workspace_size, kda_chunk_fwd_static_scratch, kda_static_scratch_size,
                  kda_status_string, kda_version, library_path, load_library)

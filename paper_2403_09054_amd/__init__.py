"""MI355X-native Keyformer decode hot path: HIP kernels behind a C ABI.

`binding` is a thin ctypes layer over libkeyformer.so (argument marshalling
only; every step of the path runs in the HIP kernels).  There is no CPU
fallback: loading fails loudly if the library has not been built.
"""
from .binding import (  # noqa: F401
    BF16, F16, F32, LAYOUT_ORDERED, LAYOUT_SLOT, POS_NEW, POS_ORIGINAL, SCORE_PER_LAYER, SCORE_SHARED, NOISE_CONSTANT, NOISE_GAUSSIAN, NOISE_GUMBEL, NOISE_NONE, Cache, KeyformerError, NOALLOC_SCRATCH_BYTES,
    kf_beam_fork, kf_decode_launch_shape, kf_decode_select_step, kf_decode_select_step_at, kf_decode_select_step_noalloc, kf_decode_step, kf_noise_bits, kf_prefill_score, kf_select_evict, kf_select_evict_into, kf_tau, kf_version,
    kf_workspace_bytes, lib, lib_path, new_workspace,
)

"""MI355X-native verification step of Speech Speculative Decoding: thin Python binding over libssd.so.

Everything of the method runs in the HIP kernels behind the C ABI of include/ssd.h; this package only
marshals arguments (torch tensors provide device memory and the stream)."""
from .binding import (SSDError, Model, KVCache, SampleConfig, sample_config, load_library, library_path,  # noqa: F401
                      upload_weights, ssd_verify, ssd_verify_noalloc, ssd_draft_step, ssd_kv_rollback, ssd_kv_follow,
                      ssd_verify_from_probs, ssd_warp_probs, ssd_prefill, ssd_profile_begin, ssd_profile_end, ssd_trace_barriers,
                      Cycle, HOOK_TIMEOUT, HOOK_LAUNCH_NUMBER, HOOK_LAUNCH_NUMBER_DEVICE_ONLY, EXPORTED_SYMBOLS)
from .session import SSDSession  # noqa: F401,E402

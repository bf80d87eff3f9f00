"""MI355X-native hot path of AdaSD (Adaptive Speculative Decoding): per-round softmax entropy,
Jensen-Shannon distance, adaptive acceptance, correction/bonus token and threshold update.

Every step runs in the HIP library ``libadasd.so`` (see ``include/adasd.h``); this package only
marshals torch tensors into that C ABI.  There is no CPU fallback: calls raise if the library has
not been built (``python -m paper_2512_11280_amd.build`` or ``__graft_entry__.build()``).
"""
from .binding import (AdasdError, Options, State, VerifyResult, draft_entropy, draft_step, library_path,  # noqa: F401
                      load_library, profile_disable, profile_enable, profile_read, stream_read,
                      update_thresholds, verify, workspace_bytes, Workspace, Shard, verify_shard_stats,
                      verify_shard_jsd, verify_shard_decide, verify_shard_sample, verify_shard_pick,
                      verify_shard_refine, verify_shard_settle)

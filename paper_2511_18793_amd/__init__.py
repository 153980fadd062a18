"""MI355X-native NEZHA draft + verify step: a thin binding over libnezha.so.

Everything is computed by the HIP kernels behind the C ABI of include/nezha.h;
this package only marshals arguments (torch tensors give device memory and
streams).  There is no CPU fallback: calls fail loudly when the library or a
GPU is missing."""
from .api import (NezhaError, ItemSet, build_itemset, verify_tuples, draft_step,
                  draft_step_workspace, verify_workspace, unpack_keys, decode,
                  library_path, load_library, DraftBuffers, profile_enable,
                  profile_reset, profile_read, bench_random_gather, user_projection, pack_weights,
                  PackedWeights, user_projection_levels, draft_levels, DecodePlan,
                  profile_event_overhead, verify_tuples_static, VERIFY_STATIC_MAX, bench_mfma_rate,
                  bench_tile_step)

__all__ = ["NezhaError", "ItemSet", "build_itemset", "verify_tuples", "draft_step",
           "draft_step_workspace", "verify_workspace", "unpack_keys", "decode",
           "library_path", "load_library", "DraftBuffers", "profile_enable", "profile_reset",
           "profile_read", "bench_random_gather", "user_projection", "pack_weights", "PackedWeights",
           "user_projection_levels", "draft_levels", "DecodePlan", "profile_event_overhead",
           "verify_tuples_static", "VERIFY_STATIC_MAX", "bench_mfma_rate", "bench_tile_step"]

"""GPU key index of a key-value-separated LSM-tree for KV-cache storage (MI355X / gfx950).

Thin ctypes binding over the C ABI declared in include/lsm_index.h.  All work runs in the
HIP library; this package only marshals arguments and owns device memory through torch.
"""
from .binding import (LSM_BOTTOMMOST, LSM_VALIDATE, LsmDriver, LsmError, TreeRun, library_path, lsm_bloom_blocks, lsm_bloom_workspace_bytes, lsm_build_bloom, lsm_build_bloom_batch, lsm_build_bloom_hashed, lsm_build_hash_index, lsm_hash_index_buckets, lsm_hash_index_workspace_bytes, lsm_hash_keys, lsm_build_fences,
                      lsm_compact, lsm_compact_batch, lsm_compact_static, lsm_driver_flush_many, lsm_flush_buffer, lsm_compact_workspace_bytes, lsm_policy_choose, lsm_policy_cost, lsm_policy_filter_fpr, lsm_policy_levels, lsm_probe,
                      lsm_probe_length, lsm_range_bounds, lsm_range_scan, lsm_strerror)

__all__ = ["LSM_BOTTOMMOST", "LSM_VALIDATE", "LsmDriver", "LsmError", "TreeRun", "library_path", "lsm_bloom_blocks", "lsm_bloom_workspace_bytes", "lsm_build_bloom", "lsm_build_bloom_batch", "lsm_build_bloom_hashed", "lsm_build_hash_index", "lsm_hash_index_buckets", "lsm_hash_index_workspace_bytes", "lsm_hash_keys", "lsm_build_fences", "lsm_compact", "lsm_compact_batch", "lsm_compact_static", "lsm_driver_flush_many", "lsm_flush_buffer",
           "lsm_compact_workspace_bytes", "lsm_policy_choose", "lsm_policy_cost", "lsm_policy_filter_fpr", "lsm_policy_levels", "lsm_probe",
           "lsm_probe_length", "lsm_range_bounds", "lsm_range_scan", "lsm_strerror"]

"""MI355X-native minibatch sampling + feature loading (libcoop) — thin Python binding.

Argument marshalling only: every step runs in the HIP kernels of libcoop.so.  PyTorch provides
device memory and streams.  Importing this package loads the in-tree library; it raises if the
library has not been built (python -m paper_2310_12403_amd.build, or __graft_entry__.build()).
"""
from .binding import (  # noqa: F401
    COOP_F16, COOP_F32, COOP_LABOR0, COOP_NS, COOP_RW, COOP_TUNE_FUSE_LAYERS, COOP_TUNE_LISTS_PER_WAVE, COOP_TUNE_PIECE_LEN, COOP_TUNE_BLEND_CANDIDATES, COOP_TUNE_DEFER_SIZES, COOP_TUNE_UNIQUE, COOP_TUNE_ENUM_DEGREE, COOP_TUNE_NS_LONG_LIST, COOP_TUNE_SPLIT_MIN, COOP_TUNE_STAGE_CAP, COOP_VALIDATE, COOP_SYMMETRIC, Arena, Block, Cache, CoopError, Graph, coop_gather, coop_gather_mean, coop_sample_rw, coop_copy_ids, coop_bucket_by_owner, coop_bucket_by_owner_static, coop_selftest_phi_inv_gap, COOP_OWNER_RANGE, COOP_OWNER_HASH,
    coop_gather_status, coop_graph_load, coop_map_host_pointer, coop_sample, coop_strerror, coop_tune, coop_version, lib, profile_enable,
    profile_filter, profile_read_all, profile_reset)

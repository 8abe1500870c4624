"""MI355X-native reshard path of Reference-Oriented Storage weight transfer.

Thin ctypes binding over libtensorhub_reshard.so (see include/th.h).  Argument
marshalling only: every step of the path runs in the library's HIP kernels.
"""
from .binding import (  # noqa: F401
    TH_BF16, TH_F32, TH_FLAG_HOST_ONLY, TH_FLAG_PTRS_ALIGNED16, TH_FLAG_CHECKSUM, TH_FLAG_NARROW_AT_UNPACK, TH_FLAG_PROGRESS, TH_CFG_TILE_BYTES_PROGRESS, TH_CFG_SHORT_TILE_SLOTS, TH_CFG_TILE_BYTES, TH_CFG_TILE_BYTES_ANY, TH_CFG_SPECIALIZE, TH_CFG_TILE_BYTES_CHECKSUM, TH_CFG_TILE_BYTES_NARROW, TH_CFG_PLANNER_THREADS,
    ThError, Plan, library_path,
    th_plan_create, th_plan_create_from_segments, th_pack, th_pack_noalloc, th_unpack, th_pack_progress, th_unpack_progress, th_pack_checksum, th_unpack_checksum, th_reshard, th_plan_destroy,
    th_signal, th_reference_copy, th_config_set, th_config_get, th_version, th_last_error,
)

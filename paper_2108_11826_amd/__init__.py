"""MI355X-native bottom-up pose post-processing (CM + PAF maps -> skeletons).

Thin Python binding over the C-ABI library `libhp.so` (declared in include/hp.h), which
implements the post-processing operator of the paper's inference engine (Section 2.2.1,
operator 4) in HIP kernels for gfx950.  PyTorch is used for device memory and streams only.
"""
from .binding import (HPError, Skeleton, Params, Buffers, PostprocessCall, lib, lib_path, hp_resize, hp_find_peaks,
                      hp_score_limbs, hp_assemble, hp_postprocess, hp_postprocess_static, hp_preprocess, hp_smooth, hp_refine_peaks, hp_pp_decode, PPBuffers, hp_cf_decode, hp_cf_field, hp_cf_workspace_bytes, CFBuffers, hp_draw_poses, hp_draw_workspace_bytes, hp_workspace_bytes, hp_workspace_init, hp_strerror,
                      hp_version, hp_profile_begin, hp_profile_end, STATUS_PEAK_OVERFLOW, STATUS_CAND_OVERFLOW, STATUS_POSE_OVERFLOW,
                      BatcherLanes, hp_batcher_create, hp_batcher_destroy, hp_batcher_acquire, hp_batcher_commit,
                      hp_batcher_submit, hp_batcher_flush, hp_batcher_next, hp_batcher_release, hp_batch_simulate,
                      hp_batcher_drive, hp_bench_copy)

__all__ = ["HPError", "Skeleton", "Params", "Buffers", "PostprocessCall", "lib", "lib_path", "hp_resize", "hp_find_peaks",
           "hp_score_limbs", "hp_assemble", "hp_postprocess", "hp_postprocess_static", "hp_preprocess", "hp_smooth", "hp_refine_peaks", "hp_pp_decode", "PPBuffers", "hp_cf_decode", "hp_cf_field", "hp_cf_workspace_bytes", "CFBuffers", "hp_draw_poses", "hp_draw_workspace_bytes", "hp_workspace_bytes", "hp_workspace_init", "hp_strerror",
           "hp_version", "hp_profile_begin", "hp_profile_end", "STATUS_PEAK_OVERFLOW", "STATUS_CAND_OVERFLOW", "STATUS_POSE_OVERFLOW",
           "BatcherLanes", "hp_batcher_create", "hp_batcher_destroy", "hp_batcher_acquire", "hp_batcher_commit",
           "hp_batcher_submit", "hp_batcher_flush", "hp_batcher_next", "hp_batcher_release", "hp_batch_simulate",
           "hp_batcher_drive", "hp_bench_copy"]

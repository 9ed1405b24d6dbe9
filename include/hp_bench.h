/*
 * hp_bench: measurement tooling of the hp library, kept apart from the operator boundary (hp.h).
 *
 * The same shared library exports these; nothing here is part of the post-processing operator of
 * the paper's inference engine (Section 2.2.1).  They exist so that a benchmark can drive the
 * streaming front at a fixed frame rate, time every kernel of a call, and calibrate a profiler's
 * memory counters against a copy of known size.
 */
#ifndef HP_BENCH_H
#define HP_BENCH_H

#include "hp.h"

#ifdef __cplusplus
extern "C" {
#endif

/* Load generator, for benchmarks only.  Hands n_frames frames to `b` from the calling thread,
 * frame k at interarrival_ns * k after the start (0: as fast as they are taken), while a second
 * thread takes the finished batches and releases their lanes at once.  With copy_frames != 0,
 * frame k is src frame k % n_src (cm_src: device [n_src][K+1][h][w], paf_src likewise) copied
 * with hp_batcher_submit; otherwise the staging tensors are used as they are (acquire + commit,
 * nothing written).  Outputs (host arrays of n_frames, may be NULL): the time from a frame's
 * scheduled arrival to the seen completion of its batch, and its batch's size; *elapsed_ns: first
 * arrival to last completion.  The batcher must be idle at the call and is idle after it. */
int hp_batcher_drive(hp_batcher *b, int n_frames, int64_t interarrival_ns, int copy_frames,
                     const void *cm_src, const void *paf_src, int n_src,
                     int64_t *latency_ns, int32_t *batch_size, int64_t *elapsed_ns);

/* Per-kernel timing, for benchmarks only.  Between hp_profile_begin and hp_profile_end every
 * kernel the library enqueues for an operator call (from this process, any stream) is launched
 * together with a pair of HIP events that receive the kernel's own begin and end times; at most
 * `max_launches` launches are recorded, later ones run untimed.  hp_profile_end waits for the
 * recorded events (it synchronises with the streams used), adds the elapsed milliseconds and the
 * launch counts per hp_kernel_id into the two host arrays of HP_K_COUNT entries (either may be
 * NULL), and leaves profiling off.  The times are kernel durations as a profiler reports them;
 * nothing is added to the stream, but a timed launch costs the host more, so whole-call
 * throughput is measured with profiling off. */
typedef enum {
    HP_K_INIT = 0,         /* clears counters and the status word */
    HP_K_RESIZE_NMS = 1,   /* upsampling + peak detection, maps kept in registers */
    HP_K_RESIZE_W = 2,     /* upsampling, hi-res maps written (hp_resize, materialising hp_postprocess) */
    HP_K_NMS_HI = 3,       /* peak detection on materialised maps */
    HP_K_SORT_PEAKS = 4,
    HP_K_SCORE_LO = 5,     /* limb scoring, PAF recomputed from lo-res (hp_postprocess) */
    HP_K_SCORE_HI = 6,     /* limb scoring, PAF read from materialised maps (hp_score_limbs) */
    HP_K_MATCH = 7,
    HP_K_ASSEMBLE = 8,
    HP_K_LIMB_SMALL = 9,     /* peak ordering + limb scoring + matching in one launch (small capacities) */
    HP_K_PREPROCESS = 10,    /* hp_preprocess */
    HP_K_DRAW_LIST = 11,     /* hp_draw_poses: the images' primitives listed in painter's order */
    HP_K_DRAW = 12,          /* hp_draw_poses: the frames painted */
    HP_K_SMOOTH = 13,        /* hp_smooth */
    HP_K_REFINE = 14,        /* hp_refine_peaks */
    HP_K_PP_DETECT = 15,     /* hp_pp_decode: scores, boxes and suppression per (image, part) */
    HP_K_PP_PARSE = 16,      /* hp_pp_decode: the limb tree walked per image */
    HP_K_CF_PIF = 17,        /* hp_cf_decode, hp_cf_field: active intensity cells and their map values */
    HP_K_CF_PAF = 18,        /* hp_cf_decode: active associations and their map samples; the seeds sorted */
    HP_K_CF_GROW = 19,       /* hp_cf_decode: persons per image */
    HP_K_CF_FIELD = 20,      /* hp_cf_field: the fine maps written out */
    HP_K_CF_LINK = 21,       /* hp_cf_decode: what every association would propose if it won a search */
    HP_K_COUNT = 22
} hp_kernel_id;
int hp_profile_begin(int max_launches);
int hp_profile_end(float *total_ms, int32_t *launches);
const char *hp_kernel_name(int id);

/* A plain device-to-device copy of `bytes` bytes (a multiple of 16; both pointers 16-byte aligned,
 * the ranges must not overlap) by one kernel of the library on `stream`: every byte is read once and
 * written once, which makes it the reference against which HBM byte counters of a profiler are
 * scaled.  Allocates nothing. */
int hp_bench_copy(void *dst, const void *src, size_t bytes, void *stream);

#ifdef __cplusplus
}
#endif

#endif /* HP_BENCH_H */

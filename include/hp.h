/*
 * hp: bottom-up (CM + PAF) pose post-processing on one AMD MI355X (gfx950).
 *
 * C boundary of the library.  It implements the post-processing operator of the
 * paper's inference engine (Section 2.2.1, operator 4: the network's activation
 * maps go in, the human pose topology comes out) for the PAF / OpenPose family
 * (Section 2.3).  The paper runs this operator on CPU threads and names it as
 * its example of a CPU-side bottleneck (Section 2.2.2); here every step runs in
 * HIP kernels.  The paper states the operator's job but not its arithmetic; the
 * rules each call follows are written at its declaration.
 *
 * Conventions common to all calls
 *   - Tensors are dense, row-major, NCHW.  "lo" tensors are the network outputs
 *     [N][C][h][w] (fp32 or fp16); "hi" tensors are fp32 [N][C][s*h][s*w], s = 8.
 *   - Every pointer named *device* must be device memory valid on the current
 *     HIP device; hp_skeleton / hp_params / the hp_* descriptor structs are read
 *     on the host before the call returns, the arrays inside descriptors are
 *     device memory.  The caller owns every buffer.  The library allocates and
 *     frees no device memory and the operator calls never synchronise: all work
 *     is enqueued on `stream` (a hipStream_t passed as void*; NULL = the default
 *     stream).  Only the hp_batcher_* calls keep host state, a thread and HIP
 *     events of their own, and block where their comments say so.
 *   - Return value: HP_OK or a negative hp_error, decided on the host before
 *     anything is enqueued (invalid calls enqueue nothing).
 *   - Conditions only the device can see (a list longer than its capacity) are
 *     reported through `status`, one device int32 that the call overwrites:
 *     0 or an OR of hp_status_bit.  `count` arrays always receive the number of
 *     entries REQUIRED; when it exceeds the capacity the stored list is an
 *     unspecified subset of `cap` entries in canonical order and every result
 *     derived from it is invalid.
 *   - Canonical orders: peaks of one (image, part) in raster order (y, then x);
 *     candidates of one (image, limb) by (i, j) ascending; connections in
 *     acceptance order of the greedy matching; persons in creation order.
 *   - A peak is referred to by its rank in its (image, part) list.
 */
#ifndef HP_H
#define HP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { HP_F32 = 0, HP_F16 = 1 } hp_dtype;

typedef enum {
    HP_OK = 0,
    HP_ERR_INVALID_ARG = -1,   /* null pointer, non-positive size, inconsistent sizes */
    HP_ERR_DTYPE = -2,         /* unknown hp_dtype */
    HP_ERR_WORKSPACE = -3,     /* workspace smaller than hp_workspace_bytes() or misaligned */
    HP_ERR_HIP = -4,           /* a launch failed (hipGetLastError) */
    HP_ERR_UNSUPPORTED = -5,   /* a size beyond the built limits (see HP_MAX_*) */
    HP_ERR_BUSY = -6,          /* hp_batcher: every lane is collecting, running or held by the caller */
    HP_ERR_TIMEOUT = -7,       /* hp_batcher: the wait ended before the condition held */
    HP_ERR_STATE = -8          /* hp_batcher: call out of order (commit without acquire, release of a lane not held) */
} hp_error;

typedef enum {
    HP_STATUS_PEAK_OVERFLOW = 1,   /* some (image, part) has more peaks than hp_peaks.cap */
    HP_STATUS_CAND_OVERFLOW = 2,   /* some (image, limb) has more candidates than its cap */
    HP_STATUS_POSE_OVERFLOW = 4    /* some image has more persons than hp_poses.cap */
} hp_status_bit;

enum {
    HP_SCALE = 8,          /* the only upsampling factor built */
    HP_MAX_PARTS = 32,
    HP_MAX_LIMBS = 64,
    HP_MAX_CAP = 16384,    /* largest hp_peaks.cap */
    HP_MAX_CCAP = 1 << 20, /* largest candidate capacity */
    HP_MAX_SAMPLES = 64,
    HP_MAX_TAPS = 65,      /* longest tap vector of hp_smooth */
    HP_PP_MAX_CELLS = 1024, /* most grid cells (Gh * Gw) of hp_pp_decode */
    HP_CF_MAX_SEEDS = 16384 /* most seeds per image of hp_cf_decode: n_parts * lists->cap may not exceed it */
};

/* Skeleton: limb l joins part limb_a[l] to part limb_b[l] and owns PAF channels
 * (2l, 2l+1) = (x, y) components.  Host arrays of n_limbs entries. */
typedef struct {
    int32_t n_parts;
    int32_t n_limbs;
    const int32_t *limb_a;
    const int32_t *limb_b;
} hp_skeleton;

typedef struct {
    float peak_thr;         /* a peak must exceed this (strictly) */
    float paf_thr;          /* a sample is valid when its projection exceeds this */
    int32_t n_samples;      /* S >= 2 samples per candidate, end points included */
    float min_valid_ratio;  /* a candidate needs ceil(ratio * S) valid samples (fp32 product) */
    int32_t min_parts;      /* persons with fewer parts are dropped */
    int32_t scale;          /* must be HP_SCALE */
} hp_params;

/* Peaks: x, y, score are device [N][K][cap]; count is device [N][K]. */
typedef struct {
    int32_t *x;
    int32_t *y;
    float *score;
    int32_t *count;
    int32_t cap;
} hp_peaks;

/* Limb candidates or connections: i, j, score are device [N][L][cap];
 * count is device [N][L].  i / j are peak ranks of parts limb_a[l] / limb_b[l]. */
typedef struct {
    int32_t *i;
    int32_t *j;
    float *score;
    int32_t *count;
    int32_t cap;
} hp_pairs;

/* Persons: slots device [N][cap][K] (peak rank or -1), nparts and score device
 * [N][cap], count device [N]. */
typedef struct {
    int32_t *slots;
    int32_t *nparts;
    float *score;
    int32_t *count;
    int32_t cap;
} hp_poses;

/* Bytes of device workspace that hp_find_peaks, hp_score_limbs, hp_assemble and
 * hp_postprocess need for these sizes (cap = peaks per (image, part), ccap =
 * candidates per (image, limb), pcap = persons per image).  0 if a size is
 * invalid.  The workspace must be 256-byte aligned and two calls running
 * concurrently must not share it. */
size_t hp_workspace_bytes(int N, int K, int L, int h, int w, int scale, int cap, int ccap, int pcap);

/* Clears a workspace (enqueues one fill kernel on `stream`).  The workspace holds
 * the append counters of the peak and candidate lists, which every call expects
 * to find at zero and leaves at zero.  Call it once after allocating the
 * workspace, again whenever the sizes it is used with (N, K, L, cap, ccap) change,
 * and after a call that returned HP_ERR_HIP; ws_bytes must be a multiple of 4. */
int hp_workspace_init(void *workspace, size_t ws_bytes, void *stream);

/* Upsampling ("resizing", Section 2.2; imaging operations, Section 2.3).
 * dst_hi[n][c][Y][X] = bilinear sample of src_lo[n][c] at ((Y+1/2)/s - 1/2,
 * (X+1/2)/s - 1/2) with edge clamping, computed in fp32 as a horizontal pass
 * r = fma(f, v[x1], (1-f)*v[x0]) on the two source rows followed by the same
 * form vertically; fp16 sources are widened exactly first.
 * src_lo: device [N][C][h][w] of `dt`; dst_hi: device fp32 [N][C][s*h][s*w]. */
int hp_resize(const void *src_lo, hp_dtype dt, int N, int C, int h, int w, int scale,
              float *dst_hi, void *stream);

/* Peak extraction from materialised hi-res confidence maps (first half of
 * "parsing human pose topology", Section 2.2.1).  Channels 0..K-1 of the C_cm
 * = K+1 channels are searched (the last one is background).  A pixel is a peak
 * when its value exceeds thr and, among its in-bounds 8 neighbours, is greater
 * than those earlier in raster order and not less than those later.
 * cm_hi: device fp32 [N][C_cm][H][W]. */
int hp_find_peaks(const float *cm_hi, int N, int C_cm, int K, int H, int W, float thr,
                  const hp_peaks *peaks, void *workspace, size_t ws_bytes,
                  int32_t *status, void *stream);

/* Optional smoothing of materialised hi-res confidence maps before hp_find_peaks (the paper gives
 * no arithmetic for the operator; implementations of the PAF family, Section 2.3, commonly smooth
 * the upsampled maps with a small Gaussian first).  Channels 0..C-1 of every image are correlated
 * with the tap vector along x and then along y, the edge pixel repeated beyond the borders:
 *   t[y][x]   = sum_i taps[i] * src[y][clamp(x + i - r)]
 *   dst[y][x] = sum_j taps[j] * t[clamp(y + j - r)][x],      r = (n_taps - 1) / 2,
 * in fp32, each sum accumulated from 0 in ascending tap order with one fused multiply-add per
 * tap.  src_hi, dst_hi: device fp32 [N][C_mem][H][W] (channels C..C_mem-1 of dst_hi are left
 * untouched; the two tensors must not overlap); taps: DEVICE array of n_taps floats, n_taps odd,
 * 1..HP_MAX_TAPS.  Allocates nothing; enqueues one kernel per 65535 planes on `stream`. */
int hp_smooth(const float *src_hi, float *dst_hi, int N, int C, int C_mem, int H, int W,
              const float *taps, int n_taps, void *stream);

/* Optional sub-pixel refinement of the peaks hp_find_peaks stored (whole pixels, reading P4), on
 * the maps they were found on (smoothed or not).  Per axis, with a, b, c the values at x-1, x, x+1:
 *   den = (a + c) - (b + b),  off = (0.5f * (a - c)) / den   (fp32, IEEE divide),
 * taken when den < 0 and clamped to [-0.5, 0.5]; off = 0 otherwise and on the first and last
 * column; xf = (float)x + off; the same along y.  maps_hi: device fp32 [N][C_mem][H][W]; peaks: as
 * written by hp_find_peaks for channels 0..K-1 (counts above cap are clamped); xf, yf: device fp32
 * [N][K][cap], entries beyond a list's count are left untouched.  Allocates nothing; one kernel. */
int hp_refine_peaks(const float *maps_hi, int N, int C_mem, int K, int H, int W, const hp_peaks *peaks,
                    float *xf, float *yf, void *stream);

/* Limb scoring on materialised hi-res PAFs (Section 2.3, PAF family).  For
 * limb l = (a, b) and every pair (i in peaks[a], j in peaks[b]) with distinct
 * pixels: unit direction u = (B - A)/|B - A|; S samples at
 * round_half_up(A + k/(S-1) * (B - A)), k = 0..S-1; d_k = fma(paf_y, u_y, paf_x*u_x);
 * score = (d_0 + ... + d_{S-1}) / S summed in k order.  The pair is a candidate
 * when at least ceil(min_valid_ratio * S) samples have d_k > paf_thr and
 * score > 0.  paf_hi: device fp32 [N][2L][H][W]; peaks: as written by
 * hp_find_peaks (counts above cap are clamped). */
int hp_score_limbs(const float *paf_hi, int N, int H, int W,
                   const hp_skeleton *skel, const hp_params *prm,
                   const hp_peaks *peaks, const hp_pairs *cands,
                   void *workspace, size_t ws_bytes, int32_t *status, void *stream);

/* Matching and assembly (second half of "parsing human pose topology").
 * Per (image, limb): candidates are taken in the strict order (score
 * descending, i ascending, j ascending) and accepted when neither peak is
 * taken yet; `conns` receives them in acceptance order (conns->cap must be at
 * least peaks->cap).  Per image, limbs are folded in table order, connection
 * (i, j, s) of limb (a, b), pa / pb = owners of the two peaks:
 *   none owned   -> new person {a: i, b: j}, score = ps(a,i) + ps(b,j) + s
 *   one owned    -> fill the owner's empty slot, score += peak score, += s
 *                   (skipped when that slot is already filled)
 *   same owner   -> score += s
 *   two owners   -> when they share no part, the later-created is merged into
 *                   the earlier-created, score = earlier + later, += s
 *                   (skipped otherwise)
 * Persons alive at the end with >= min_parts parts are written in creation order. */
int hp_assemble(const hp_skeleton *skel, const hp_params *prm, int N,
                const hp_peaks *peaks, const hp_pairs *cands,
                const hp_pairs *conns, const hp_poses *poses,
                void *workspace, size_t ws_bytes, int32_t *status, void *stream);

/* The whole operator in one call: cm_lo / paf_lo in, peaks, candidates,
 * connections and persons out, identical to hp_resize -> hp_find_peaks ->
 * hp_score_limbs -> hp_assemble.  cm_lo: device [N][K+1][h][w], paf_lo: device
 * [N][2L][h][w], both of `dt`.  cm_hi / paf_hi are optional outputs (device
 * fp32 [N][K+1][8h][8w] and [N][2L][8h][8w]): when both are NULL the
 * upsampled maps are never written to memory; when both are given they are
 * materialised as hp_resize would.  Giving only one of them is an error.
 * In both cases peaks are found on upsampled values kept in registers and PAF
 * samples are recomputed from the lo-res tensor with the same arithmetic,
 * which gives the bits the materialised maps hold. */
int hp_postprocess(const void *cm_lo, const void *paf_lo, hp_dtype dt, int N, int h, int w,
                   const hp_skeleton *skel, const hp_params *prm,
                   float *cm_hi, float *paf_hi,
                   const hp_peaks *peaks, const hp_pairs *cands, const hp_pairs *conns,
                   const hp_poses *poses,
                   void *workspace, size_t ws_bytes, int32_t *status, void *stream);

/* hp_postprocess for callers that cannot allocate device memory and have no workspace to pass:
 * code recorded into a HIP graph, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, checks, kernels and results as hp_postprocess, but the workspace is a fixed array of
 * HP_STATIC_WS_BYTES inside the library's device image (every GPU the library runs on holds its
 * own copy until the process ends; its address on the current device is looked up at the first
 * call there).  The call allocates and frees nothing.  Sizes whose workspace
 * (hp_workspace_bytes) exceeds HP_STATIC_WS_BYTES are rejected with HP_ERR_WORKSPACE before
 * anything is enqueued.  The array keeps what the last call left in it; the call clears the list
 * counters it needs with one small kernel of its own (four or more launches on `stream`, no
 * memset).  Every call on a GPU shares that GPU's array: calls that overlap on one GPU (two
 * streams, two threads) race and give undefined results; order them on one stream or with events. */
enum { HP_STATIC_WS_BYTES = 8 << 20 };
int hp_postprocess_static(const void *cm_lo, const void *paf_lo, hp_dtype dt, int N, int h, int w,
                          const hp_skeleton *skel, const hp_params *prm,
                          float *cm_hi, float *paf_hi,
                          const hp_peaks *peaks, const hp_pairs *cands, const hp_pairs *conns,
                          const hp_poses *poses, int32_t *status, void *stream);

/* Pre-processing (Section 2.2.1, operator 2: decoded images are resized and switched to the
 * channel-first layout the network expects; Section 2.2 names "resizing and data layout
 * switching").  src: device uint8 [N][Hs][Ws][C], interleaved channels, C = 1..4; dst: device
 * fp32 or fp16 (`out_dt`) [N][C][Hd][Wd].
 *   dst[n][c][Y][X] = fma(alpha[c], u, beta[c]),
 * u = bilinear sample of channel c (channel C-1-c when reverse_channels != 0) of image n at
 * ((Y+1/2) Hs/Hd - 1/2, (X+1/2) Ws/Wd - 1/2) with edge clamping, computed in fp32 on the 0..255
 * values: along an axis, num = (2X+1) Ws - Wd, den = 2 Wd, lower node x0 = floor(num/den) and
 * weight f = (float)(num mod den) / (float)den on the upper node min(x0+1, Ws-1) (x0 = 0, f = 0
 * when num < 0); horizontal pass r = fma(f, v[x1], (1-f)*v[x0]) on the two source rows, then the
 * same form vertically.  fp16 output is the fp32 result rounded to nearest even.
 * alpha, beta: host arrays of C floats, read before the call returns.  Sizes up to 16384 per
 * side, N up to 65535.  Allocates nothing; enqueues one kernel on `stream`. */
int hp_preprocess(const uint8_t *src, int N, int Hs, int Ws, int C, hp_dtype out_dt, void *dst,
                  int Hd, int Wd, int reverse_channels, const float *alpha, const float *beta,
                  void *stream);

/* Visualisation (Section 2.2.1, operator 5: the pose topology is placed onto the original image).
 * src / dst: device uint8 [N][Hf][Wf][C], interleaved channels, C = 3 or 4 (a fourth channel is
 * copied unchanged); dst may be src (drawing in place), otherwise the two must not overlap.
 * peaks / poses: as written by hp_postprocess or hp_assemble for the same N images, peak
 * coordinates on a W x H map (only peaks->x, peaks->y, peaks->cap, poses->slots, poses->count and
 * poses->cap are read; counts above cap are clamped).  Rules, all in exact integer arithmetic:
 *   - a peak at map pixel (x, y) lands on frame pixel (floor((2x+1) Wf / (2W)), floor((2y+1) Hf / (2H)));
 *   - limb l of a person that holds both its parts covers the pixels within thickness / 2 of the
 *     segment between the two parts' frame pixels, in colour limb_rgb[l]; a part c the person holds
 *     covers the pixels within `radius` of its frame pixel, in colour part_rgb[c] (Euclidean
 *     distances between pixel coordinates, bounds included);
 *   - painter's order: persons in list order, for each its limbs in table order, then its parts in
 *     index order; a pixel gets the colour of the last primitive covering it, else the source pixel.
 * limb_rgb / part_rgb: host arrays of n_limbs x 3 and n_parts x 3 bytes, read before the call
 * returns.  Frame and map sides up to 16384, N up to 65535, thickness and radius 0..1024.
 * workspace: device memory of hp_draw_workspace_bytes(N, n_parts, n_limbs, poses->cap, Hf, Wf)
 * bytes, 256-byte aligned, no need to clear it (it receives the images' primitives in painter's
 * order and, per frame tile of 64 x 16 pixels, up to 64 of those that can touch it: about one byte
 * per frame pixel); two calls running concurrently must not share it.  poses->cap x (n_parts +
 * n_limbs) may not exceed 2^24.
 * Allocates nothing; enqueues two kernels on `stream`. */
size_t hp_draw_workspace_bytes(int N, int K, int L, int pcap, int Hf, int Wf);
int hp_draw_poses(const uint8_t *src, uint8_t *dst, int N, int Hf, int Wf, int C, int H, int W,
                  const hp_skeleton *skel, const hp_peaks *peaks, const hp_poses *poses,
                  const uint8_t *limb_rgb, const uint8_t *part_rgb, int thickness, int radius,
                  void *workspace, size_t ws_bytes, void *stream);

/* ---- Post-processing of the pose-proposal family -------------------------------------------
 * Section 2.3 lists PoseProposal as the second algorithm class the engine post-processes and gives
 * no arithmetic.  The cited method detects every part (and a whole-person "instance") as a box on
 * a coarse grid and predicts, per limb and grid cell, how likely the parent part in that cell
 * connects to the child part in each cell of a small neighbourhood.  Inputs, all device fp32:
 *   resp, conf [N][K][Gh][Gw]   (their product is the detection score);
 *   box [N][K][4][Gh][Gw]       (ox, oy: centre offset inside the cell; bw, bh: fractions of the image);
 *   edge [N][L][Nh][Nw][Gh][Gw] (connection value from the parent in cell i to the child in cell
 *                                i + (dy - (Nh-1)/2, dx - (Nw-1)/2)).
 * The skeleton's limbs are parent -> child in table order: the parent of limb 0 is the root part,
 * every other parent is the root or the child of an earlier limb, a part is a child at most once.
 * Rules (fp32, one operation per step as written):
 *   D1 score = resp * conf; a cell is a candidate when score > det_thr;
 *   D2 box: cx = ((float)gx + ox) * cell_w, cy = ((float)gy + oy) * cell_h, w = bw * img_w,
 *      h = bh * img_h, corners cx -/+ 0.5f * w, cy -/+ 0.5f * h; cell_w = img_w / (float)Gw, cell_h likewise;
 *   D3 per part, candidates in (score descending, cell index ascending) order are kept when their
 *      IoU with every box kept before is at most nms_thr; IoU = inter / ((area_a + area_b) - inter),
 *      inter = iw * ih when both overlaps are positive, else 0; IoU = 0 when the denominator is not
 *      positive.  `dets` receives the kept detections in that order (corners x0, y0, x1, y1);
 *   D4 every kept root detection starts a person, in order; limbs in table order; for a limb whose
 *      parent the person holds in cell i, the child detection, among those no earlier person took
 *      (dropped persons included) and whose cell lies in the Nh x Nw neighbourhood of i, with the
 *      largest connection value is attached when that value exceeds edge_thr (ties: the earlier);
 *   D5 person score = root score, then per attached limb in table order + connection value,
 *      + child score; persons with >= min_parts parts are written in root order: slots = rank in
 *      the part's detection list or -1.
 * `status` (device int32, overwritten): HP_STATUS_PEAK_OVERFLOW when a detection list needs more
 * than dets->cap entries, HP_STATUS_POSE_OVERFLOW for persons; counts are always the required ones.
 * Limits: Gh * Gw <= HP_PP_MAX_CELLS, Nh and Nw odd and at most 31, dets->cap <= 1024 and
 * n_parts * dets->cap <= 4096.  Allocates nothing; enqueues three kernels on `stream`. */
typedef struct {
    float det_thr;
    float nms_thr;
    float edge_thr;
    int32_t min_parts;
    float img_w;
    float img_h;
} hp_pp_params;

typedef struct {
    int32_t *cell;    /* device [N][K][cap], gy * Gw + gx */
    float *score;     /* device [N][K][cap] */
    float *box;       /* device [N][K][cap][4] */
    int32_t *count;   /* device [N][K] */
    int32_t cap;
} hp_pp_dets;

int hp_pp_decode(const float *resp, const float *conf, const float *box, const float *edge,
                 int N, int Gh, int Gw, int Nh, int Nw, const hp_skeleton *skel,
                 const hp_pp_params *prm, const hp_pp_dets *dets, const hp_poses *poses,
                 int32_t *status, void *stream);

/* ---- Decoder of the composite-field family ----------------------------------------------------
 * Section 2.3 lists PifPaf as the third algorithm class the engine post-processes and gives no
 * arithmetic.  The cited method predicts, on an Fh x Fw grid of cells `stride` pixels apart, a part
 * intensity field per part (confidence c, a vector to the part, a spread unused by decoding, a
 * scale sigma) and a part association field per limb (confidence c and, for each of the limb's two
 * parts, a vector and a spread); its decoder builds a fine confidence map per part (one Gaussian of
 * width sigma per cell, placed where the cell's vector points), seeds persons at the cells with
 * the highest map values and grows them along the association fields, an association a scoring
 * c * exp(-|x - a1| / b1) * f2(a2) for a joint at x, each step confirmed by the reverse search,
 * found joints suppressing later seeds.  Inputs, device fp32, vectors, spreads and scales in cell units:
 *   pif [N][K][5][Fh][Fw]   (c, x, y, b, sigma);
 *   paf [N][L][7][Fh][Fw]   (c, x1, y1, b1, x2, y2, b2), limb l joining parts (limb_a[l], limb_b[l]).
 * The limb table may hold cycles.  Rules (fp32, one operation per step as written; s = stride,
 * the map is H = Fh * s by W = Fw * s):
 *   C0 E(t) ~ exp(-t) in fixed arithmetic: tc = max(min(t, 80), 0); y = tc * 0x1.715476p+0f;
 *      n = rint(y); z = (y - n) * -0x1.62e430p-1f; p = 0x1.6c16c2p-10f, then p = fma(p, z, q) for
 *      q = 0x1.111112p-7f, 0x1.555556p-5f, 0x1.555556p-3f, 0.5f, 1.0f, 1.0f; E = ldexp(p, -n);
 *   C1 cell (gy, gx) of part k points to X = ((float)gx + x) * s, Y = ((float)gy + y) * s and is
 *      active when c > pif_thr, 0 <= X <= W - 1 and 0 <= Y <= H - 1; sg = max(sigma * s, 1);
 *      window w = (int)min(ceil(3 * sg), 24); nearest pixel (xr, yr) = (rint X, rint Y), ties to even;
 *   C2 map: f_k(px, py) = sum over the active cells of k, ascending cell index, with
 *      |px - xr| <= w and |py - yr| <= w, of c * E(d2 * inv); d2 = dx * dx + dy * dy,
 *      dx = (float)px - X, inv = 0.5f / (sg * sg);
 *   C3 an active cell's value is v = f_k(xr, yr); it is a seed when v > seed_thr; seeds are taken by
 *      (v descending, part ascending, cell ascending);
 *   C4 cell (gy, gx) of limb l: P1 = (((float)gx + x1) * s, ((float)gy + y1) * s), P2 likewise; active
 *      when c > paf_thr and both points lie on the map (as in C1); iB1 = 1 / max(b1 * s, 1), iB2
 *      likewise; F1 = f_a(rint P1), F2 = f_b(rint P2).  For a joint of part a at Q the cell scores
 *      (c * F2) * E(|Q - P1| * iB1) and proposes P2 for part b; for a joint of part b it scores
 *      (c * F1) * E(|Q - P2| * iB2) and proposes P1; |.| = sqrt(dx * dx + dy * dy).  A search takes
 *      the active cell with the largest score (ties: the lowest cell);
 *   C5 a person starts as the seed's joint (position (X, Y), value v, radius sg) and grows in
 *      rounds.  A round looks at every limb of which the person held exactly one part when the
 *      round began: the search from that joint must score above grow_thr; the search back from the
 *      proposed point T over the same limb in the other direction must find a cell (score above 0)
 *      whose proposal lies within rev_tol of the joint (dx * dx + dy * dy <= rev_tol * rev_tol); T
 *      must not be occupied (C7) for its part.  Of a round's proposals for one part the highest
 *      score wins (ties: the earlier limb); the part is then held at T, its value that score, its
 *      radius max(sigma * s, 1) of the part's intensity cell ((int)rint(T.y) / s, (int)rint(T.x) / s).
 *      Growing ends with the first round that adds nothing;
 *   C6 a person with at least min_parts parts is recorded: score = (sum of the held values in part
 *      order, from 0) / (float)K;
 *   C7 (x, y) is occupied for part k when a recorded person holds k at (xj, yj) with radius r and
 *      (x - xj)^2 + (y - yj)^2 <= r * r; a seed occupied for its part is skipped, and so is a seed
 *      within the radius of an earlier seed of its part whose person was grown and not recorded
 *      (the same test with that seed's position and radius);
 *   C8 decoding of an image stops when a seed passes C7 while poses->cap persons are recorded;
 *      HP_STATUS_POSE_OVERFLOW is then set.
 * `lists` receives, in ascending cell order, the active cells of every (image, part) with their
 * values and the active cells of every (image, limb) with F1 and F2; counts are the required ones,
 * HP_STATUS_PEAK_OVERFLOW / HP_STATUS_CAND_OVERFLOW tell that a list needed more than cap / acap
 * entries (everything computed from it is then incomplete).  `poses`: xyv holds (x, y, value) per
 * part, zeros for a part not held.  `status`: device int32, overwritten.
 * Limits: 1 <= lists->cap <= 1024, n_parts * lists->cap <= HP_CF_MAX_SEEDS, lists->acap >= 1,
 * n_parts * poses->cap <= 4096, Fw * stride and Fh * stride below 2^23, thresholds not negative.
 * `workspace`: hp_cf_workspace_bytes(N, n_parts, n_limbs, cap, acap) bytes of device memory, 16-byte
 * aligned, no initialisation needed (HP_ERR_WORKSPACE when too small or misaligned).  Every check
 * is made on the host before anything is enqueued.  Allocates nothing; enqueues five kernels on
 * `stream`. */
typedef struct {
    float pif_thr;
    float paf_thr;
    float seed_thr;
    float grow_thr;
    float rev_tol;
    int32_t min_parts;
    int32_t stride;
} hp_cf_params;

typedef struct {
    int32_t *pif_cell;    /* device [N][K][cap], gy * Fw + gx */
    float *pif_val;       /* device [N][K][cap] */
    int32_t *pif_count;   /* device [N][K] */
    int32_t *paf_cell;    /* device [N][L][acap] */
    float *paf_f1;        /* device [N][L][acap] */
    float *paf_f2;        /* device [N][L][acap] */
    int32_t *paf_count;   /* device [N][L] */
    int32_t cap;
    int32_t acap;
} hp_cf_lists;

typedef struct {
    float *xyv;           /* device [N][cap][K][3] */
    int32_t *nparts;      /* device [N][cap] */
    float *score;         /* device [N][cap] */
    int32_t *count;       /* device [N] */
    int32_t cap;
} hp_cf_poses;

size_t hp_cf_workspace_bytes(int N, int n_parts, int n_limbs, int cap, int acap);

int hp_cf_decode(const float *pif, const float *paf, int N, int Fh, int Fw, const hp_skeleton *skel,
                 const hp_cf_params *prm, const hp_cf_lists *lists, const hp_cf_poses *poses,
                 void *workspace, size_t ws_bytes, int32_t *status, void *stream);

/* The fine confidence maps of rule C2 as arrays: out device fp32 [N][K][Fh * stride][Fw * stride].
 * Uses pif_thr and stride of `prm`; cell, val and count as in hp_cf_lists ([N][K][cap], [N][K]);
 * `workspace`: hp_cf_workspace_bytes(N, K, 0, cap, 0); cap <= 1024, N * K <= 65535.
 * HP_STATUS_PEAK_OVERFLOW as above. */
int hp_cf_field(const float *pif, int N, int K, int Fh, int Fw, const hp_cf_params *prm, int32_t *cell,
                float *val, int32_t *count, int cap, float *out, void *workspace, size_t ws_bytes,
                int32_t *status, void *stream);

/* ---- Streaming front with a dynamic batch slot ---------------------------------------------
 * Section 2.2.1 runs the operators asynchronously, a FIFO between each pair; Section 2.2.2 puts a
 * batch slot in front of the GPU operator that collects more input tensors only while the GPU is
 * the bottleneck, so that batches grow under load and stay small (low per-image delay) otherwise.
 * Here the post-processing operator is the GPU operator, and hp_batcher is that slot in front of
 * hp_postprocess:
 *   - the caller provides n_lanes "lanes", each the buffers of one batch of up to max_batch frames
 *     (frame staging, outputs, workspace, status word) and a HIP stream of its own;
 *   - frames are handed in one at a time (hp_batcher_submit copies a frame into the open lane;
 *     hp_batcher_acquire / hp_batcher_commit let the producer write it there itself);
 *   - a frame that arrives while fewer than `depth` batches are running starts the open batch at
 *     once; while `depth` batches are running the open batch keeps collecting (up to max_batch) and
 *     starts when a running batch completes.  Batches start, complete and are handed out in
 *     arrival order, so frames leave in the order they came;
 *   - hp_batcher_next hands out the oldest finished batch: image b of the lane's outputs belongs to
 *     the b-th frame of the batch, exactly what hp_postprocess returns for that frame alone or in
 *     any other batch (images are independent).  The lane is the caller's until hp_batcher_release.
 * A batcher keeps one host thread (it waits for the running batches) and two HIP events per lane.
 * Thread model: one producer thread (acquire / commit / submit / flush) and one consumer thread
 * (next / release) may run concurrently; they may be the same thread. */
typedef struct {
    void *cm_lo;          /* device [max_batch][K+1][h][w] of the batcher's dtype: frame staging */
    void *paf_lo;         /* device [max_batch][2L][h][w] */
    hp_peaks peaks;       /* all outputs sized for max_batch images, as for hp_postprocess */
    hp_pairs cands;
    hp_pairs conns;
    hp_poses poses;
    void *workspace;      /* hp_workspace_bytes(max_batch, ...), cleared once with hp_workspace_init */
    size_t ws_bytes;
    int32_t *status;      /* device int32 */
    void *stream;         /* hipStream_t; lanes must not share streams for batches to overlap */
} hp_lane;

typedef struct {
    int32_t max_batch;    /* 1..HP_MAX_BATCH frames per batch */
    int32_t depth;        /* 1..n_lanes batches allowed to run at once */
    int32_t n_lanes;      /* 1..HP_MAX_LANES; depth + 1 or more lets a batch collect while `depth` run */
} hp_batcher_config;

enum { HP_MAX_BATCH = 1024, HP_MAX_LANES = 64 };

typedef struct {
    int32_t lane;         /* index of the lane that holds the results */
    int32_t n_frames;     /* frames in the batch */
    int32_t rc;           /* what hp_postprocess returned for the batch */
    int32_t reserved;
    uint64_t seq;         /* batches are numbered 0, 1, 2, ... in start order */
    int64_t start_ns;     /* host clock (ns since hp_batcher_create) when the batch was enqueued */
    int64_t done_ns;      /* host clock when its completion was seen */
} hp_batch_info;

typedef struct hp_batcher hp_batcher;

/* Creates a batcher on the current device for lo-res tensors [.][K+1 | 2L][h][w] of `dt`.  The
 * skeleton, parameters and lane descriptors are copied; the buffers they point to stay the
 * caller's and must outlive the batcher.  Checks everything hp_postprocess would check for a
 * batch of max_batch frames. */
int hp_batcher_create(hp_dtype dt, int h, int w, const hp_skeleton *skel, const hp_params *prm,
                      const hp_batcher_config *cfg, const hp_lane *lanes, hp_batcher **out);

/* Waits for the running batches, stops the thread, destroys the events.  Lanes still held or
 * finished are dropped; an open batch that never started is discarded. */
int hp_batcher_destroy(hp_batcher *b);

/* Place for the next frame: *cm_slot / *paf_slot point into the open lane's staging tensors
 * (device memory, one frame each).  Waits up to timeout_ms for a free lane (0: not at all, < 0:
 * without limit) and returns HP_ERR_BUSY otherwise.  One place at a time: HP_ERR_STATE when the
 * previous one is not committed yet. */
int hp_batcher_acquire(hp_batcher *b, int timeout_ms, void **cm_slot, void **paf_slot);

/* The acquired frame is handed over under the caller's `tag`.  When ready == 0 the frame is being
 * written by work already enqueued on producer_stream and the batch is ordered after that work
 * (an event, no host wait); when ready != 0 the frame is complete in memory and producer_stream is
 * ignored. */
int hp_batcher_commit(hp_batcher *b, uint64_t tag, void *producer_stream, int ready);

/* hp_batcher_acquire + a device-to-device copy of one frame (cm_frame: device [K+1][h][w],
 * paf_frame: device [2L][h][w]; one small kernel enqueued on the lane's stream) + hp_batcher_commit.
 * `ready` and producer_stream say, as for hp_batcher_commit, whether the source frame is still
 * being written. */
int hp_batcher_submit(hp_batcher *b, int timeout_ms, const void *cm_frame, const void *paf_frame,
                      uint64_t tag, void *producer_stream, int ready);

/* Closes the open batch whatever its size (end of a stream of frames). */
int hp_batcher_flush(hp_batcher *b);

/* Oldest finished batch: fills *info, and tags[0..n_frames) / commit_ns[0..n_frames) (host arrays
 * of max_batch entries, either may be NULL) with the frames' tags and hand-over times.  Waits up
 * to timeout_ms (0: not at all, < 0: without limit); HP_ERR_TIMEOUT when none finished in time,
 * HP_ERR_STATE when none can finish (nothing running or waiting) and the wait has no limit. */
int hp_batcher_next(hp_batcher *b, int timeout_ms, hp_batch_info *info, uint64_t *tags, int64_t *commit_ns);

/* Gives a lane handed out by hp_batcher_next back for new frames. */
int hp_batcher_release(hp_batcher *b, int lane);

/* The batch-slot decisions alone, in virtual time, for tests and capacity planning (no GPU call).
 * Frame k arrives at arrival_ns[k] (non-decreasing); a batch of n frames started at t is finished
 * at t + service_base_ns + n * service_per_frame_ns, completions are seen in start order, and the
 * consumer releases a lane the moment it is handed out; a frame that finds every lane taken
 * waits for the next release.  Outputs (host arrays of n_frames): the sequence number and size of
 * each frame's batch and the time its completion is seen. */
int hp_batch_simulate(int n_frames, const int64_t *arrival_ns, const hp_batcher_config *cfg,
                      int64_t service_base_ns, int64_t service_per_frame_ns,
                      int64_t *batch_seq, int32_t *batch_size, int64_t *done_ns);

/* Static string for an hp_error value. */
const char *hp_strerror(int code);

/* Library version, major * 10000 + minor * 100 + patch. */
int hp_version(void);

#ifdef __cplusplus
}
#endif

#endif /* HP_H */

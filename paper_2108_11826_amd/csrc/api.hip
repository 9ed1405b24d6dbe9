// C boundary of the library: argument checks, workspace layout and the order in which
// the kernels are enqueued.  Declarations and contracts are in include/hp.h.
#include <math.h>
#include <string.h>

#include <mutex>
#include <vector>

#include "hp_dev.h"

namespace hp {

static size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Lays the workspace out from `base` (may be null when only the size is wanted).
static bool layout(void *base, int N, int K, int L, int cap, int ccap, Workspace &ws)
{
    if (N <= 0 || K <= 0 || L <= 0 || cap <= 0 || ccap <= 0) return false;
    if (K > HP_MAX_PARTS || L > HP_MAX_LIMBS || cap > HP_MAX_CAP || ccap > HP_MAX_CCAP) return false;
    ws.cap2 = next_pow2(cap);
    ws.ccap2 = next_pow2(ccap);
    ws.wcap = (int)(((long long)K * cap) / 2 + 1);
    size_t off = 0;
    char *b = (char *)base;
    auto take = [&](size_t bytes) {
        char *p = b ? b + off : nullptr;
        off = align_up(off + bytes, 256);
        return p;
    };
    ws.peak_ctr = (int32_t *)take(sizeof(int32_t) * (size_t)N * K * kCtrStride);
    ws.peak_stage = (uint64_t *)take(sizeof(uint64_t) * (size_t)N * K * ws.cap2);
    ws.cand_ctr = (int32_t *)take(sizeof(int32_t) * (size_t)N * L * kCtrStride);
    ws.cand_stage = (uint64_t *)take(sizeof(uint64_t) * (size_t)N * L * ws.ccap2);
    ws.owner = (int32_t *)take(sizeof(int32_t) * (size_t)N * K * cap);
    ws.wslots = (int32_t *)take(sizeof(int32_t) * (size_t)N * ws.wcap * K);
    ws.wmask = (int32_t *)take(sizeof(int32_t) * (size_t)N * ws.wcap);
    ws.wscore = (float *)take(sizeof(float) * (size_t)N * ws.wcap);
    ws.bytes = off;
    return true;
}

static int check_skeleton(const hp_skeleton *sk, LimbTable &tab)
{
    if (!sk || !sk->limb_a || !sk->limb_b) return HP_ERR_INVALID_ARG;
    if (sk->n_parts <= 0 || sk->n_limbs <= 0) return HP_ERR_INVALID_ARG;
    if (sk->n_parts > HP_MAX_PARTS || sk->n_limbs > HP_MAX_LIMBS) return HP_ERR_UNSUPPORTED;
    memset(&tab, 0, sizeof(tab));
    for (int c = 0; c < HP_MAX_PARTS; ++c) tab.writer[c] = -1;
    for (int l = 0; l < sk->n_limbs; ++l) {
        int a = sk->limb_a[l], b = sk->limb_b[l];
        if (a < 0 || a >= sk->n_parts || b < 0 || b >= sk->n_parts || a == b) return HP_ERR_INVALID_ARG;
        tab.a[l] = (int8_t)a;
        tab.b[l] = (int8_t)b;
        if (tab.writer[a] < 0) tab.writer[a] = (int8_t)l;
        if (tab.writer[b] < 0) tab.writer[b] = (int8_t)l;
    }
    return HP_OK;
}

static int check_params(const hp_params *p, int &need)
{
    if (!p) return HP_ERR_INVALID_ARG;
    if (p->scale != HP_SCALE) return HP_ERR_UNSUPPORTED;
    if (p->n_samples < 2 || p->min_parts < 0) return HP_ERR_INVALID_ARG;
    if (p->n_samples > HP_MAX_SAMPLES) return HP_ERR_UNSUPPORTED;
    if (!(p->min_valid_ratio >= 0.0f && p->min_valid_ratio <= 1.0f)) return HP_ERR_INVALID_ARG;
    if (!(p->peak_thr == p->peak_thr) || !(p->paf_thr == p->paf_thr)) return HP_ERR_INVALID_ARG;
    need = (int)ceilf(p->min_valid_ratio * (float)p->n_samples);
    return HP_OK;
}

static int check_peaks(const hp_peaks *p)
{
    if (!p || !p->x || !p->y || !p->score || !p->count) return HP_ERR_INVALID_ARG;
    if (p->cap <= 0) return HP_ERR_INVALID_ARG;
    if (p->cap > HP_MAX_CAP) return HP_ERR_UNSUPPORTED;
    return HP_OK;
}

static int check_pairs(const hp_pairs *p, int max_cap)
{
    if (!p || !p->i || !p->j || !p->score || !p->count) return HP_ERR_INVALID_ARG;
    if (p->cap <= 0) return HP_ERR_INVALID_ARG;
    if (p->cap > max_cap) return HP_ERR_UNSUPPORTED;
    return HP_OK;
}

static int check_poses(const hp_poses *p)
{
    if (!p || !p->slots || !p->nparts || !p->score || !p->count) return HP_ERR_INVALID_ARG;
    if (p->cap <= 0) return HP_ERR_INVALID_ARG;
    return HP_OK;
}

static int check_dims(int N, int C, int h, int w)
{
    if (N <= 0 || C <= 0 || h <= 0 || w <= 0) return HP_ERR_INVALID_ARG;
    // hi-res plane keys (Y * W + X) and thread indices must fit 31 bits
    if ((long long)h * w * 64 >= (1LL << 31)) return HP_ERR_UNSUPPORTED;
    // row offsets in the kernels are 24-bit products (row index x row length), hi-res rows included
    if (h >= (1 << 21) || w >= (1 << 21)) return HP_ERR_UNSUPPORTED;
    if (2LL * N * C * h * w >= (1LL << 31) - 4096) return HP_ERR_UNSUPPORTED;
    return HP_OK;
}

static int check_ws(void *workspace, size_t ws_bytes, int N, int K, int L, int cap, int ccap, Workspace &ws)
{
    if (!layout(workspace, N, K, L, cap, ccap, ws)) return HP_ERR_INVALID_ARG;
    if (!workspace || ((uintptr_t)workspace & 255) != 0 || ws_bytes < ws.bytes) return HP_ERR_WORKSPACE;
    return HP_OK;
}

#define HP_TRY(expr)                      \
    do {                                  \
        int rc_ = (expr);                 \
        if (rc_ != HP_OK) return rc_;     \
    } while (0)

// Optional per-kernel timing (hp_profile_begin / hp_profile_end): every kernel launched inside a
// ProfScope gets a pair of events stamped with its begin and end times.
struct ProfRecord {
    hipEvent_t start, stop;
    int id;
};
static std::mutex g_prof_mu;
static bool g_prof_on = false;
static size_t g_prof_max = 0;
static std::vector<ProfRecord> g_prof;
static thread_local int t_prof_id = -1;   // kernel id of the enclosing HP_LAUNCH, -1 outside

bool launch_events(hipEvent_t &start, hipEvent_t &stop)
{
    if (t_prof_id < 0) return false;
    std::lock_guard<std::mutex> lk(g_prof_mu);
    if (!g_prof_on || g_prof.size() >= g_prof_max) return false;
    ProfRecord r;
    r.id = t_prof_id;
    if (hipEventCreate(&r.start) != hipSuccess) return false;
    if (hipEventCreate(&r.stop) != hipSuccess) {
        (void)hipEventDestroy(r.start);
        return false;
    }
    g_prof.push_back(r);
    start = r.start;
    stop = r.stop;
    return true;
}

struct ProfScope {
    int saved;
    explicit ProfScope(int id) : saved(t_prof_id) { t_prof_id = id; }
    ~ProfScope() { t_prof_id = saved; }
};

#define HP_LAUNCH(id, expr)                          \
    do {                                             \
        ProfScope scope_((id));                      \
        if ((expr) != hipSuccess) return HP_ERR_HIP; \
    } while (0)

// The reference copy of hp_bench_copy: 16 bytes per thread and step, every byte read and written once.
__global__ void k_copy16(uint4 *__restrict__ dst, const uint4 *__restrict__ src, size_t n)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) dst[i] = src[i];
}

}  // namespace hp

using namespace hp;

extern "C" {

size_t hp_workspace_bytes(int N, int K, int L, int h, int w, int scale, int cap, int ccap, int pcap)
{
    Workspace ws;
    if (h <= 0 || w <= 0 || scale != HP_SCALE || pcap <= 0) return 0;
    if (!layout(nullptr, N, K, L, cap, ccap, ws)) return 0;
    return ws.bytes;
}

int hp_resize(const void *src_lo, hp_dtype dt, int N, int C, int h, int w, int scale, float *dst_hi, void *stream)
{
    if (!src_lo || !dst_hi) return HP_ERR_INVALID_ARG;
    if (dt != HP_F32 && dt != HP_F16) return HP_ERR_DTYPE;
    if (scale != HP_SCALE) return HP_ERR_UNSUPPORTED;
    HP_TRY(check_dims(N, C, h, w));
    if (((uintptr_t)dst_hi & 15) != 0) return HP_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    HP_LAUNCH(HP_K_RESIZE_W, launch_resize_write(src_lo, nullptr, dt, dst_hi, nullptr, N, C, C, 0, h, w, s));
    return HP_OK;
}

int hp_find_peaks(const float *cm_hi, int N, int C_cm, int K, int H, int W, float thr,
                  const hp_peaks *peaks, void *workspace, size_t ws_bytes, int32_t *status, void *stream)
{
    if (!cm_hi || !status) return HP_ERR_INVALID_ARG;
    if (N <= 0 || H <= 0 || W <= 0 || K <= 0 || C_cm < K) return HP_ERR_INVALID_ARG;
    if (K > HP_MAX_PARTS) return HP_ERR_UNSUPPORTED;
    if ((long long)H * W >= (1LL << 31) || (long long)N * K * ((H + 7) / 8) * ((W + 3) / 4) >= (1LL << 31) - 4096)
        return HP_ERR_UNSUPPORTED;
    if (!(thr == thr)) return HP_ERR_INVALID_ARG;
    HP_TRY(check_peaks(peaks));
    Workspace ws;
    // only the peak counters and the peak staging area are used: the first two regions of the
    // common layout
    ws.cap2 = next_pow2(peaks->cap);
    const size_t ctr_bytes = align_up(sizeof(int32_t) * (size_t)N * K * kCtrStride, 256);
    const size_t need = ctr_bytes + sizeof(uint64_t) * (size_t)N * K * ws.cap2;
    if (!workspace || ((uintptr_t)workspace & 255) != 0 || ws_bytes < need) return HP_ERR_WORKSPACE;
    ws.peak_ctr = (int32_t *)workspace;
    ws.peak_stage = (uint64_t *)((char *)workspace + ctr_bytes);
    hipStream_t s = (hipStream_t)stream;
    HP_LAUNCH(HP_K_NMS_HI, launch_nms_hi(cm_hi, N, C_cm, K, H, W, thr, ws.peak_ctr, ws.peak_stage, peaks->cap, ws.cap2, status, s));
    HP_LAUNCH(HP_K_SORT_PEAKS, launch_sort_peaks(ws.peak_ctr, ws.peak_stage, peaks->cap, ws.cap2, N * K, W, *peaks, status, s));
    return HP_OK;
}

int hp_score_limbs(const float *paf_hi, int N, int H, int W, const hp_skeleton *skel, const hp_params *prm,
                   const hp_peaks *peaks, const hp_pairs *cands, void *workspace, size_t ws_bytes,
                   int32_t *status, void *stream)
{
    if (!paf_hi || !status) return HP_ERR_INVALID_ARG;
    LimbTable tab;
    int need;
    HP_TRY(check_skeleton(skel, tab));
    HP_TRY(check_params(prm, need));
    if (N <= 0 || H <= 0 || W <= 0 || (H % HP_SCALE) != 0 || (W % HP_SCALE) != 0) return HP_ERR_INVALID_ARG;
    HP_TRY(check_dims(N, 2 * skel->n_limbs, H / HP_SCALE, W / HP_SCALE));
    HP_TRY(check_peaks(peaks));
    HP_TRY(check_pairs(cands, HP_MAX_CCAP));
    Workspace ws;
    HP_TRY(check_ws(workspace, ws_bytes, N, skel->n_parts, skel->n_limbs, peaks->cap, cands->cap, ws));
    hipStream_t s = (hipStream_t)stream;
    const int K = skel->n_parts, L = skel->n_limbs;
    HP_LAUNCH(HP_K_SCORE_HI, launch_score(paf_hi, nullptr, HP_F32, N, H / HP_SCALE, W / HP_SCALE, tab, K, L, *prm, need, *peaks,
                           ws.cand_ctr, ws.cand_stage, cands->cap, ws.ccap2, status, s));
    HP_LAUNCH(HP_K_MATCH, launch_match(0, tab, N, K, L, *peaks, ws.cand_ctr, ws.cand_stage, ws.ccap2, *cands, *cands, status, s));
    return HP_OK;
}

int hp_assemble(const hp_skeleton *skel, const hp_params *prm, int N, const hp_peaks *peaks,
                const hp_pairs *cands, const hp_pairs *conns, const hp_poses *poses,
                void *workspace, size_t ws_bytes, int32_t *status, void *stream)
{
    if (!status || N <= 0) return HP_ERR_INVALID_ARG;
    LimbTable tab;
    int need;
    HP_TRY(check_skeleton(skel, tab));
    HP_TRY(check_params(prm, need));
    HP_TRY(check_peaks(peaks));
    HP_TRY(check_pairs(cands, HP_MAX_CCAP));
    HP_TRY(check_pairs(conns, HP_MAX_CAP));
    HP_TRY(check_poses(poses));
    if (conns->cap < peaks->cap) return HP_ERR_INVALID_ARG;
    Workspace ws;
    HP_TRY(check_ws(workspace, ws_bytes, N, skel->n_parts, skel->n_limbs, peaks->cap, cands->cap, ws));
    hipStream_t s = (hipStream_t)stream;
    const int K = skel->n_parts, L = skel->n_limbs;
    HP_LAUNCH(HP_K_MATCH, launch_match(2, tab, N, K, L, *peaks, ws.cand_ctr, ws.cand_stage, ws.ccap2, *cands, *conns, status, s));
    HP_LAUNCH(HP_K_ASSEMBLE, launch_assemble(tab, N, K, L, prm->min_parts, *peaks, cands, *conns, ws, *poses, status, s));
    return HP_OK;
}

int hp_postprocess(const void *cm_lo, const void *paf_lo, hp_dtype dt, int N, int h, int w,
                   const hp_skeleton *skel, const hp_params *prm, float *cm_hi, float *paf_hi,
                   const hp_peaks *peaks, const hp_pairs *cands, const hp_pairs *conns, const hp_poses *poses,
                   void *workspace, size_t ws_bytes, int32_t *status, void *stream)
{
    return hp::postprocess(cm_lo, paf_lo, dt, N, N, h, w, skel, prm, cm_hi, paf_hi, peaks, cands, conns, poses,
                           workspace, ws_bytes, status, stream, false);
}

}  // extern "C"

// Workspace of hp_postprocess_static: a fixed array in the library's device image.  Each GPU that
// loads the library holds its own copy at its own address until the process ends.  In host code
// the array's name is only a handle for hipGetSymbolAddress; the address it returns, looked up
// once per device with that device current, is what kernels and launchers are given.
static __device__ __align__(256) unsigned char scratch[HP_STATIC_WS_BYTES];

namespace hp {

constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mu;
static void *g_scratch_ptr[kMaxDevices];       // per device, null until the first call there

static int static_workspace(void **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return HP_ERR_HIP;
    if (dev < 0 || dev >= kMaxDevices) return HP_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return HP_ERR_HIP;
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return HP_OK;
}

}  // namespace hp

extern "C" int hp_postprocess_static(const void *cm_lo, const void *paf_lo, hp_dtype dt, int N, int h, int w,
                                     const hp_skeleton *skel, const hp_params *prm, float *cm_hi, float *paf_hi,
                                     const hp_peaks *peaks, const hp_pairs *cands, const hp_pairs *conns,
                                     const hp_poses *poses, int32_t *status, void *stream)
{
    // everything hp_postprocess checks, against a stand-in workspace address that is never used
    HP_TRY(hp::postprocess(cm_lo, paf_lo, dt, N, N, h, w, skel, prm, cm_hi, paf_hi, peaks, cands, conns, poses,
                           (void *)(uintptr_t)256, (size_t)-1, status, stream, true));
    Workspace ws;
    if (!layout(nullptr, N, skel->n_parts, skel->n_limbs, peaks->cap, cands->cap, ws)) return HP_ERR_INVALID_ARG;
    if (ws.bytes > (size_t)HP_STATIC_WS_BYTES) return HP_ERR_WORKSPACE;
    void *base = nullptr;
    HP_TRY(static_workspace(&base));
    layout(base, N, skel->n_parts, skel->n_limbs, peaks->cap, cands->cap, ws);
    // the array keeps the last call's contents and its layout follows the sizes, so the append
    // counters of this call may lie where an earlier call staged its lists: cleared by a kernel
    // (not a memset node: the call may be recorded into a graph)
    HP_LAUNCH(HP_K_INIT, launch_init(ws.peak_ctr, N * skel->n_parts * kCtrStride, ws.cand_ctr,
                                     N * skel->n_limbs * kCtrStride, nullptr, (hipStream_t)stream));
    return hp::postprocess(cm_lo, paf_lo, dt, N, N, h, w, skel, prm, cm_hi, paf_hi, peaks, cands, conns, poses, base,
                           (size_t)HP_STATIC_WS_BYTES, status, stream, false);
}

// The operator on the first N images of buffers laid out for N_layout >= N images: every per-image
// region of the workspace sits where a call on N_layout images puts it, so calls with different N
// can share one workspace without clearing it in between (each call leaves its counters at zero).
// With check_only set, the arguments are checked and nothing is enqueued.
int hp::postprocess(const void *cm_lo, const void *paf_lo, hp_dtype dt, int N, int N_layout, int h, int w,
                    const hp_skeleton *skel, const hp_params *prm, float *cm_hi, float *paf_hi,
                    const hp_peaks *peaks, const hp_pairs *cands, const hp_pairs *conns, const hp_poses *poses,
                    void *workspace, size_t ws_bytes, int32_t *status, void *stream, bool check_only)
{
    if (!cm_lo || !paf_lo || !status) return HP_ERR_INVALID_ARG;
    if (N <= 0 || N > N_layout) return HP_ERR_INVALID_ARG;
    if (dt != HP_F32 && dt != HP_F16) return HP_ERR_DTYPE;
    if ((cm_hi == nullptr) != (paf_hi == nullptr)) return HP_ERR_INVALID_ARG;
    LimbTable tab;
    int need;
    HP_TRY(check_skeleton(skel, tab));
    HP_TRY(check_params(prm, need));
    const int K = skel->n_parts, L = skel->n_limbs;
    HP_TRY(check_dims(N_layout, K + 1 + 2 * L, h, w));
    HP_TRY(check_peaks(peaks));
    HP_TRY(check_pairs(cands, HP_MAX_CCAP));
    HP_TRY(check_pairs(conns, HP_MAX_CAP));
    HP_TRY(check_poses(poses));
    if (conns->cap < peaks->cap) return HP_ERR_INVALID_ARG;
    if (cm_hi && ((((uintptr_t)cm_hi) | ((uintptr_t)paf_hi)) & 15) != 0) return HP_ERR_INVALID_ARG;
    Workspace ws;
    HP_TRY(check_ws(workspace, ws_bytes, N_layout, K, L, peaks->cap, cands->cap, ws));
    if (check_only) return HP_OK;
    hipStream_t s = (hipStream_t)stream;
    const int rc = enqueue_postprocess(cm_lo, paf_lo, dt, N, h, w, tab, K, L, prm, need, cm_hi, paf_hi, peaks, cands, conns,
                                       poses, ws, status, s);
    // a launch that failed half way leaves append counters that the kernels after it would have reset: clear them
    // (best effort) so that the workspace is usable again without hp_workspace_init
    if (rc == HP_ERR_HIP)
        (void)launch_init(ws.peak_ctr, N_layout * K * kCtrStride, ws.cand_ctr, N_layout * L * kCtrStride, nullptr, s);
    return rc;
}

// The launches of hp_postprocess, in order, on stream s.
int hp::enqueue_postprocess(const void *cm_lo, const void *paf_lo, hp_dtype dt, int N, int h, int w, const LimbTable &tab,
                            int K, int L, const hp_params *prm, int need, float *cm_hi, float *paf_hi,
                            const hp_peaks *peaks, const hp_pairs *cands, const hp_pairs *conns, const hp_poses *poses,
                            const Workspace &ws, int32_t *status, hipStream_t s)
{
    if (cm_hi) {
        // materialising form: every CM and PAF channel is written once, in one launch
        HP_LAUNCH(HP_K_RESIZE_W, launch_resize_write(cm_lo, paf_lo, dt, cm_hi, paf_hi, N, K + 1, K + 1, 2 * L, h, w, s));
    }
    // peaks come from upsampled values recomputed in registers where the map can reach the threshold
    HP_LAUNCH(HP_K_RESIZE_NMS, launch_resize_nms(cm_lo, dt, N, K, K + 1, h, w, prm->peak_thr, ws.peak_ctr,
                                                 ws.peak_stage, peaks->cap, ws.cap2, status, s));
    // limbs are scored on PAF values recomputed from the lo-res tensor in both forms: they are the
    // same bits as the materialised maps hold, and the lo-res tensor stays in cache where gathers
    // from the 64 times larger maps would not
    if (limb_small_applies(peaks->cap, cands->cap)) {
        // small capacities: peak ordering, scoring and matching in one launch
        HP_LAUNCH(HP_K_LIMB_SMALL, launch_limb_small(paf_lo, dt, N, h, w, tab, K, L, *prm, need, ws.peak_ctr,
                                                        ws.peak_stage, ws.cap2, *peaks, *cands, *conns, status, s));
    } else {
        HP_LAUNCH(HP_K_SORT_PEAKS, launch_sort_peaks(ws.peak_ctr, ws.peak_stage, peaks->cap, ws.cap2, N * K, HP_SCALE * w, *peaks, status, s));
        HP_LAUNCH(HP_K_SCORE_LO, launch_score(nullptr, paf_lo, dt, N, h, w, tab, K, L, *prm, need, *peaks, ws.cand_ctr,
                                              ws.cand_stage, cands->cap, ws.ccap2, nullptr, s));
        HP_LAUNCH(HP_K_MATCH, launch_match(1, tab, N, K, L, *peaks, ws.cand_ctr, ws.cand_stage, ws.ccap2, *cands, *conns, status, s));
    }
    HP_LAUNCH(HP_K_ASSEMBLE, launch_assemble(tab, N, K, L, prm->min_parts, *peaks, nullptr, *conns, ws, *poses, status, s));
    return HP_OK;
}

extern "C" {

int hp_preprocess(const uint8_t *src, int N, int Hs, int Ws, int C, hp_dtype out_dt, void *dst, int Hd, int Wd,
                  int reverse_channels, const float *alpha, const float *beta, void *stream)
{
    if (!src || !dst || !alpha || !beta) return HP_ERR_INVALID_ARG;
    if (out_dt != HP_F32 && out_dt != HP_F16) return HP_ERR_DTYPE;
    if (N <= 0 || Hs <= 0 || Ws <= 0 || Hd <= 0 || Wd <= 0 || C <= 0) return HP_ERR_INVALID_ARG;
    if (C > 4 || Hs > 16384 || Ws > 16384 || Hd > 16384 || Wd > 16384 || N > 65535) return HP_ERR_UNSUPPORTED;
    if (((uintptr_t)dst & (out_dt == HP_F32 ? 3 : 1)) != 0) return HP_ERR_INVALID_ARG;
    if (C == 4 && ((uintptr_t)src & 3) != 0) return HP_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    HP_LAUNCH(HP_K_PREPROCESS, launch_preprocess(src, N, Hs, Ws, C, out_dt, dst, Hd, Wd, reverse_channels, alpha, beta, s));
    return HP_OK;
}

int hp_pp_decode(const float *resp, const float *conf, const float *box, const float *edge, int N, int Gh, int Gw, int Nh,
                 int Nw, const hp_skeleton *skel, const hp_pp_params *prm, const hp_pp_dets *dets, const hp_poses *poses,
                 int32_t *status, void *stream)
{
    if (!resp || !conf || !box || !edge || !prm || !status) return HP_ERR_INVALID_ARG;
    LimbTable tab;
    HP_TRY(check_skeleton(skel, tab));
    const int K = skel->n_parts, L = skel->n_limbs;
    // the limbs must form a tree walked from the root in table order
    {
        bool reached[HP_MAX_PARTS] = {false};
        reached[tab.a[0]] = true;
        for (int l = 0; l < L; ++l) {
            if (!reached[tab.a[l]] || reached[tab.b[l]]) return HP_ERR_INVALID_ARG;
            reached[tab.b[l]] = true;
        }
    }
    if (N <= 0 || Gh <= 0 || Gw <= 0 || Nh <= 0 || Nw <= 0 || (Nh & 1) == 0 || (Nw & 1) == 0) return HP_ERR_INVALID_ARG;
    if (prm->min_parts < 0 || !(prm->img_w > 0.0f) || !(prm->img_h > 0.0f)) return HP_ERR_INVALID_ARG;
    if (!(prm->det_thr == prm->det_thr) || !(prm->nms_thr == prm->nms_thr) || !(prm->edge_thr == prm->edge_thr))
        return HP_ERR_INVALID_ARG;
    if (!dets || !dets->cell || !dets->score || !dets->box || !dets->count || dets->cap <= 0) return HP_ERR_INVALID_ARG;
    HP_TRY(check_poses(poses));
    if ((long long)Gh * Gw > HP_PP_MAX_CELLS || Nh > 31 || Nw > 31 || N > 65535 || dets->cap > 1024 ||
        (long long)K * dets->cap > 4096)
        return HP_ERR_UNSUPPORTED;
    hipStream_t s = (hipStream_t)stream;
    HP_LAUNCH(HP_K_INIT, launch_clear_status(status, s));
    HP_LAUNCH(HP_K_PP_DETECT, launch_pp_detect(resp, conf, box, N, Gh, Gw, K, *prm, *dets, status, s));
    HP_LAUNCH(HP_K_PP_PARSE, launch_pp_parse(edge, N, Gh, Gw, Nh, Nw, tab, K, L, *prm, *dets, *poses, status, s));
    return HP_OK;
}

static int check_cf_params(const hp_cf_params *prm, int Fh, int Fw)
{
    if (!prm) return HP_ERR_INVALID_ARG;
    if (Fh <= 0 || Fw <= 0 || prm->stride <= 0 || prm->min_parts < 0) return HP_ERR_INVALID_ARG;
    if (!(prm->pif_thr >= 0.0f) || !(prm->paf_thr >= 0.0f) || !(prm->seed_thr >= 0.0f) || !(prm->grow_thr >= 0.0f) ||
        !(prm->rev_tol >= 0.0f))
        return HP_ERR_INVALID_ARG;
    if ((long long)Fh * prm->stride >= (1 << 23) || (long long)Fw * prm->stride >= (1 << 23) ||
        (long long)Fh * Fw >= (1LL << 27))
        return HP_ERR_UNSUPPORTED;
    return HP_OK;
}

size_t hp_cf_workspace_bytes(int N, int n_parts, int n_limbs, int cap, int acap)
{
    if (N <= 0 || n_parts <= 0 || n_limbs < 0 || cap <= 0 || acap < 0) return 0;
    return cf_workspace_bytes(N, n_parts, n_limbs, cap, acap);
}

int hp_cf_decode(const float *pif, const float *paf, int N, int Fh, int Fw, const hp_skeleton *skel, const hp_cf_params *prm,
                 const hp_cf_lists *lists, const hp_cf_poses *poses, void *workspace, size_t ws_bytes, int32_t *status,
                 void *stream)
{
    if (!pif || !paf || !status || !workspace) return HP_ERR_INVALID_ARG;
    LimbTable tab;
    HP_TRY(check_skeleton(skel, tab));
    const int K = skel->n_parts, L = skel->n_limbs;
    HP_TRY(check_cf_params(prm, Fh, Fw));
    if (N <= 0) return HP_ERR_INVALID_ARG;
    if (!lists || !lists->pif_cell || !lists->pif_val || !lists->pif_count || !lists->paf_cell || !lists->paf_f1 ||
        !lists->paf_f2 || !lists->paf_count || lists->cap <= 0 || lists->acap <= 0)
        return HP_ERR_INVALID_ARG;
    if (!poses || !poses->xyv || !poses->nparts || !poses->score || !poses->count || poses->cap <= 0) return HP_ERR_INVALID_ARG;
    if (N > 65535 || lists->cap > 1024 || (long long)K * lists->cap > HP_CF_MAX_SEEDS || lists->acap > (1 << 24) ||
        (long long)K * poses->cap > 4096)
        return HP_ERR_UNSUPPORTED;
    if (ws_bytes < cf_workspace_bytes(N, K, L, lists->cap, lists->acap) || ((uintptr_t)workspace & 15)) return HP_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    HP_LAUNCH(HP_K_INIT, launch_clear_status(status, s));
    HP_LAUNCH(HP_K_CF_PIF, launch_cf_pif(pif, N, Fh, Fw, K, *prm, lists->cap, lists->pif_cell, lists->pif_val, lists->pif_count,
                                         workspace, L, lists->acap, status, s));
    HP_LAUNCH(HP_K_CF_PAF, launch_cf_paf(paf, N, Fh, Fw, tab, K, L, *prm, *lists, workspace, status, s));
    HP_LAUNCH(HP_K_CF_LINK, launch_cf_link(pif, N, Fh, Fw, tab, K, L, *prm, *lists, workspace, s));
    HP_LAUNCH(HP_K_CF_GROW, launch_cf_grow(N, Fh, Fw, tab, K, L, *prm, *lists, *poses, workspace, status, s));
    return HP_OK;
}

int hp_cf_field(const float *pif, int N, int K, int Fh, int Fw, const hp_cf_params *prm, int32_t *cell, float *val,
                int32_t *count, int cap, float *out, void *workspace, size_t ws_bytes, int32_t *status, void *stream)
{
    if (!pif || !cell || !val || !count || !out || !status || !workspace) return HP_ERR_INVALID_ARG;
    if (N <= 0 || K <= 0 || cap <= 0) return HP_ERR_INVALID_ARG;
    HP_TRY(check_cf_params(prm, Fh, Fw));
    if (K > HP_MAX_PARTS || cap > 1024 || (long long)N * K > 65535) return HP_ERR_UNSUPPORTED;
    if (ws_bytes < cf_workspace_bytes(N, K, 0, cap, 0) || ((uintptr_t)workspace & 15)) return HP_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    HP_LAUNCH(HP_K_INIT, launch_clear_status(status, s));
    HP_LAUNCH(HP_K_CF_PIF, launch_cf_pif(pif, N, Fh, Fw, K, *prm, cap, cell, val, count, workspace, 0, 0, status, s));
    HP_LAUNCH(HP_K_CF_FIELD, launch_cf_field(N, Fh, Fw, K, *prm, cap, count, out, workspace, s));
    return HP_OK;
}

int hp_refine_peaks(const float *maps_hi, int N, int C_mem, int K, int H, int W, const hp_peaks *peaks, float *xf, float *yf,
                    void *stream)
{
    if (!maps_hi || !xf || !yf) return HP_ERR_INVALID_ARG;
    if (N <= 0 || K <= 0 || C_mem < K || H <= 0 || W <= 0) return HP_ERR_INVALID_ARG;
    if (K > HP_MAX_PARTS || (long long)H * W >= (1LL << 31)) return HP_ERR_UNSUPPORTED;
    HP_TRY(check_peaks(peaks));
    hipStream_t s = (hipStream_t)stream;
    HP_LAUNCH(HP_K_REFINE, launch_refine(maps_hi, N, C_mem, K, H, W, *peaks, xf, yf, s));
    return HP_OK;
}

int hp_smooth(const float *src_hi, float *dst_hi, int N, int C, int C_mem, int H, int W, const float *taps, int n_taps,
              void *stream)
{
    if (!src_hi || !dst_hi || !taps) return HP_ERR_INVALID_ARG;
    if (N <= 0 || C <= 0 || C_mem < C || H <= 0 || W <= 0 || n_taps <= 0 || (n_taps & 1) == 0) return HP_ERR_INVALID_ARG;
    if (n_taps > HP_MAX_TAPS || C > 65535 || (long long)H * W >= (1LL << 31)) return HP_ERR_UNSUPPORTED;
    {
        // the filter reads neighbours that another workgroup may already have replaced: no smoothing in place
        const size_t bytes = sizeof(float) * (size_t)N * C_mem * H * W;
        const uintptr_t a = (uintptr_t)src_hi, b = (uintptr_t)dst_hi;
        if (a < b + bytes && b < a + bytes) return HP_ERR_INVALID_ARG;
    }
    hipStream_t s = (hipStream_t)stream;
    HP_LAUNCH(HP_K_SMOOTH, launch_smooth(src_hi, dst_hi, N, C, C_mem, H, W, taps, n_taps, s));
    return HP_OK;
}

size_t hp_draw_workspace_bytes(int N, int K, int L, int pcap, int Hf, int Wf)
{
    if (N <= 0 || K <= 0 || L <= 0 || pcap <= 0 || K > HP_MAX_PARTS || L > HP_MAX_LIMBS) return 0;
    if (Hf <= 0 || Wf <= 0 || Hf > 16384 || Wf > 16384) return 0;
    return draw_workspace_bytes(N, K, L, pcap, Hf, Wf);
}

int hp_draw_poses(const uint8_t *src, uint8_t *dst, int N, int Hf, int Wf, int C, int H, int W,
                  const hp_skeleton *skel, const hp_peaks *peaks, const hp_poses *poses, const uint8_t *limb_rgb,
                  const uint8_t *part_rgb, int thickness, int radius, void *workspace, size_t ws_bytes, void *stream)
{
    if (!src || !dst || !limb_rgb || !part_rgb) return HP_ERR_INVALID_ARG;
    LimbTable tab;
    HP_TRY(check_skeleton(skel, tab));
    if (!peaks || !peaks->x || !peaks->y || peaks->cap <= 0) return HP_ERR_INVALID_ARG;
    if (!poses || !poses->slots || !poses->count || poses->cap <= 0) return HP_ERR_INVALID_ARG;
    if (N <= 0 || Hf <= 0 || Wf <= 0 || H <= 0 || W <= 0 || thickness < 0 || radius < 0) return HP_ERR_INVALID_ARG;
    if (C != 3 && C != 4) return HP_ERR_UNSUPPORTED;
    if (Hf > 16384 || Wf > 16384 || H > 16384 || W > 16384 || N > 65535 || thickness > 1024 || radius > 1024 ||
        peaks->cap > HP_MAX_CAP)
        return HP_ERR_UNSUPPORTED;
    if (src != dst) {
        // partial overlap would let one workgroup read what another has already painted
        const size_t bytes = (size_t)N * Hf * Wf * C;
        const uintptr_t a = (uintptr_t)src, b = (uintptr_t)dst;
        if (a < b + bytes && b < a + bytes) return HP_ERR_INVALID_ARG;
    }
    const int K = skel->n_parts, L = skel->n_limbs;
    if ((long long)poses->cap * (K + L) > (1 << 24)) return HP_ERR_UNSUPPORTED;   // a primitive's rank takes 24 bits
    if (!workspace || ((uintptr_t)workspace & 255) != 0 || ws_bytes < draw_workspace_bytes(N, K, L, poses->cap, Hf, Wf))
        return HP_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    HP_LAUNCH(HP_K_DRAW_LIST, launch_draw_list(N, Hf, Wf, H, W, tab, K, L, *peaks, *poses, limb_rgb, part_rgb, thickness, radius,
                                               workspace, s));
    HP_LAUNCH(HP_K_DRAW, launch_draw_tiles(src, dst, N, Hf, Wf, C, H, W, tab, K, L, *peaks, *poses, thickness, radius,
                                           workspace, s));
    return HP_OK;
}

int hp_profile_begin(int max_launches)
{
    if (max_launches <= 0) return HP_ERR_INVALID_ARG;
    std::lock_guard<std::mutex> lk(g_prof_mu);
    for (auto &r : g_prof) {
        (void)hipEventDestroy(r.start);
        (void)hipEventDestroy(r.stop);
    }
    g_prof.clear();
    g_prof.reserve((size_t)max_launches);
    g_prof_max = (size_t)max_launches;
    g_prof_on = true;
    return HP_OK;
}

int hp_profile_end(float *total_ms, int32_t *launches)
{
    std::lock_guard<std::mutex> lk(g_prof_mu);
    g_prof_on = false;
    int rc = HP_OK;
    if (total_ms) for (int k = 0; k < HP_K_COUNT; ++k) total_ms[k] = 0.0f;
    if (launches) for (int k = 0; k < HP_K_COUNT; ++k) launches[k] = 0;
    for (auto &r : g_prof) {
        float ms = 0.0f;
        if (hipEventSynchronize(r.stop) != hipSuccess || hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess)
            rc = HP_ERR_HIP;
        else {
            if (total_ms) total_ms[r.id] += ms;
            if (launches) launches[r.id] += 1;
        }
        (void)hipEventDestroy(r.start);
        (void)hipEventDestroy(r.stop);
    }
    g_prof.clear();
    return rc;
}

const char *hp_kernel_name(int id)
{
    switch (id) {
    case HP_K_INIT: return "init";
    case HP_K_RESIZE_NMS: return "resize_nms";
    case HP_K_RESIZE_W: return "resize_write";
    case HP_K_NMS_HI: return "nms_hi";
    case HP_K_SORT_PEAKS: return "sort_peaks";
    case HP_K_SCORE_LO: return "score_lo";
    case HP_K_SCORE_HI: return "score_hi";
    case HP_K_MATCH: return "match";
    case HP_K_LIMB_SMALL: return "limb_small";
    case HP_K_ASSEMBLE: return "assemble";
    case HP_K_PREPROCESS: return "preprocess";
    case HP_K_DRAW_LIST: return "draw_list";
    case HP_K_DRAW: return "draw";
    case HP_K_SMOOTH: return "smooth";
    case HP_K_REFINE: return "refine";
    case HP_K_PP_DETECT: return "pp_detect";
    case HP_K_PP_PARSE: return "pp_parse";
    case HP_K_CF_PIF: return "cf_pif";
    case HP_K_CF_PAF: return "cf_paf";
    case HP_K_CF_LINK: return "cf_link";
    case HP_K_CF_GROW: return "cf_grow";
    case HP_K_CF_FIELD: return "cf_field";
    default: return "unknown";
    }
}

int hp_bench_copy(void *dst, const void *src, size_t bytes, void *stream)
{
    if (!dst || !src || bytes == 0) return HP_ERR_INVALID_ARG;
    if ((bytes & 15) != 0 || (((uintptr_t)dst | (uintptr_t)src) & 15) != 0) return HP_ERR_INVALID_ARG;
    const uintptr_t a = (uintptr_t)src, b = (uintptr_t)dst;
    if (a < b + bytes && b < a + bytes) return HP_ERR_INVALID_ARG;
    const size_t n = bytes / 16;
    size_t blocks = (n + kBlock - 1) / kBlock;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(hp::k_copy16, dim3((unsigned)blocks), dim3(kBlock), 0, (hipStream_t)stream, (uint4 *)dst,
                       (const uint4 *)src, n);
    return hipGetLastError() == hipSuccess ? HP_OK : HP_ERR_HIP;
}

int hp_workspace_init(void *workspace, size_t ws_bytes, void *stream)
{
    if (!workspace || ((uintptr_t)workspace & 255) != 0 || ws_bytes == 0 || (ws_bytes & 3) != 0) return HP_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    HP_LAUNCH(HP_K_INIT, launch_zero(workspace, ws_bytes, s));
    return HP_OK;
}

const char *hp_strerror(int code)
{
    switch (code) {
    case HP_OK: return "ok";
    case HP_ERR_INVALID_ARG: return "invalid argument";
    case HP_ERR_DTYPE: return "unknown dtype";
    case HP_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case HP_ERR_HIP: return "kernel launch failed";
    case HP_ERR_UNSUPPORTED: return "size beyond the built limits";
    case HP_ERR_BUSY: return "every lane is taken";
    case HP_ERR_TIMEOUT: return "timed out";
    case HP_ERR_STATE: return "call out of order";
    default: return "unknown error";
    }
}

int hp_version(void) { return 400; }

}  // extern "C"

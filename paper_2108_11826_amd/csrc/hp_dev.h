// Device-side helpers and launcher declarations shared by the kernel files.
// Internal to the library; the public boundary is include/hp.h.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "hp_bench.h"

namespace hp {

constexpr int kBlock = 256;       // threads per workgroup (4 wavefronts of 64)
constexpr int kWave = 64;
constexpr int kCtrStride = 32;    // ints between append counters: atomics on one cache line serialise,
                                  // so every list gets a line of its own
constexpr int kLdsSort = 4096;    // 64-bit keys a workgroup sorts in LDS; longer lists sort in global memory

// Limb table passed to kernels by value.
struct LimbTable {
    int8_t a[HP_MAX_LIMBS];
    int8_t b[HP_MAX_LIMBS];
    int8_t writer[HP_MAX_PARTS];   // first limb that uses the part (it publishes the part's peak list), -1 if none
};

// Where the pieces of the caller's workspace live (element offsets resolved on the host).
struct Workspace {
    int32_t *peak_ctr;      // [N*K][kCtrStride] append counters, one cache line each
    int32_t *cand_ctr;      // [N*L][kCtrStride]
    uint64_t *peak_stage;   // [N*K][cap2]   unordered (key << 32 | score bits)
    uint64_t *cand_stage;   // [N*L][ccap2]  unordered ((i << 16 | j) << 32 | score bits)
    int32_t *owner;         // [N][K][cap]   person owning each peak
    int32_t *wslots;        // [N][wcap][K]  working person table
    int32_t *wmask;         // [N][wcap]     filled-part bit mask (0 = merged away)
    float *wscore;          // [N][wcap]
    int cap2, ccap2, wcap;
    size_t bytes;
};

inline int next_pow2(int v)
{
    int p = 1;
    while (p < v) p <<= 1;
    return p;
}

template <typename T> __device__ __forceinline__ float ld(const T *p);
template <> __device__ __forceinline__ float ld<float>(const float *p) { return *p; }
template <> __device__ __forceinline__ float ld<__half>(const __half *p) { return __half2float(*p); }

// One axis of the x8 half-pixel bilinear map: output index X reads nodes i0, i1 with weight f on i1.
__device__ __forceinline__ void axis8(int X, int n, int &i0, int &i1, float &f)
{
    // 16 * source coordinate; left of node 0 it is clamped to 0, which gives node 0 and weight 0
    const int num = max(2 * X - 7, 0);
    i0 = num >> 4;
    f = (float)(num & 15) * 0.0625f;
    i1 = min(i0 + 1, n - 1);
}

// Upsampled value of one lo-res plane at hi-res pixel (Y, X): horizontal pass on the two
// source rows, then the vertical pass, each a rounded product followed by one fma.
template <typename T>
__device__ __forceinline__ float up_lo(const T *lo, int h, int w, int Y, int X)
{
    int x0, x1, y0, y1;
    float f, g;
    axis8(X, w, x0, x1, f);
    axis8(Y, h, y0, y1, g);
    const T *r0p = lo + (size_t)y0 * w, *r1p = lo + (size_t)y1 * w;
    float r0 = __fmaf_rn(f, ld(r0p + x1), (1.0f - f) * ld(r0p + x0));
    float r1 = __fmaf_rn(f, ld(r1p + x1), (1.0f - f) * ld(r1p + x0));
    return __fmaf_rn(g, r1, (1.0f - g) * r0);
}

// Monotone map of a float to an unsigned integer (larger float, larger integer), and back.
__device__ __forceinline__ uint32_t float_order(float v)
{
    const uint32_t u = __float_as_uint(v);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float float_unorder(uint32_t o)
{
    return __uint_as_float((o & 0x80000000u) ? (o & 0x7FFFFFFFu) : ~o);
}

// Ascending bitonic sort of n2 (a power of two) 64-bit keys by the whole workgroup.
// `a` may be LDS or global memory; ends with a barrier.
__device__ __forceinline__ void block_bitonic_sort(uint64_t *a, int n2)
{
    for (int k = 2; k <= n2; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int t = threadIdx.x; t < (n2 >> 1); t += blockDim.x) {
                int i = ((t & ~(j - 1)) << 1) | (t & (j - 1));
                int p = i | j;
                uint64_t x = a[i], y = a[p];
                bool up = (i & k) == 0;
                if ((x > y) == up) {
                    a[i] = y;
                    a[p] = x;
                }
            }
            __syncthreads();
        }
    }
}

// Exclusive prefix of a per-thread flag over the workgroup (thread order) and the total.
// `scratch` holds at least blockDim.x / 64 + 1 ints of LDS.  Contains two barriers.
__device__ __forceinline__ int block_flag_scan(bool flag, int *scratch, int &total)
{
    unsigned long long m = __ballot(flag);
    int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x >> 6;
    int within = __popcll(m & ((1ull << lane) - 1ull));
    if (lane == 0) scratch[wv] = __popcll(m);
    __syncthreads();
    int nw = (blockDim.x + kWave - 1) >> 6;
    int before = 0, tot = 0;
    for (int q = 0; q < nw; ++q) {
        int c = scratch[q];
        if (q < wv) before += c;
        tot += c;
    }
    __syncthreads();
    total = tot;
    return before + within;
}

// ---- kernel launches --------------------------------------------------------
// Per-kernel timing (hp_profile_begin / hp_profile_end): when it is on, launch_events hands out a
// fresh pair of events and the launch goes through the extended launch call, which stamps them
// with the kernel's own begin and end times (no extra packets on the stream, so the measured time
// is the kernel's duration as a profiler reports it).  Otherwise it returns false and the launch
// is an ordinary one.
bool launch_events(hipEvent_t &start, hipEvent_t &stop);

#define HP_KERNEL(kernel, grid, block, lds, stream, ...)                                             \
    do {                                                                                             \
        hipEvent_t ev0_ = nullptr, ev1_ = nullptr;                                                   \
        if (hp::launch_events(ev0_, ev1_))                                                           \
            hipExtLaunchKernelGGL(kernel, grid, block, lds, stream, ev0_, ev1_, 0, __VA_ARGS__);     \
        else                                                                                         \
            hipLaunchKernelGGL(kernel, grid, block, lds, stream, __VA_ARGS__);                       \
    } while (0)

// ---- launchers (each enqueues on `s` and returns the launch error) ----------

hipError_t launch_init(int32_t *a, int na, int32_t *b, int nb, int32_t *status, hipStream_t s);

// Upsampling into materialised hi-res maps: channels [0, Ca) of tensor a (Ca_mem channels per
// image in memory) and all Cb channels of tensor b (Cb may be 0) in one launch.
hipError_t launch_resize_write(const void *lo_a, const void *lo_b, hp_dtype dt, float *hi_a, float *hi_b, int N,
                               int Ca, int Ca_mem, int Cb, int h, int w, hipStream_t s);

// Peak search on the upsampled values of channels [0, K) of a lo-res tensor with C_mem channels
// per image; the upsampled maps stay in registers.
// A non-null `status` is cleared by this launch.
hipError_t launch_resize_nms(const void *lo, hp_dtype dt, int N, int K, int C_mem, int h, int w, float thr,
                             int32_t *counts, uint64_t *stage, int cap, int cap2, int32_t *status, hipStream_t s);

hipError_t launch_zero(void *p, size_t bytes, hipStream_t s);

// A non-null `status` is cleared by this launch.
hipError_t launch_nms_hi(const float *cm_hi, int N, int C_cm, int K, int H, int W, float thr,
                         int32_t *counts, uint64_t *stage, int cap, int cap2, int32_t *status, hipStream_t s);

// `ctr` are the strided append counters; the dense counts go to pk.count.
hipError_t launch_sort_peaks(int32_t *ctr, uint64_t *stage, int cap, int cap2, int planes, int W,
                             const hp_peaks &pk, int32_t *status, hipStream_t s);

// PAF sampled either from hi-res fp32 maps (paf_hi != nullptr) or recomputed from lo-res.
// A non-null `status` is cleared by this launch.
hipError_t launch_score(const float *paf_hi, const void *paf_lo, hp_dtype dt, int N, int h, int w,
                        const LimbTable &T, int K, int L, const hp_params &prm, int need,
                        const hp_peaks &pk, int32_t *ccounts, uint64_t *cstage, int ccap, int ccap2,
                        int32_t *status, hipStream_t s);

// mode 0: staged candidates -> ordered candidate lists; 1: the same, then matching;
// 2: ordered candidate lists in -> matching.  `cctr` are the strided append counters of the
// staged candidates (modes 0 and 1 copy them to cands.count).  Modes 0 and 1 set the candidate
// overflow bit of `status`; mode 2 is the first kernel of hp_assemble: it clears the status word
// and leaves the overflow bit to launch_assemble (which is given the candidate counts).
hipError_t launch_match(int mode, const LimbTable &T, int N, int K, int L, const hp_peaks &pk,
                        int32_t *cctr, uint64_t *cstage, int ccap2, const hp_pairs &cands,
                        const hp_pairs &conns, int32_t *status, hipStream_t s);

// Peak ordering + scoring + matching in one launch for small capacities (see limb_small_applies).
bool limb_small_applies(int cap, int ccap);
hipError_t launch_limb_small(const void *paf_lo, hp_dtype dt, int N, int h, int w, const LimbTable &T, int K, int L,
                             const hp_params &prm, int need, const int32_t *peak_ctr, const uint64_t *peak_stage,
                             int cap2, const hp_peaks &pk, const hp_pairs &cands, const hp_pairs &conns,
                             int32_t *status, hipStream_t s);

// Also clears the image's append counters, which leaves the workspace ready for the next call.
// With `cands` given, lists longer than cands->cap set the candidate overflow bit of `status`.
hipError_t launch_assemble(const LimbTable &T, int N, int K, int L, int min_parts, const hp_peaks &pk,
                           const hp_pairs *cands, const hp_pairs &conns, const Workspace &ws,
                           const hp_poses &poses, int32_t *status, hipStream_t s);

// Pre-processing: uint8 [N][Hs][Ws][C] -> `out_dt` [N][C][Hd][Wd]; alpha / beta are host arrays of C.
hipError_t launch_preprocess(const uint8_t *src, int N, int Hs, int Ws, int C, hp_dtype out_dt, void *dst, int Hd, int Wd,
                             int reverse_channels, const float *alpha, const float *beta, hipStream_t s);

// Visualisation: limbs (capsules) and parts (discs) of every person painted over the frames.  launch_draw_list
// writes every image's primitives, in painter's order, into the workspace; launch_draw_tiles paints them.
// limb_rgb / part_rgb are host arrays of L x 3 and K x 3 bytes.
size_t draw_workspace_bytes(int N, int K, int L, int pcap, int Hf, int Wf);
hipError_t launch_draw_list(int N, int Hf, int Wf, int H, int W, const LimbTable &T, int K, int L, const hp_peaks &pk,
                            const hp_poses &poses, const uint8_t *limb_rgb, const uint8_t *part_rgb, int thickness,
                            int radius, void *workspace, hipStream_t s);
hipError_t launch_draw_tiles(const uint8_t *src, uint8_t *dst, int N, int Hf, int Wf, int C, int H, int W,
                             const LimbTable &T, int K, int L, const hp_peaks &pk, const hp_poses &poses, int thickness,
                             int radius, const void *workspace, hipStream_t s);

// Separable smoothing of channels [0, C) of fp32 maps [N][C_mem][H][W]; taps is a device array of n_taps (odd) floats.
hipError_t launch_smooth(const float *src, float *dst, int N, int C, int C_mem, int H, int W, const float *taps,
                         int n_taps, hipStream_t s);

// Sub-pixel positions of the stored peaks of channels [0, K) on fp32 maps [N][C_mem][H][W]; xf, yf: [N][K][cap].
hipError_t launch_refine(const float *maps, int N, int C_mem, int K, int H, int W, const hp_peaks &pk, float *xf, float *yf,
                         hipStream_t s);

// The status word cleared (first launch of hp_pp_decode, hp_cf_decode and hp_cf_field).
hipError_t launch_clear_status(int32_t *status, hipStream_t s);
// Pose-proposal post-processing: detections per (image, part), persons per image.
hipError_t launch_pp_detect(const float *resp, const float *conf, const float *box, int N, int Gh, int Gw, int K,
                            const hp_pp_params &prm, const hp_pp_dets &dets, int32_t *status, hipStream_t s);
hipError_t launch_pp_parse(const float *edge, int N, int Gh, int Gw, int Nh, int Nw, const LimbTable &T, int K, int L,
                           const hp_pp_params &prm, const hp_pp_dets &dets, const hp_poses &poses, int32_t *status,
                           hipStream_t s);

// Composite-field decoding: active cells and seed values per (image, part), active associations and their map
// samples per (image, limb), persons per image; the fine map as an array.  `workspace`: cf_workspace_bytes.
size_t cf_workspace_bytes(int N, int K, int L, int cap, int acap);
hipError_t launch_cf_pif(const float *pif, int N, int Fh, int Fw, int K, const hp_cf_params &prm, int cap, int32_t *cell,
                         float *val, int32_t *count, void *workspace, int L, int acap, int32_t *status, hipStream_t s);
hipError_t launch_cf_paf(const float *paf, int N, int Fh, int Fw, const LimbTable &T, int K, int L,
                         const hp_cf_params &prm, const hp_cf_lists &lists, void *workspace, int32_t *status, hipStream_t s);
hipError_t launch_cf_link(const float *pif, int N, int Fh, int Fw, const LimbTable &T, int K, int L, const hp_cf_params &prm,
                          const hp_cf_lists &lists, void *workspace, hipStream_t s);
hipError_t launch_cf_grow(int N, int Fh, int Fw, const LimbTable &T, int K, int L, const hp_cf_params &prm,
                          const hp_cf_lists &lists, const hp_cf_poses &poses, void *workspace, int32_t *status, hipStream_t s);
hipError_t launch_cf_field(int N, int Fh, int Fw, int K, const hp_cf_params &prm, int cap, const int32_t *count, float *out,
                           void *workspace, hipStream_t s);

// hp_postprocess on the first N images of outputs and a workspace laid out for N_layout >= N images;
// check_only: validate the arguments, enqueue nothing.
int postprocess(const void *cm_lo, const void *paf_lo, hp_dtype dt, int N, int N_layout, int h, int w,
                const hp_skeleton *skel, const hp_params *prm, float *cm_hi, float *paf_hi,
                const hp_peaks *peaks, const hp_pairs *cands, const hp_pairs *conns, const hp_poses *poses,
                void *workspace, size_t ws_bytes, int32_t *status, void *stream, bool check_only);

int enqueue_postprocess(const void *cm_lo, const void *paf_lo, hp_dtype dt, int N, int h, int w, const LimbTable &tab,
                        int K, int L, const hp_params *prm, int need, float *cm_hi, float *paf_hi,
                        const hp_peaks *peaks, const hp_pairs *cands, const hp_pairs *conns, const hp_poses *poses,
                        const Workspace &ws, int32_t *status, hipStream_t s);

}  // namespace hp

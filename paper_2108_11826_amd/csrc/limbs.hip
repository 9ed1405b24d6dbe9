// Limb scoring (PAF line integral over every candidate pair) and per-limb greedy
// matching: the PAF-family part (Section 2.3) of the post-processing operator of the
// paper's inference engine (Section 2.2.1, operator 4).  Arithmetic as stated at
// hp_score_limbs / hp_assemble in hp.h.
#include "hp_dev.h"

namespace hp {

// How many PAF samples a full score of the tiled scorer fetches together (first, then `rest` at a time) for a
// survivor of its screen: two at a time, which keeps the register count low enough for eight wavefronts per SIMD.
struct ChunksSurvivor { static constexpr int first = 2, singles = 0, rest = 2; };
constexpr int kRankSort = 256; // lists up to this length are ordered by counting ranks through LDS

// Sample positions along a candidate, t_k = k / (S - 1), divided on the host (the same
// correctly rounded fp32 quotient the device would form) and passed by value.
struct SampleT {
    float t[HP_MAX_SAMPLES];
};

// Two horizontally adjacent nodes in one load (the pair is only aligned like a single node).
struct FloatPair { float a, b; };
struct HalfPair { __half a, b; };
__device__ __forceinline__ void ld_pair(const float *p, float &a, float &b)
{
    const FloatPair v = *reinterpret_cast<const FloatPair *>(p);
    a = v.a;
    b = v.b;
}
__device__ __forceinline__ void ld_pair(const __half *p, float &a, float &b)
{
    const HalfPair v = *reinterpret_cast<const HalfPair *>(p);
    a = __half2float(v.a);
    b = __half2float(v.b);
}

// Number of keys in a[0 .. n) that are smaller than `key`, for a list padded with ~0 up to a multiple of eight
// entries (16-byte aligned, in LDS).  All lanes read the same addresses; eight keys are fetched per step so that a
// list of a few dozen keys costs a few LDS round trips, not one per key.
__device__ __forceinline__ int rank_below(const uint64_t *a, int n, uint64_t key)
{
    int r = 0;
    for (int u = 0; u < n; u += 8) {
        uint64_t k[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) k[q] = a[u + q];
#pragma unroll
        for (int q = 0; q < 8; ++q) r += k[q] < key;
    }
    return r;
}

// The two PAF components of limb l at hi-res pixel (sy, sx), recomputed from the lo-res planes
// with the upsampling arithmetic (horizontal pass on the two source rows, then vertical); the
// node indices and weights are shared by the two components.  The two nodes of a row are
// neighbours in memory and come in one load; in the last column, where the upper node is
// clamped onto the lower one, the pair is read one node to the left and its second half is
// used twice.
template <typename T>
__device__ __forceinline__ void paf_from_lo(const T *__restrict__ lx, const T *__restrict__ ly, int h, int w, int sy,
                                            int sx, float &vx, float &vy)
{
    int x0, x1, y0, y1;
    float f, g;
    axis8(sx, w, x0, x1, f);
    axis8(sy, h, y0, y1, g);
    const unsigned r0 = (unsigned)__mul24(y0, w), r1 = (unsigned)__mul24(y1, w);
    const float f1 = 1.0f - f, g1 = 1.0f - g;
    float ax, bx, cx, dx, ay, by, cy, dy;
    if (w >= 2) {
        const int xs = min(x0, w - 2);
        const bool last = x0 > xs;
        ld_pair(lx + (r0 + xs), ax, bx);
        ld_pair(lx + (r1 + xs), cx, dx);
        ld_pair(ly + (r0 + xs), ay, by);
        ld_pair(ly + (r1 + xs), cy, dy);
        if (last) {
            ax = bx; cx = dx;
            ay = by; cy = dy;
        }
    } else {
        ax = bx = ld(lx + r0); cx = dx = ld(lx + r1);
        ay = by = ld(ly + r0); cy = dy = ld(ly + r1);
    }
    vx = __fmaf_rn(g, __fmaf_rn(f, dx, f1 * cx), g1 * __fmaf_rn(f, bx, f1 * ax));
    vy = __fmaf_rn(g, __fmaf_rn(f, dy, f1 * cy), g1 * __fmaf_rn(f, by, f1 * ay));
}

// Fetches CH consecutive samples of one candidate together (their loads are in flight at the
// same time), then takes validity and the running sum in sample order.
template <typename T, bool FROM_HI, int CH>
__device__ __forceinline__ void score_chunk(int k0, int S, const SampleT &st, float fdx, float fdy, float fx0,
                                            float fy0, float ux, float uy, float paf_thr, int max_bad, int H, int W,
                                            int h, int w, const float *hx, const float *hy, const T *lx, const T *ly,
                                            float &acc, int &bad)
{
    float vx[CH], vy[CH];
#pragma unroll
    for (int q = 0; q < CH; ++q) {
        const float t = st.t[min(k0 + q, S - 1)];
        // samples of a segment between two in-map pixels are in the map; the clamp only guards
        // against peak lists that were not produced by this library
        const int sx = min(max((int)floorf(__fmaf_rn(t, fdx, fx0) + 0.5f), 0), W - 1);
        const int sy = min(max((int)floorf(__fmaf_rn(t, fdy, fy0) + 0.5f), 0), H - 1);
        if (FROM_HI) {
            const unsigned o = (unsigned)__mul24(sy, W) + (unsigned)sx;
            vx[q] = hx[o];
            vy[q] = hy[o];
        } else {
            paf_from_lo(lx, ly, h, w, sy, sx, vx[q], vy[q]);
        }
    }
#pragma unroll
    for (int q = 0; q < CH; ++q) {
        if (k0 + q < S && bad <= max_bad) {
            const float d = __fmaf_rn(vy[q], uy, vx[q] * ux);
            if (!(d > paf_thr)) ++bad;
            acc = acc + d;
        }
    }
}

// Scores the candidate from pixel (x0, y0) to pixel (x1, y1).  Returns whether it is accepted
// (enough valid samples and a positive mean); CH is the chunk schedule.
template <typename T, bool FROM_HI, typename CH>
__device__ __forceinline__ bool score_pair(int x0, int y0, int x1, int y1, int S, const SampleT &st, float paf_thr,
                                           int max_bad, int H, int W, int h, int w, const float *hx, const float *hy,
                                           const T *lx, const T *ly, float &score)
{
    const int dx = x1 - x0, dy = y1 - y0;
    if (dx == 0 && dy == 0) return false;
    const float fdx = (float)dx, fdy = (float)dy, fx0 = (float)x0, fy0 = (float)y0;
    const float norm = sqrtf((float)(dx * dx + dy * dy));
    const float ux = fdx / norm, uy = fdy / norm;
    float acc = 0.0f;
    int bad = 0;
    score_chunk<T, FROM_HI, CH::first>(0, S, st, fdx, fdy, fx0, fy0, ux, uy, paf_thr, max_bad, H, W, h, w, hx, hy, lx, ly,
                                       acc, bad);
    int k0 = CH::first;
#pragma unroll
    for (int q = 0; q < CH::singles; ++q) {
        if (k0 < S && bad <= max_bad)
            score_chunk<T, FROM_HI, 1>(k0, S, st, fdx, fdy, fx0, fy0, ux, uy, paf_thr, max_bad, H, W, h, w, hx, hy, lx, ly,
                                       acc, bad);
        ++k0;
    }
    for (; k0 < S && bad <= max_bad; k0 += CH::rest)
        score_chunk<T, FROM_HI, CH::rest>(k0, S, st, fdx, fdy, fx0, fy0, ux, uy, paf_thr, max_bad, H, W, h, w, hx, hy,
                                            lx, ly, acc, bad);
    if (bad > max_bad) return false;
    score = acc / (float)S;
    return score > 0.0f;
}

// General scorer.  grid = (tiles, N*L); a workgroup owns a tile of peak pairs of its (image,
// limb): 64 peaks j of part b, one per lane, times a range of peaks i of part a, whose
// coordinates sit in LDS; the workgroup's four wavefronts take every fourth i each, so short
// lists still occupy all of them.  A score is never reduced across lanes, so the summation
// order is the sample order.
//
// Most pairs join unrelated peaks and are rejected because too few samples are valid.  Which
// samples are looked at first does not change that verdict, and a pair that is rejected emits
// nothing, so rejection is decided as cheaply as possible, in two steps.
//
// Screen (every pair).  Sample 0 lies on peak A and sample S-1 on peak B (t = 0 and t = 1 round
// to the end points exactly), so the PAF there is a property of the peak, fetched once per peak
// and limb instead of once per pair; one more sample (k = 1) is fetched.  The unit vector is
// approximated, u' = (dx, dy) * rsq(dx^2 + dy^2): rsq is good to one unit in the last place and
// the exact u carries two roundings, so u' and u differ by less than 3e-7 relative and the
// projection d' = fma(py, u'y, px * u'x) differs from the exact d by less than
// 5e-7 * (|px| + |py|).  A sample is counted as invalid only if d' + 4e-6 * (|px| + |py|) is
// still below the threshold, i.e. only when the exact test is certain to fail; a pair is
// dropped when more than S - need samples are invalid for certain.  The screen therefore drops
// nothing that the full score would keep.
//
// Survivors (a few percent) are queued in LDS and handled by whole wavefronts of survivors,
// with the exact unit vector: first the validity of all samples, one at a time in the order
// 0, S-1, 1, 2, ... with each lane leaving at its (S - need + 1)-th invalid sample; what is
// left after that is scored in full, in sample order.  Accepted pairs are appended unordered,
// tagged with (i << 16 | j), and ordered by the matching kernel.
constexpr float kScreenMargin = 4e-6f;
constexpr int kTileI = 256;           // peaks of part a staged in LDS at a time
constexpr int kTileJ = kWave;         // peaks of part b of a tile: one per lane
constexpr int kScreenUnroll = 2;      // pairs a thread screens between two looks at the queue (more costs occupancy)
constexpr int kQueue = 512;           // survivors ring of one wavefront; >= 64 * (kScreenUnroll + 1), power of two

template <typename T, bool FROM_HI>
__device__ __forceinline__ void paf_at(const float *hx, const float *hy, const T *lx, const T *ly, int h, int w, int W,
                                       int y, int x, float &vx, float &vy)
{
    if (FROM_HI) {
        const unsigned o = (unsigned)__mul24(y, W) + (unsigned)x;
        vx = hx[o];
        vy = hy[o];
    } else {
        paf_from_lo(lx, ly, h, w, y, x, vx, vy);
    }
}

// Scoring of the candidate from peak A to peak B when the PAF at the two peaks is already known (samples 0 and S-1
// lie on the peaks, since t = 0 and t = 1 round to them exactly, so they are fetched once per peak and limb, not
// once per pair), in two stages.  Stage 1: the two end samples and samples 1 and 2 (fetched together); nearly all
// unrelated pairs have more than max_bad invalid samples by then and leave.  Stage 2: the remaining samples eight
// at a time, leaving as soon as the pair is beyond max_bad.  Rejection does not depend on the order in which samples
// are looked at, and a pair that is still alive at the end has had every sample looked at, so its sum is formed on
// the way in sample order: d_0, the interior samples ascending, d_{S-1} last.
struct PairGeom {
    float fdx, fdy, fx0, fy0, ux, uy;
};

// false for a pair on one pixel (never a candidate)
__device__ __forceinline__ bool pair_geometry(int xA, int yA, int xB, int yB, PairGeom &g)
{
    const int dx = xB - xA, dy = yB - yA;
    if (dx == 0 && dy == 0) return false;
    g.fdx = (float)dx;
    g.fdy = (float)dy;
    g.fx0 = (float)xA;
    g.fy0 = (float)yA;
    const float norm = sqrtf((float)(dx * dx + dy * dy));
    g.ux = g.fdx / norm;
    g.uy = g.fdy / norm;
    return true;
}

template <typename T, bool FROM_HI>
__device__ __forceinline__ float pair_project(const PairGeom &g, float t, int H, int W, int h, int w, const float *hx,
                                              const float *hy, const T *lx, const T *ly)
{
    // the clamp only guards against peak lists that were not produced by this library
    const int sx = min(max((int)floorf(__fmaf_rn(t, g.fdx, g.fx0) + 0.5f), 0), W - 1);
    const int sy = min(max((int)floorf(__fmaf_rn(t, g.fdy, g.fy0) + 0.5f), 0), H - 1);
    float vx, vy;
    paf_at<T, FROM_HI>(hx, hy, lx, ly, h, w, W, sy, sx, vx, vy);
    return __fmaf_rn(vy, g.uy, vx * g.ux);
}

// Returns whether the pair is still alive; bad = invalid samples so far, acc = d_0 + d_1 + d_2.
template <typename T, bool FROM_HI>
__device__ __forceinline__ bool pair_stage1(const PairGeom &g, float pAx, float pAy, float pBx, float pBy, int S,
                                            const SampleT &st, float paf_thr, int max_bad, int H, int W, int h, int w,
                                            const float *hx, const float *hy, const T *lx, const T *ly, int &bad,
                                            float &acc)
{
    const float d_first = __fmaf_rn(pAy, g.uy, pAx * g.ux), d_last = __fmaf_rn(pBy, g.uy, pBx * g.ux);
    bad = (d_first > paf_thr ? 0 : 1) + (d_last > paf_thr ? 0 : 1);
    acc = 0.0f + d_first;
    if (bad <= max_bad && S > 2) {
        const float d1 = pair_project<T, FROM_HI>(g, st.t[1], H, W, h, w, hx, hy, lx, ly);
        const float d2 = S > 3 ? pair_project<T, FROM_HI>(g, st.t[2], H, W, h, w, hx, hy, lx, ly) : 0.0f;
        bad += d1 > paf_thr ? 0 : 1;
        acc = acc + d1;
        if (S > 3) {
            bad += d2 > paf_thr ? 0 : 1;
            acc = acc + d2;
        }
    }
    return bad <= max_bad;
}

// Returns whether the pair is accepted, with its score.
template <typename T, bool FROM_HI>
__device__ __forceinline__ bool pair_stage2(const PairGeom &g, float pBx, float pBy, int bad, float acc, int S,
                                            const SampleT &st, float paf_thr, int max_bad, int H, int W, int h, int w,
                                            const float *hx, const float *hy, const T *lx, const T *ly, float &score)
{
    for (int k0 = 3; k0 < S - 1 && bad <= max_bad; k0 += 8) {
        float d[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) d[q] = pair_project<T, FROM_HI>(g, st.t[min(k0 + q, S - 2)], H, W, h, w, hx, hy, lx, ly);
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            if (k0 + q < S - 1) {
                bad += d[q] > paf_thr ? 0 : 1;
                acc = acc + d[q];
            }
        }
    }
    if (bad > max_bad) return false;
    acc = acc + __fmaf_rn(pBy, g.uy, pBx * g.ux);
    score = acc / (float)S;
    return score > 0.0f;
}

// Both stages in one go.
template <typename T, bool FROM_HI>
__device__ __forceinline__ bool score_pair_ends(int xA, int yA, int xB, int yB, float pAx, float pAy, float pBx, float pBy,
                                                int S, const SampleT &st, float paf_thr, int max_bad, int H, int W, int h,
                                                int w, const float *hx, const float *hy, const T *lx, const T *ly,
                                                float &score)
{
    PairGeom g;
    int bad;
    float acc;
    if (!pair_geometry(xA, yA, xB, yB, g)) return false;
    if (!pair_stage1<T, FROM_HI>(g, pAx, pAy, pBx, pBy, S, st, paf_thr, max_bad, H, W, h, w, hx, hy, lx, ly, bad, acc)) return false;
    return pair_stage2<T, FROM_HI>(g, pBx, pBy, bad, acc, S, st, paf_thr, max_bad, H, W, h, w, hx, hy, lx, ly, score);
}

// WIDE: the lo-res map has at least two columns (the launcher's choice).  Stating it to the compiler removes the
// one-column form of the bilinear gather, whose merged results would otherwise make every gather wait for the
// one before it.
template <typename T, bool FROM_HI, bool WIDE>
__global__ __launch_bounds__(kBlock) void k_score(const float *__restrict__ paf_hi, const T *__restrict__ paf_lo,
                                                  int h, int w, LimbTable tab, SampleT st, int K, int L, int S,
                                                  float paf_thr, int need, int tiles_j, int sub_tiles,
                                                  const int32_t *__restrict__ pcounts,
                                                  const int32_t *__restrict__ px, const int32_t *__restrict__ py,
                                                  int cap, int32_t *ccounts, uint64_t *cstage, int ccap, int ccap2,
                                                  int32_t *status)
{
    __shared__ int4 sA[kTileI];                 // x, y, PAF x bits, PAF y bits at the peak
    __shared__ int2 sB[kTileJ];                 // x, y
    __shared__ uint32_t queues[kBlock / kWave][kQueue];   // i << 16 | j_local of pairs that passed the screen
    if (WIDE) __builtin_assume(w >= 2);
    const int tid = threadIdx.x;
    const int nl = blockIdx.y;
    // first kernel of hp_score_limbs: it clears the status word (the ordering kernel that follows sets bits)
    if (status && (blockIdx.x | blockIdx.y) == 0 && tid == 0) *status = 0;
    const int n = nl / L, l = nl - n * L;
    const int a = tab.a[l], b = tab.b[l];
    const int nA = max(min(pcounts[n * K + a], cap), 0), nB = max(min(pcounts[n * K + b], cap), 0);
    const int ti = blockIdx.x / tiles_j, tj = blockIdx.x - ti * tiles_j;
    const int j0 = tj * kTileJ;
    const int i_begin = ti * sub_tiles * kTileI;
    if (j0 >= nB || i_begin >= nA) return;      // uniform over the workgroup
    const int i_end = min(i_begin + sub_tiles * kTileI, nA);

    const int32_t *xa = px + (size_t)(n * K + a) * cap, *ya = py + (size_t)(n * K + a) * cap;
    const int32_t *xb = px + (size_t)(n * K + b) * cap, *yb = py + (size_t)(n * K + b) * cap;
    const int H = 8 * h, W = 8 * w;
    const float *hx = FROM_HI ? paf_hi + ((size_t)n * 2 * L + 2 * l) * (size_t)H * W : nullptr;
    const float *hy = FROM_HI ? hx + (size_t)H * W : nullptr;
    const T *lx = FROM_HI ? nullptr : paf_lo + ((size_t)n * 2 * L + 2 * l) * (size_t)h * w;
    const T *ly = FROM_HI ? nullptr : lx + (size_t)h * w;
    const int max_bad = S - need;

    // this thread's peak of part b and the PAF there (sample S-1 of every pair it ends)
    const int lane = tid & (kWave - 1), wv = tid >> 6;
    const int j = j0 + lane;
    const bool jv = j < nB;
    int xB = 0, yB = 0;
    float pBx = 0.0f, pBy = 0.0f;
    if (jv) {
        xB = xb[j];
        yB = yb[j];
        paf_at<T, FROM_HI>(hx, hy, lx, ly, h, w, W, min(max(yB, 0), H - 1), min(max(xB, 0), W - 1), pBx, pBy);
    }
    const float mB = kScreenMargin * (fabsf(pBx) + fabsf(pBy));
    if (wv == 0) sB[lane] = make_int2(xB, yB);
    // every wavefront queues its own survivors: the ring and its two counters are private to
    // it, so that no wavefront ever waits for another one's survivors
    uint32_t *queue = queues[wv];
    const unsigned long long lanes_below = (1ull << lane) - 1ull;
    int q_head = 0, q_tail = 0;                 // uniform over the wavefront

    // a queued pair: exact validity of its samples with early exit, then the full score
    auto score_queued = [&](uint32_t e) {
        const int i = (int)(e >> 16), jl = (int)(e & 0xffffu);
        const int4 A = sA[i & (kTileI - 1)];
        const int2 B = sB[jl];
        const int dx = B.x - A.x, dy = B.y - A.y;              // not both zero: the screen dropped those
        const float fdx = (float)dx, fdy = (float)dy, fx0 = (float)A.x, fy0 = (float)A.y;
        const float norm = sqrtf((float)(dx * dx + dy * dy));
        const float ux = fdx / norm, uy = fdy / norm;
        float ex, ey;
        paf_at<T, FROM_HI>(hx, hy, lx, ly, h, w, W, min(max(B.y, 0), H - 1), min(max(B.x, 0), W - 1), ex, ey);
        int bad = (__fmaf_rn(__uint_as_float((uint32_t)A.w), uy, __uint_as_float((uint32_t)A.z) * ux) > paf_thr ? 0 : 1) +
                  (S >= 2 && !(__fmaf_rn(ey, uy, ex * ux) > paf_thr) ? 1 : 0);
        for (int k = 1; k < S - 1 && bad <= max_bad; ++k) {
            const float t = st.t[k];
            const int sx = min(max((int)floorf(__fmaf_rn(t, fdx, fx0) + 0.5f), 0), W - 1);
            const int sy = min(max((int)floorf(__fmaf_rn(t, fdy, fy0) + 0.5f), 0), H - 1);
            float vx, vy;
            paf_at<T, FROM_HI>(hx, hy, lx, ly, h, w, W, sy, sx, vx, vy);
            if (!(__fmaf_rn(vy, uy, vx * ux) > paf_thr)) ++bad;
        }
        if (bad > max_bad) return;
        float score;
        if (score_pair<T, FROM_HI, ChunksSurvivor>(A.x, A.y, B.x, B.y, S, st, paf_thr, max_bad, H, W, h, w, hx, hy, lx, ly,
                                                   score)) {
            const int slot = atomicAdd(&ccounts[nl * kCtrStride], 1);
            if (slot < ccap)
                cstage[(size_t)nl * ccap2 + slot] =
                    ((uint64_t)(((uint32_t)i << 16) | (uint32_t)(j0 + jl)) << 32) | (uint64_t)__float_as_uint(score);
        }
    };

    for (int i0 = i_begin; i0 < i_end; i0 += kTileI) {
        const int ni = min(kTileI, i_end - i0);
        __syncthreads();                        // the previous tile's queue is empty, sA is free
        if (tid < ni) {
            const int x = xa[i0 + tid], y = ya[i0 + tid];
            float vx, vy;
            paf_at<T, FROM_HI>(hx, hy, lx, ly, h, w, W, min(max(y, 0), H - 1), min(max(x, 0), W - 1), vx, vy);
            sA[tid] = make_int4(x, y, (int)__float_as_uint(vx), (int)__float_as_uint(vy));
        }
        __syncthreads();
        constexpr int kWaves = kBlock / kWave;
        for (int ii = wv; ii < ni; ii += kWaves * kScreenUnroll) {
            // the screen of kScreenUnroll pairs, written without branches so that the loads of
            // all of them are in flight together (idle slots repeat the tile's last peak and
            // are masked at the end; all sample coordinates are clamped into the map)
            bool pass[kScreenUnroll];
            float sux[kScreenUnroll], suy[kScreenUnroll], svx[kScreenUnroll], svy[kScreenUnroll];
            int sbad[kScreenUnroll];
#pragma unroll
            for (int u = 0; u < kScreenUnroll; ++u) {
                const int4 A = sA[min(ii + kWaves * u, ni - 1)];
                const int dx = xB - A.x, dy = yB - A.y;
                pass[u] = ii + kWaves * u < ni && jv && (dx != 0 || dy != 0);
                const float fdx = (float)dx, fdy = (float)dy;
                const float rn = __builtin_amdgcn_rsqf((float)max(dx * dx + dy * dy, 1));
                const float ux = fdx * rn, uy = fdy * rn;
                const float pAx = __uint_as_float((uint32_t)A.z), pAy = __uint_as_float((uint32_t)A.w);
                // certainly invalid: the projection plus its error bound is below the threshold
                const float d0 = __fmaf_rn(pAy, uy, pAx * ux) + kScreenMargin * (fabsf(pAx) + fabsf(pAy));
                const float dl = __fmaf_rn(pBy, uy, pBx * ux) + mB;
                sbad[u] = (d0 < paf_thr ? 1 : 0) + (dl < paf_thr ? 1 : 0);
                sux[u] = ux;
                suy[u] = uy;
                const float t = st.t[1];
                const int sx = min(max((int)floorf(__fmaf_rn(t, fdx, (float)A.x) + 0.5f), 0), W - 1);
                const int sy = min(max((int)floorf(__fmaf_rn(t, fdy, (float)A.y) + 0.5f), 0), H - 1);
                paf_at<T, FROM_HI>(hx, hy, lx, ly, h, w, W, sy, sx, svx[u], svy[u]);
            }
#pragma unroll
            for (int u = 0; u < kScreenUnroll; ++u) {
                const float d1 = __fmaf_rn(svy[u], suy[u], svx[u] * sux[u]) + kScreenMargin * (fabsf(svx[u]) + fabsf(svy[u]));
                if (S >= 3 && d1 < paf_thr) ++sbad[u];
                pass[u] = pass[u] && sbad[u] <= max_bad;
            }
            // survivors join the wavefront's queue
#pragma unroll
            for (int u = 0; u < kScreenUnroll; ++u) {
                const unsigned long long m = __ballot(pass[u]);
                if (pass[u])
                    queue[(q_tail + __popcll(m & lanes_below)) & (kQueue - 1)] = ((uint32_t)(i0 + ii + kWaves * u) << 16) | (uint32_t)lane;
                q_tail += __popcll(m);
            }
            // the queue is written and read by the lanes of one wavefront only
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            while (q_tail - q_head >= kWave) {
                score_queued(queue[(q_head + lane) & (kQueue - 1)]);
                q_head += kWave;
            }
        }
        // the tile's coordinates go away: finish its survivors
        if (lane < q_tail - q_head) score_queued(queue[(q_head + lane) & (kQueue - 1)]);
        q_head = q_tail;
    }
}

// Scorer for short lists (capacity up to kFlatPeaks peaks per part): one workgroup per (image, limb), one lane per
// pair, all pairs of the limb spread over the workgroup's threads.  With a few hundred pairs per limb a launch is
// a chain of dependent memory round trips, and the tiled scorer above spends a dozen of them (screen sample, then a
// survivor's samples one or two at a time).  Here the chain is: the peak lists; the PAF at every peak; the pairs
// through score_pair_ends (two fetch rounds for nearly all of them).  Same candidates as the definition's
// sample-by-sample loop, bit for bit.
constexpr int kFlatPeaks = 256;
constexpr int kFlatBlock = 1024;

template <typename T, bool FROM_HI>
__global__ __launch_bounds__(kFlatBlock) void k_score_flat(const float *__restrict__ paf_hi, const T *__restrict__ paf_lo,
                                                           int h, int w, LimbTable tab, SampleT st, int K, int L, int S,
                                                           float paf_thr, int need, const int32_t *__restrict__ pcounts,
                                                           const int32_t *__restrict__ px, const int32_t *__restrict__ py,
                                                           int cap, int32_t *ccounts, uint64_t *cstage, int ccap, int ccap2,
                                                           int32_t *status)
{
    __shared__ int lxy[4][kFlatPeaks];          // xA, yA, xB, yB
    __shared__ float lpaf[4][kFlatPeaks];       // PAF x, y at the peaks of A; x, y at the peaks of B
    const int tid = threadIdx.x;
    const int nl = blockIdx.x;
    if (status && nl == 0 && tid == 0) *status = 0;
    const int n = nl / L, l = nl - n * L;
    const int a = tab.a[l], b = tab.b[l];
    const int nA = max(min(pcounts[n * K + a], cap), 0), nB = max(min(pcounts[n * K + b], cap), 0);
    const int H = 8 * h, W = 8 * w;
    const float *hx = FROM_HI ? paf_hi + ((size_t)n * 2 * L + 2 * l) * (size_t)H * W : nullptr;
    const float *hy = FROM_HI ? hx + (size_t)H * W : nullptr;
    const T *lx = FROM_HI ? nullptr : paf_lo + ((size_t)n * 2 * L + 2 * l) * (size_t)h * w;
    const T *ly = FROM_HI ? nullptr : lx + (size_t)h * w;
    {
        // threads [0, 256) bring in list A, [256, 512) list B, each peak with the PAF at its pixel
        const int half = tid >> 8, t = tid & (kFlatPeaks - 1);
        if (half < 2 && t < (half == 0 ? nA : nB)) {
            const size_t o = (size_t)(n * K + (half == 0 ? a : b)) * cap + t;
            const int x = px[o], y = py[o];
            lxy[2 * half][t] = x;
            lxy[2 * half + 1][t] = y;
            float vx, vy;
            paf_at<T, FROM_HI>(hx, hy, lx, ly, h, w, W, min(max(y, 0), H - 1), min(max(x, 0), W - 1), vx, vy);
            lpaf[2 * half][t] = vx;
            lpaf[2 * half + 1][t] = vy;
        }
    }
    __syncthreads();
    const int P = nA * nB, max_bad = S - need;
    for (int p = tid; p < P; p += kFlatBlock) {
        const int i = p / nB, j = p - i * nB;
        float score;
        if (score_pair_ends<T, FROM_HI>(lxy[0][i], lxy[1][i], lxy[2][j], lxy[3][j], lpaf[0][i], lpaf[1][i], lpaf[2][j],
                                        lpaf[3][j], S, st, paf_thr, max_bad, H, W, h, w, hx, hy, lx, ly, score)) {
            const int slot = atomicAdd(&ccounts[nl * kCtrStride], 1);
            if (slot < ccap)
                cstage[(size_t)nl * ccap2 + slot] =
                    ((uint64_t)(((uint32_t)i << 16) | (uint32_t)j) << 32) | (uint64_t)__float_as_uint(score);
        }
    }
}

hipError_t launch_score(const float *paf_hi, const void *paf_lo, hp_dtype dt, int N, int h, int w,
                        const LimbTable &T, int K, int L, const hp_params &prm, int need,
                        const hp_peaks &pk, int32_t *ccounts, uint64_t *cstage, int ccap, int ccap2,
                        int32_t *status, hipStream_t s)
{
    SampleT st;
    for (int k = 0; k < HP_MAX_SAMPLES; ++k) st.t[k] = (float)k / (float)(prm.n_samples - 1);
    if (pk.cap <= kFlatPeaks) {
        auto go = [&](auto kernel, const float *hi, auto lo) {
            HP_KERNEL(kernel, dim3(N * L), dim3(kFlatBlock), 0, s, hi, lo, h, w, T, st, K, L, prm.n_samples, prm.paf_thr,
                      need, pk.count, pk.x, pk.y, pk.cap, ccounts, cstage, ccap, ccap2, status);
        };
        const float *none = nullptr;
        if (paf_hi)
            go(k_score_flat<float, true>, paf_hi, none);
        else if (dt == HP_F16)
            go(k_score_flat<__half, false>, none, (const __half *)paf_lo);
        else
            go(k_score_flat<float, false>, none, (const float *)paf_lo);
        return hipGetLastError();
    }
    // tiles of kTileJ peaks of part b x (sub_tiles * kTileI) peaks of part a cover cap x cap pairs;
    // workgroups whose tile lies beyond the actual counts leave at once, so their number is kept
    // moderate by letting a workgroup walk over several tiles of part a
    const int tiles_j = (pk.cap + kTileJ - 1) / kTileJ;
    const int tiles_i = (pk.cap + kTileI - 1) / kTileI;
    int sub_tiles = (tiles_i * tiles_j + 1023) / 1024;
    if (sub_tiles < 1) sub_tiles = 1;
    const int tiles = ((tiles_i + sub_tiles - 1) / sub_tiles) * tiles_j;
    dim3 grid(tiles, N * L), block(kBlock);
    auto go = [&](auto kernel, const float *hi, auto lo) {
        HP_KERNEL(kernel, grid, block, 0, s, hi, lo, h, w, T, st, K, L, prm.n_samples, prm.paf_thr, need, tiles_j,
                  sub_tiles, pk.count, pk.x, pk.y, pk.cap, ccounts, cstage, ccap, ccap2, status);
    };
    const float *none = nullptr;
    const bool wide = w >= 2;
    if (paf_hi)
        go(k_score<float, true, false>, paf_hi, none);
    else if (dt == HP_F16)
        wide ? go(k_score<__half, false, true>, none, (const __half *)paf_lo)
             : go(k_score<__half, false, false>, none, (const __half *)paf_lo);
    else
        wide ? go(k_score<float, false, true>, none, (const float *)paf_lo)
             : go(k_score<float, false, false>, none, (const float *)paf_lo);
    return hipGetLastError();
}

// Greedy one-to-one matching by one wavefront.  keys[0 .. c) hold the candidates in matching
// order as (~score bits) << 32 | (i << 16 | j).  They are taken 64 at a time, one per lane: a
// candidate whose peak i or j is already used (bit maps usedA / usedB in LDS, cleared by the
// caller) is out; of the rest the lowest lane is accepted, every candidate of the chunk that
// shares a peak with it dies, and so on: one step per connection instead of one per candidate.
// The order of acceptance is the order of the sequential scan.  Called by all 64 lanes of one
// wavefront; returns the number of connections written to mi / mj / ms (at most `limit`).
__device__ __forceinline__ int wave_greedy_match(const uint64_t *keys, int c, int nA, int nB, int limit, uint32_t *usedA,
                                                 uint32_t *usedB, int32_t *mi, int32_t *mj, float *ms)
{
    const int lane = threadIdx.x & (kWave - 1);
    const bool more_chunks = c > kWave;          // a single chunk needs no memory of used peaks
    int m = 0;
    for (int base = 0; base < c && m < limit; base += kWave) {
        const bool have = base + lane < c;
        const uint64_t e = have ? keys[base + lane] : ~0ull;
        const uint32_t i = (uint32_t)e >> 16, j = (uint32_t)e & 0xffffu;
        // indices beyond the peak lists are only possible for candidate lists this library did not write
        bool ok = have && i < (uint32_t)nA && j < (uint32_t)nB;
        if (ok && more_chunks) ok = !((usedA[i >> 5] >> (i & 31)) & 1u) && !((usedB[j >> 5] >> (j & 31)) & 1u);
        unsigned long long alive = __ballot(ok), accepted = 0ull;
        int taken = 0;
        // the chain itself is scalar work and two lane reads a connection; what the accepted lanes have to store waits
        // until the chunk is through (stores inside the loop put a dozen more instructions on every step of the chain)
        while (alive && m + taken < limit) {
            const int r = __ffsll((long long)alive) - 1;
            const uint32_t ir = __builtin_amdgcn_readlane(i, r), jr = __builtin_amdgcn_readlane(j, r);
            accepted |= 1ull << r;
            ++taken;
            alive &= ~__ballot(i == ir || j == jr);
        }
        if ((accepted >> lane) & 1ull) {
            const int at = m + __popcll(accepted & ((1ull << lane) - 1ull));     // acceptance order = lane order
            mi[at] = (int32_t)i;
            mj[at] = (int32_t)j;
            ms[at] = __uint_as_float(~(uint32_t)(e >> 32));
            if (more_chunks) {
                atomicOr(&usedA[i >> 5], 1u << (i & 31));
                atomicOr(&usedB[j >> 5], 1u << (j & 31));
            }
        }
        m += taken;
        // the bit maps are written and read by this wavefront only
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    }
    return m;
}

// One workgroup per (image, limb).
//   MODE 0: staged candidates -> sorted by (i, j) -> candidate lists.
//   MODE 1: the same, then sorted by (score desc, i, j) -> greedy matching -> connections.
//   MODE 2: candidate lists in -> matching -> connections.
// Scores are positive, so their bit patterns order like the values; the matching key is
// (~score bits) << 32 | (i << 16 | j), ascending.
template <int MODE>
__global__ __launch_bounds__(kBlock) void k_match(LimbTable tab, int K, int L,
                                                  const int32_t *__restrict__ pcounts, int cap,
                                                  int32_t *cctr, uint64_t *cstage, int ccap2,
                                                  int32_t *ccounts, int32_t *ci, int32_t *cj, float *cs, int ccap,
                                                  int32_t *mcounts, int32_t *mi, int32_t *mj, float *ms, int mcap,
                                                  int32_t *status)
{
    __shared__ uint64_t sk[kLdsSort];
    __shared__ uint32_t usedA[HP_MAX_CAP / 32], usedB[HP_MAX_CAP / 32];
    const int nl = blockIdx.x;
    const int n = nl / L, l = nl - n * L;
    const int cnt = (MODE != 2) ? cctr[nl * kCtrStride] : ccounts[nl];
    const int c = max(min(cnt, ccap), 0);
    if (MODE != 2) {
        __syncthreads();
        if (threadIdx.x == 0) {
            ccounts[nl] = cnt;
            cctr[nl * kCtrStride] = 0;        // sole reader of this list: leave it ready for the next call
        }
    }
    if (MODE != 2) {
        if (cnt > ccap && threadIdx.x == 0) atomicOr(status, (int)HP_STATUS_CAND_OVERFLOW);
    } else if (nl == 0 && threadIdx.x == 0) {
        *status = 0;      // first kernel of hp_assemble; the assembly kernel reports lists beyond their capacity
    }
    uint64_t *g = cstage + (size_t)nl * ccap2;
    const size_t co = (size_t)nl * ccap;
    const int a = tab.a[l], b = tab.b[l];
    const int nA = max(min(pcounts[n * K + a], cap), 0), nB = max(min(pcounts[n * K + b], cap), 0);
    const size_t mo = (size_t)nl * mcap;
    uint64_t *keys;

    if (c <= kRankSort) {
        // Short list: one element per thread, its rank is the number of smaller keys (keys are
        // distinct), counted through LDS broadcasts.
        const int t = threadIdx.x;
        uint64_t e = ~0ull;
        if (t < c) {
            if (MODE != 2)
                e = g[t];
            else
                e = ((uint64_t)(((uint32_t)ci[co + t] << 16) | (uint32_t)cj[co + t]) << 32) |
                    (uint64_t)__float_as_uint(cs[co + t]);
        }
        if (MODE != 2) {
            sk[t] = e;
            __syncthreads();
            if (t < c) {
                int r = 0;
                for (int u = 0; u < c; ++u) r += sk[u] < e;
                ci[co + r] = (int32_t)(e >> 48);
                cj[co + r] = (int32_t)((e >> 32) & 0xffffu);
                cs[co + r] = __uint_as_float((uint32_t)e);
            }
            if (MODE == 0) return;
            __syncthreads();
        }
        const uint64_t key = (t < c) ? ((uint64_t)(~(uint32_t)e) << 32) | (e >> 32) : ~0ull;
        sk[t] = key;
        __syncthreads();
        int r = 0;
        if (t < c)
            for (int u = 0; u < c; ++u) r += sk[u] < key;
        __syncthreads();
        if (t < c) sk[r] = key;
        __syncthreads();
        keys = sk;
    } else {
        int n2 = 1;
        while (n2 < c) n2 <<= 1;
        const bool in_lds = n2 <= kLdsSort;
        keys = in_lds ? sk : g;
        if (MODE != 2) {
            if (in_lds) {
                for (int t = threadIdx.x; t < n2; t += kBlock) sk[t] = t < c ? g[t] : ~0ull;
            } else {
                for (int t = c + threadIdx.x; t < n2; t += kBlock) g[t] = ~0ull;
            }
            __syncthreads();
            block_bitonic_sort(keys, n2);
            for (int t = threadIdx.x; t < c; t += kBlock) {
                uint64_t e = keys[t];
                uint32_t ij = (uint32_t)(e >> 32);
                ci[co + t] = (int32_t)(ij >> 16);
                cj[co + t] = (int32_t)(ij & 0xffffu);
                cs[co + t] = __uint_as_float((uint32_t)e);
                keys[t] = ((uint64_t)(~(uint32_t)e) << 32) | ij;
            }
            if (MODE == 0) return;
        } else {
            for (int t = threadIdx.x; t < n2; t += kBlock) {
                uint64_t e = ~0ull;
                if (t < c) {
                    uint32_t ij = ((uint32_t)ci[co + t] << 16) | (uint32_t)cj[co + t];
                    e = ((uint64_t)(~__float_as_uint(cs[co + t])) << 32) | ij;
                }
                keys[t] = e;
            }
        }
        __syncthreads();
        block_bitonic_sort(keys, n2);
    }

    // keys[0 .. c) now hold (~score bits) << 32 | (i << 16 | j) in matching order
    for (int t = threadIdx.x; t < (nA + 31) / 32; t += kBlock) usedA[t] = 0;
    for (int t = threadIdx.x; t < (nB + 31) / 32; t += kBlock) usedB[t] = 0;
    __syncthreads();
    if (threadIdx.x >= kWave) return;
    const int m = wave_greedy_match(keys, c, nA, nB, min(min(nA, nB), mcap), usedA, usedB, mi + mo, mj + mo, ms + mo);
    if (threadIdx.x == 0) mcounts[nl] = m;
}

// Small-list form of peak ordering + limb scoring + matching in one launch, used when the
// capacities promise at most kSmallPeaks peaks per (image, part) and kSmallCands candidates per
// (image, limb).  Workgroups [0, N*L) each own one (image, limb): they order the two staged
// peak lists in LDS (rank = number of smaller raster keys), score every pair from the LDS
// coordinates, collect the accepted ones in LDS, order them by (i, j) for the candidate output
// and by (score desc, i, j) for the greedy matching.  The workgroup of the first limb that uses a
// part also writes the part's ordered peak list to the caller's arrays.  Results are identical to the general
// kernels; only the number of launches and global-memory round trips differs.
constexpr int kSmallPeaks = 256;
constexpr int kSmallCands = 1024;
constexpr int kSmallBlock = 1024;

template <typename T>
__global__ __launch_bounds__(kSmallBlock) void k_limb_small(
    const T *__restrict__ paf_lo, int h, int w, LimbTable tab, SampleT st, int K,
    int L, int NL, int S, float paf_thr, int need, const int32_t *__restrict__ peak_ctr,
    const uint64_t *__restrict__ peak_stage, int cap, int cap2, int32_t *pcounts, int32_t *px, int32_t *py, float *ps,
    int32_t *ccounts, int32_t *ci, int32_t *cj, float *cs, int ccap, int32_t *mcounts, int32_t *mi, int32_t *mj,
    float *ms, int mcap, int32_t *status, int planes_in_lds)
{
    __shared__ __align__(16) uint64_t sk[kSmallCands];
    __shared__ int lxy[4][kSmallPeaks];          // xA, yA, xB, yB in rank order
    __shared__ float lpaf[4][kSmallPeaks];       // PAF x, y at the peaks of A; x, y at the peaks of B
    __shared__ int lds_cnt, lds_alive;
    __shared__ uint32_t alive_id[kSmallCands];   // pairs alive after stage 1: invalid samples << 16 | i << 8 | j
    __shared__ float alive_acc[kSmallCands];     // and their running sums
    __shared__ uint32_t usedA[kSmallPeaks / 32], usedB[kSmallPeaks / 32];
    extern __shared__ uint32_t lds_paf[];        // the limb's two lo-res PAF planes, when they fit
    const int tid = threadIdx.x;
    const int H = 8 * h, W = 8 * w;

    const int nl = blockIdx.x;
    const int n = nl / L, l = nl - n * L;
    const int a = tab.a[l], b = tab.b[l];
    const int pa = n * K + a, pb = n * K + b;
    const int nA = max(min(peak_ctr[pa * kCtrStride], cap), 0), nB = max(min(peak_ctr[pb * kCtrStride], cap), 0);

    // The x and y planes of a limb lie one after the other.  Every sample of the workgroup's
    // pairs reads them, and the first reads find them in no cache (two dependent rounds of such
    // reads were 6 of the kernel's 15 us), so they are copied to LDS up front, while the peak
    // lists are being ordered; the scoring then runs out of LDS.
    const T *planes = paf_lo + ((size_t)n * 2 * L + 2 * l) * (size_t)h * w;
    if (planes_in_lds) {
        const uint32_t *src = reinterpret_cast<const uint32_t *>(planes);
        const int words = (int)((size_t)2 * h * w * sizeof(T) / 4);
#pragma unroll 8
        for (int t = tid; t < words; t += kSmallBlock) lds_paf[t] = src[t];
    }

    // order the two peak lists: threads [0, 256) take list A, [256, 512) list B.  The first limb
    // that uses a part also publishes the part's ordered list and its count.
    {
        const int half = tid >> 8, t = tid & (kSmallPeaks - 1);
        const int plane = half == 0 ? pa : pb;
        const int cnt = half == 0 ? nA : nB;
        const bool mine = half < 2 && t < cnt;
        const bool publish = half < 2 && tab.writer[half == 0 ? a : b] == l;
        const uint64_t e = mine ? peak_stage[(size_t)plane * cap2 + t] : ~0ull;
        if (half < 2) sk[tid] = e;
        if (tid == 0) lds_cnt = lds_alive = 0;
        if (publish && t == 0) {
            const int raw = peak_ctr[plane * kCtrStride];
            pcounts[plane] = raw;
            if (raw > cap) atomicOr(status, (int)HP_STATUS_PEAK_OVERFLOW);
        }
        __syncthreads();
        if (mine) {
            const int r = rank_below(sk + half * kSmallPeaks, cnt, e);      // entries beyond the list hold ~0
            const int key = (int)(e >> 32);
            const int y = key / W, x = key - y * W;
            lxy[2 * half][r] = x;
            lxy[2 * half + 1][r] = y;
            if (publish) {
                const size_t o = (size_t)plane * cap + r;
                px[o] = x;
                py[o] = y;
                ps[o] = __uint_as_float((uint32_t)e);
            }
        }
        __syncthreads();
    }
    // parts that no limb uses are published by the image's first limb
    if (l == 0) {
        for (int c = 0; c < K; ++c) {
            if (tab.writer[c] >= 0) continue;
            const int plane = n * K + c;
            const int raw = peak_ctr[plane * kCtrStride];
            const int cnt = max(min(raw, cap), 0);
            const uint64_t e = tid < cnt ? peak_stage[(size_t)plane * cap2 + tid] : ~0ull;
            __syncthreads();
            if (tid < kSmallPeaks) sk[tid] = e;
            if (tid == 0) {
                pcounts[plane] = raw;
                if (raw > cap) atomicOr(status, (int)HP_STATUS_PEAK_OVERFLOW);
            }
            __syncthreads();
            if (tid < cnt) {
                const int r = rank_below(sk, cnt, e);
                const int key = (int)(e >> 32);
                const int y = key / W;
                const size_t o = (size_t)plane * cap + r;
                px[o] = key - y * W;
                py[o] = y;
                ps[o] = __uint_as_float((uint32_t)e);
            }
        }
        __syncthreads();
    }

    // score every pair; accepted ones go to the LDS list, tagged (i << 16 | j) << 32 | score bits
    {
        const int P = nA * nB, max_bad = S - need;
        const float inv_nB = 1.0f / (float)nB;
        auto score_all = [&](const T *lx, const T *ly) {
            const float *hx = nullptr, *hy = nullptr;          // the PAFs are recomputed from the lo-res planes
            // the PAF at every peak of the two lists: samples 0 and S-1 of all pairs that start or end there
            {
                const int half = tid >> 8, t = tid & (kSmallPeaks - 1);
                if (half < 2 && t < (half == 0 ? nA : nB))
                    paf_from_lo(lx, ly, h, w, min(max(lxy[2 * half + 1][t], 0), H - 1), min(max(lxy[2 * half][t], 0), W - 1),
                                lpaf[2 * half][t], lpaf[2 * half + 1][t]);
            }
            __syncthreads();
            auto accept = [&](int i, int j, float score) {
                const int slot = atomicAdd(&lds_cnt, 1);
                if (slot < kSmallCands)
                    sk[slot] = ((uint64_t)(((uint32_t)i << 16) | (uint32_t)j) << 32) | (uint64_t)__float_as_uint(score);
            };
            // stage 1 for every pair; the few that are still alive are listed, so that stage 2 (most of a pair's
            // samples) is run by as many lanes as there are such pairs instead of by every wavefront for a few lanes
            for (int p = tid; p < P; p += kSmallBlock) {
                int i = (int)((float)p * inv_nB);
                int j = p - i * nB;
                while (j < 0) { --i; j += nB; }
                while (j >= nB) { ++i; j -= nB; }
                PairGeom g;
                int bad;
                float acc;
                if (!pair_geometry(lxy[0][i], lxy[1][i], lxy[2][j], lxy[3][j], g)) continue;
                if (!pair_stage1<T, false>(g, lpaf[0][i], lpaf[1][i], lpaf[2][j], lpaf[3][j], S, st, paf_thr, max_bad, H, W, h, w,
                                           hx, hy, lx, ly, bad, acc))
                    continue;
                const int slot = atomicAdd(&lds_alive, 1);
                if (slot < kSmallCands) {
                    alive_id[slot] = ((uint32_t)bad << 16) | ((uint32_t)i << 8) | (uint32_t)j;
                    alive_acc[slot] = acc;
                } else {
                    // the list is full: finished on the spot
                    float score;
                    if (pair_stage2<T, false>(g, lpaf[2][j], lpaf[3][j], bad, acc, S, st, paf_thr, max_bad, H, W, h, w, hx, hy, lx,
                                              ly, score))
                        accept(i, j, score);
                }
            }
            __syncthreads();
            const int n_alive = min(lds_alive, kSmallCands);
            for (int q = tid; q < n_alive; q += kSmallBlock) {
                const uint32_t id = alive_id[q];
                const int i = (int)((id >> 8) & 0xffu), j = (int)(id & 0xffu);
                PairGeom g;
                pair_geometry(lxy[0][i], lxy[1][i], lxy[2][j], lxy[3][j], g);
                float score;
                if (pair_stage2<T, false>(g, lpaf[2][j], lpaf[3][j], (int)(id >> 16), alive_acc[q], S, st, paf_thr, max_bad, H, W, h,
                                          w, hx, hy, lx, ly, score))
                    accept(i, j, score);
            }
        };
        if (planes_in_lds)
            score_all(reinterpret_cast<const T *>(lds_paf), reinterpret_cast<const T *>(lds_paf) + (size_t)h * w);
        else
            score_all(planes, planes + (size_t)h * w);
        __syncthreads();
    }

    const int cnt = lds_cnt;
    const int c = min(cnt, min(ccap, kSmallCands));
    if (tid == 0) {
        ccounts[nl] = cnt;
        if (cnt > ccap) atomicOr(status, (int)HP_STATUS_CAND_OVERFLOW);
    }
    // candidates in (i, j) order; the list is padded with ~0 for the rank counts (one entry per thread)
    const uint64_t e = tid < c ? sk[tid] : ~0ull;
    __syncthreads();
    sk[tid] = e;
    __syncthreads();
    const size_t co = (size_t)nl * ccap;
    if (tid < c) {
        const int r = rank_below(sk, c, e);
        ci[co + r] = (int32_t)(e >> 48);
        cj[co + r] = (int32_t)((e >> 32) & 0xffffu);
        cs[co + r] = __uint_as_float((uint32_t)e);
    }
    __syncthreads();
    // matching order: (~score bits) << 32 | (i << 16 | j), ascending
    const uint64_t key = tid < c ? ((uint64_t)(~(uint32_t)e) << 32) | (e >> 32) : ~0ull;
    sk[tid] = key;
    if (tid < kSmallPeaks / 32) usedA[tid] = usedB[tid] = 0;
    __syncthreads();
    const int r2 = tid < c ? rank_below(sk, c, key) : 0;
    __syncthreads();
    if (tid < c) sk[r2] = key;
    __syncthreads();

    const size_t mo = (size_t)nl * mcap;
    if (tid >= kWave) return;
    const int m = wave_greedy_match(sk, c, nA, nB, min(min(nA, nB), mcap), usedA, usedB, mi + mo, mj + mo, ms + mo);
    if (tid == 0) mcounts[nl] = m;
}

bool limb_small_applies(int cap, int ccap) { return cap <= kSmallPeaks && ccap <= kSmallCands; }

hipError_t launch_limb_small(const void *paf_lo, hp_dtype dt, int N, int h, int w, const LimbTable &T, int K, int L,
                             const hp_params &prm, int need, const int32_t *peak_ctr, const uint64_t *peak_stage,
                             int cap2, const hp_peaks &pk, const hp_pairs &cands, const hp_pairs &conns,
                             int32_t *status, hipStream_t s)
{
    SampleT st;
    for (int k = 0; k < HP_MAX_SAMPLES; ++k) st.t[k] = (float)k / (float)(prm.n_samples - 1);
    dim3 grid(N * L), block(kSmallBlock);
    // the two PAF planes of a limb go to LDS when they fit beside the kernel's own tables (and can
    // be copied as whole 32-bit words)
    const size_t plane_bytes = (size_t)2 * h * w * (dt == HP_F16 ? 2 : 4);
    // (the kernel's own tables take 24 KB of the 64 KB a workgroup gets without asking for more)
    const int in_lds = plane_bytes <= 39 * 1024 && plane_bytes % 4 == 0 && ((uintptr_t)paf_lo & 3) == 0;
    const size_t lds = in_lds ? plane_bytes : 0;
#define HP_LIMB_SMALL_ARGS(LO)                                                                                        \
    LO, h, w, T, st, K, L, N *L, prm.n_samples, prm.paf_thr, need, peak_ctr, peak_stage, pk.cap, cap2, pk.count, pk.x, \
        pk.y, pk.score, cands.count, cands.i, cands.j, cands.score, cands.cap, conns.count, conns.i, conns.j,          \
        conns.score, conns.cap, status, in_lds
    if (dt == HP_F16)
        HP_KERNEL((k_limb_small<__half>), grid, block, lds, s, HP_LIMB_SMALL_ARGS((const __half *)paf_lo));
    else
        HP_KERNEL((k_limb_small<float>), grid, block, lds, s, HP_LIMB_SMALL_ARGS((const float *)paf_lo));
#undef HP_LIMB_SMALL_ARGS
    return hipGetLastError();
}

hipError_t launch_match(int mode, const LimbTable &T, int N, int K, int L, const hp_peaks &pk,
                        int32_t *cctr, uint64_t *cstage, int ccap2, const hp_pairs &cands,
                        const hp_pairs &conns, int32_t *status, hipStream_t s)
{
    dim3 grid(N * L), block(kBlock);
    if (mode == 0)
        HP_KERNEL((k_match<0>), grid, block, 0, s, T, K, L, pk.count, pk.cap, cctr, cstage, ccap2, cands.count,
                           cands.i, cands.j, cands.score, cands.cap, (int32_t *)nullptr, (int32_t *)nullptr,
                           (int32_t *)nullptr, (float *)nullptr, 0, status);
    else if (mode == 1)
        HP_KERNEL((k_match<1>), grid, block, 0, s, T, K, L, pk.count, pk.cap, cctr, cstage, ccap2, cands.count,
                           cands.i, cands.j, cands.score, cands.cap, conns.count, conns.i, conns.j, conns.score,
                           conns.cap, status);
    else
        HP_KERNEL((k_match<2>), grid, block, 0, s, T, K, L, pk.count, pk.cap, cctr, cstage, ccap2, cands.count,
                           cands.i, cands.j, cands.score, cands.cap, conns.count, conns.i, conns.j, conns.score,
                           conns.cap, status);
    return hipGetLastError();
}

}  // namespace hp

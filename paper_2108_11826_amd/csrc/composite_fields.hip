// Decoder of the composite-field family (Section 2.3 names PifPaf as the engine's third algorithm class): the fine
// confidence map of the part intensity fields, seeds, and persons grown along the part association fields.  The
// rules (C0-C8) are written at hp_cf_decode in hp.h; every float operation below is one of theirs, in their order.
//
// The method's own description builds the fine map of every part (one Gaussian per grid cell, summed at image
// resolution) and then reads it at a few hundred points: the seeds and the two end points of every association.
// At 368 x 656 and 17 parts that map is 16 MB per image to fill and throw away.  Here the map is a function, not an
// array: k_cf_pif lists the active cells of a part in ascending cell order (the order the sum is defined in), and
// whoever needs a map value sums, in that order, the listed cells whose window holds the pixel: the same additions,
// bit for bit, as reading the filled array.  hp_cf_field still fills the array for callers who want to look at it.
//   k_cf_pif   one workgroup per (image, part): ordered compaction of the active cells, then every listed cell's
//              own map value (its seed value);
//   k_cf_paf   one workgroup per (image, limb): ordered compaction of the active associations and the two map
//              samples of each (the two parts' cell lists held in LDS); one more workgroup per image sorts the seeds;
//   k_cf_link  what each association would propose if it won a search: the target's radius and the point the reverse
//              search leads back to, neither of which depends on the person (a wavefront per association and
//              direction);
//   k_cf_grow  one workgroup per image: the occupancy test of up to 256 seeds at a time is one test per thread,
//              repeated only against each newly finished person; a person grows in rounds, a wavefront per
//              frontier limb (the search, 64 associations at a time, over records held in LDS);
//   k_cf_field one wavefront per strip of 64 x 8 pixels: the part's listed cells whose window meets the strip, then
//              the sum per pixel, eight 8 x 8 groups of pixels a lane.
#include <limits.h>
#include <string.h>

#include <algorithm>

#include "hp_dev.h"

namespace hp {

constexpr int kCfBlock = 256;       // k_cf_pif, k_cf_paf, k_cf_field
constexpr int kCfGrowBlock = 256;   // k_cf_grow: four wavefronts, one per frontier limb of a round
// hp_cf_field: a wavefront fills a strip of kCfTileW x kCfStripH pixels, a workgroup four strips one above the other
constexpr int kCfTileW = 64, kCfStripH = 8, kCfTileH = kCfStripH * (kCfBlock / 64);

struct CFParams {
    float pif_thr, paf_thr, seed_thr, grow_thr, rev_tol;
    int min_parts, stride, Fh, Fw, K, L, cap, acap, pcap;
};

// Records of the active cells, in the caller's workspace.
struct CFWork {
    float4 *pif_a;        // [N][K][cap]   X, Y, inv, c
    int4 *pif_b;          // [N][K][cap]   xr, yr, bits of sg, window
    float4 *fwd_s;        // [N][L][acap]  searched from part a: P1.x, P1.y, 1 / B1, c * F2
    float4 *bwd_s;        // [N][L][acap]  searched from part b: P2.x, P2.y, 1 / B2, c * F1
    float4 *fwd_r;        // [N][L][acap]  followed forwards: radius at P2, the point the reverse search leads back to, 1 (0: none)
    float4 *bwd_r;        // [N][L][acap]  followed backwards
    float4 *seed;         // [N][K * cap]  the seeds in the order they are taken: X, Y, sg, value
    float4 *ghost;        // [N][K * cap]  the seeds grown in vain: X, Y, sg, bits of the part
    int32_t *seed_part;   // [N][K * cap]
    int32_t *seed_count;  // [N]
    size_t bytes;
};

static CFWork cf_layout(void *base, int N, int K, int L, int cap, int acap)
{
    CFWork w;
    char *p = (char *)base;
    size_t off = 0;
    auto take = [&](size_t bytes) {
        char *q = p ? p + off : nullptr;
        off += (bytes + 255) & ~(size_t)255;
        return q;
    };
    w.pif_a = (float4 *)take(sizeof(float4) * (size_t)N * K * cap);
    w.pif_b = (int4 *)take(sizeof(int4) * (size_t)N * K * cap);
    w.fwd_s = (float4 *)take(sizeof(float4) * (size_t)N * L * acap);
    w.bwd_s = (float4 *)take(sizeof(float4) * (size_t)N * L * acap);
    w.fwd_r = (float4 *)take(sizeof(float4) * (size_t)N * L * acap);
    w.bwd_r = (float4 *)take(sizeof(float4) * (size_t)N * L * acap);
    w.seed = (float4 *)take(sizeof(float4) * (size_t)N * K * cap);
    w.ghost = (float4 *)take(sizeof(float4) * (size_t)N * K * cap);
    w.seed_part = (int32_t *)take(sizeof(int32_t) * (size_t)N * K * cap);
    w.seed_count = (int32_t *)take(sizeof(int32_t) * (size_t)N);
    w.bytes = off;
    return w;
}

size_t cf_workspace_bytes(int N, int K, int L, int cap, int acap) { return cf_layout(nullptr, N, K, L, cap, acap).bytes; }

// C0: exp(-t) with fixed arithmetic.
__device__ __forceinline__ float cf_expneg(float t)
{
    const float tc = fmaxf(fminf(t, 80.0f), 0.0f);
    const float y = tc * 0x1.715476p+0f;
    const float n = rintf(y);
    const float z = (y - n) * -0x1.62e430p-1f;
    float p = 0x1.6c16c2p-10f;
    p = __fmaf_rn(p, z, 0x1.111112p-7f);
    p = __fmaf_rn(p, z, 0x1.555556p-5f);
    p = __fmaf_rn(p, z, 0x1.555556p-3f);
    p = __fmaf_rn(p, z, 0.5f);
    p = __fmaf_rn(p, z, 1.0f);
    p = __fmaf_rn(p, z, 1.0f);
    return ldexpf(p, -(int)n);
}

__device__ __forceinline__ bool cf_on_map(float X, float Y, int H, int W)
{
    return X >= 0.0f && X <= (float)(W - 1) && Y >= 0.0f && Y <= (float)(H - 1);
}

__device__ __forceinline__ int cf_window(float sg) { return (int)fminf(ceilf(3.0f * sg), 24.0f); }

// C2 at one pixel: the listed cells of a part, in list (ascending cell) order.  The list is walked 32 cells at a time
// in two passes: the window tests first (independent LDS reads that go out together), then the cells whose window
// holds the pixel, still in ascending order, each with its Gaussian (a thread working alone spends its time waiting
// for LDS: one pass with the test and the sum interleaved took three times as long).
__device__ __forceinline__ float cf_sample(const float4 *ra, const int4 *rb, int n, int px, int py)
{
    float f = 0.0f;
    for (int j0 = 0; j0 < n; j0 += 32) {
        uint32_t in = 0u;
#pragma unroll 8
        for (int u = 0; u < 32; ++u) {
            if (j0 + u < n) {
                const int4 b = rb[j0 + u];
                in |= (abs(px - b.x) <= b.w && abs(py - b.y) <= b.w) ? 1u << u : 0u;
            }
        }
        while (in) {
            const int u = __ffs((int)in) - 1;
            in &= in - 1u;
            const float4 a = ra[j0 + u];
            const float dx = (float)px - a.x, dy = (float)py - a.y;
            const float d2 = dx * dx + dy * dy;
            f = f + a.w * cf_expneg(d2 * a.z);
        }
    }
    return f;
}

// Ordered compaction of kCfPer * 256 items a step: flag u of thread t stands for item u * 256 + t of the step (so that
// a wavefront's loads stay contiguous); returns where each flagged item goes, counting from the step's first one, and
// the step's total.  `scratch` holds kCfPer * 4 ints of LDS.  Contains two barriers.
constexpr int kCfPer = 8;
__device__ __forceinline__ void cf_scan(const bool (&flag)[kCfPer], int *scratch, int (&at)[kCfPer], int &total)
{
    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x >> 6;
    int within[kCfPer];
#pragma unroll
    for (int u = 0; u < kCfPer; ++u) {
        const unsigned long long m = __ballot(flag[u]);
        within[u] = __popcll(m & ((1ull << lane) - 1ull));
        if (lane == 0) scratch[u * 4 + wv] = __popcll(m);
    }
    __syncthreads();
    int run = 0;
#pragma unroll
    for (int u = 0; u < kCfPer; ++u) {
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            if (w == wv) at[u] = run + within[u];
            run += scratch[u * 4 + w];
        }
    }
    total = run;
    __syncthreads();
}

// ---- C1, C3: active cells of a part and their map values ---------------------------------------------------------
__global__ __launch_bounds__(kCfBlock) void k_cf_pif(const float *__restrict__ pif, CFParams P, CFWork ws,
                                                     int32_t *__restrict__ out_cell, float *__restrict__ out_val,
                                                     int32_t *__restrict__ out_count, int32_t *__restrict__ status)
{
    extern __shared__ float4 s_dyn4[];
    float4 *s_a = s_dyn4;                     // [cap]
    int4 *s_b = (int4 *)(s_dyn4 + P.cap);     // [cap]
    int *s_cell = (int *)(s_dyn4 + 2 * P.cap);  // [cap]
    __shared__ int s_scan[kCfPer * 4];

    const int k = blockIdx.x, n = blockIdx.y, tid = threadIdx.x;
    const int cells = P.Fh * P.Fw, H = P.Fh * P.stride, W = P.Fw * P.stride;
    const float *f = pif + ((size_t)n * P.K + k) * 5 * cells;
    const size_t list = ((size_t)n * P.K + k) * P.cap;
    const float s = (float)P.stride;

    int count = 0;
    for (int c0 = 0; c0 < cells; c0 += kCfPer * kCfBlock) {
        bool act[kCfPer];
        float X[kCfPer], Y[kCfPer], c[kCfPer], sig[kCfPer];
#pragma unroll
        for (int u = 0; u < kCfPer; ++u) {
            const int cell = c0 + u * kCfBlock + tid;
            act[u] = false;
            X[u] = Y[u] = c[u] = sig[u] = 0.0f;
            if (cell < cells) {
                const int gy = cell / P.Fw, gx = cell - gy * P.Fw;
                c[u] = f[cell];
                X[u] = ((float)gx + f[1 * cells + cell]) * s;
                Y[u] = ((float)gy + f[2 * cells + cell]) * s;
                sig[u] = f[4 * cells + cell];   // fetched with the rest: a second round of loads would cost as much again
                act[u] = c[u] > P.pif_thr && cf_on_map(X[u], Y[u], H, W);
            }
        }
        int at[kCfPer], total;
        cf_scan(act, s_scan, at, total);
#pragma unroll
        for (int u = 0; u < kCfPer; ++u) {
            const int cell = c0 + u * kCfBlock + tid, to = count + at[u];
            if (act[u] && to < P.cap) {
                const float sg = fmaxf(sig[u] * s, 1.0f);
                s_a[to] = make_float4(X[u], Y[u], 0.5f / (sg * sg), c[u]);
                s_b[to] = make_int4((int)rintf(X[u]), (int)rintf(Y[u]), __float_as_int(sg), cf_window(sg));
                s_cell[to] = cell;
            }
        }
        count += total;
    }
    __syncthreads();
    // the list leaves LDS once, after the last barrier (a barrier also waits for the stores issued before it)
    const int m = min(count, P.cap);
    for (int i = tid; i < m; i += kCfBlock) {
        ws.pif_a[list + i] = s_a[i];
        ws.pif_b[list + i] = s_b[i];
        out_cell[list + i] = s_cell[i];
    }
    for (int i = tid; i < m; i += kCfBlock) out_val[list + i] = cf_sample(s_a, s_b, m, s_b[i].x, s_b[i].y);
    if (tid == 0) {
        out_count[(size_t)n * P.K + k] = count;
        if (count > P.cap) atomicOr(status, HP_STATUS_PEAK_OVERFLOW);
    }
}

// ---- C4: active associations of a limb, their map samples, and what each would propose ---------------------------
struct CFLimbs {
    uint8_t a[HP_MAX_LIMBS], b[HP_MAX_LIMBS];
};

// C4 score of one search record (source point x, y; 1 / spread; c * F of the other end) for a joint at (qx, qy)
__device__ __forceinline__ float cf_score(const float4 r, float qx, float qy)
{
    const float dx = qx - r.x, dy = qy - r.y;
    const float d = sqrtf(dx * dx + dy * dy);
    return r.w * cf_expneg(d * r.z);
}

// C3 for one image: the seeds sorted by (value descending, part ascending, cell ascending), written to the workspace.
__device__ void cf_sort_seeds(const CFParams &P, const CFWork &ws, int n, const int32_t *__restrict__ pif_count,
                              const float *__restrict__ pif_val, uint64_t *s_key)
{
    __shared__ int s_nseeds, s_cnt[HP_MAX_PARTS];
    const int tid = threadIdx.x, K = P.K;
    if (tid == 0) s_nseeds = 0;
    if (tid < K) s_cnt[tid] = min(pif_count[(size_t)n * K + tid], P.cap);
    __syncthreads();
    // every (part, rank) slot of the image, four a thread at a time: the values are fetched before it is known which
    // of them exist (a slot beyond its list's end lies inside the array and is not used), so that the loads of all
    // parts go out together; the keys are unique, so the order they are appended in does not matter
    constexpr int kPer = 4;
    const int slots = K * P.cap;
    for (int s0 = 0; s0 < slots; s0 += kPer * kCfBlock) {
        float v[kPer];
#pragma unroll
        for (int u = 0; u < kPer; ++u) {
            const int idx = s0 + u * kCfBlock + tid;
            v[u] = idx < slots ? pif_val[(size_t)n * slots + idx] : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < kPer; ++u) {
            const int idx = s0 + u * kCfBlock + tid;
            if (idx >= slots) continue;
            const int k = idx / P.cap, q = idx - k * P.cap;
            if (q < s_cnt[k] && v[u] > P.seed_thr)
                s_key[atomicAdd(&s_nseeds, 1)] = ((uint64_t)(~float_order(v[u])) << 32) | (uint32_t)((k << 16) | q);
        }
    }
    __syncthreads();
    const int ns = s_nseeds;                                   // at most K * cap <= the seed capacity
    int n2 = 1;
    while (n2 < ns) n2 <<= 1;
    for (int i = ns + tid; i < n2; i += kCfBlock) s_key[i] = ~0ull;
    __syncthreads();
    block_bitonic_sort(s_key, n2);   // ends with a barrier
    const size_t base = (size_t)n * K * P.cap;
    for (int i = tid; i < ns; i += kCfBlock) {
        const uint64_t key = s_key[i];
        const int k = (int)((uint32_t)key >> 16), rank = (int)((uint32_t)key & 0xFFFFu);
        const float4 ra = ws.pif_a[((size_t)n * K + k) * P.cap + rank];
        const int4 rb = ws.pif_b[((size_t)n * K + k) * P.cap + rank];
        ws.seed[base + i] = make_float4(ra.x, ra.y, __int_as_float(rb.z), float_unorder(~(uint32_t)(key >> 32)));
        ws.seed_part[base + i] = k;
    }
    if (tid == 0) ws.seed_count[n] = ns;
}

// Workgroups (l < L, n): limb l of image n.  Workgroups (L, n): the seeds of image n.
// kStaged: the records stay in LDS until their map values are known and go to the lists once (a barrier also waits
// for the global stores issued before it, and the records written early would be read back and written again).
constexpr int kCfPafStage = 1024;   // records a list may hold for the staged form
template <bool kStaged>
__global__ __launch_bounds__(kCfBlock) void k_cf_paf(const float *__restrict__ paf, CFParams P,
                                                     CFWork ws, CFLimbs limbs, const int32_t *__restrict__ pif_count,
                                                     const float *__restrict__ pif_val, int32_t *__restrict__ out_cell,
                                                     float *__restrict__ out_f1, float *__restrict__ out_f2,
                                                     int32_t *__restrict__ out_count, int32_t *__restrict__ status)
{
    extern __shared__ float4 s_dyn4[];
    const int l = blockIdx.x, n = blockIdx.y, tid = threadIdx.x;
    if (l == P.L) {
        cf_sort_seeds(P, ws, n, pif_count, pif_val, (uint64_t *)s_dyn4);
        return;
    }
    float4 *s_aa = s_dyn4;                        // part a: [cap] X, Y, inv, c
    int4 *s_ab = (int4 *)(s_dyn4 + P.cap);        //         [cap] xr, yr, sg, cell
    float4 *s_ba = s_dyn4 + 2 * P.cap;            // part b
    int4 *s_bb = (int4 *)(s_dyn4 + 3 * P.cap);
    float4 *s_fs = s_dyn4 + 4 * P.cap;            // staged records: [acap] forwards, [acap] backwards, [acap] cells
    float4 *s_bs = s_fs + P.acap;
    int *s_cell = (int *)(s_bs + P.acap);
    __shared__ int s_scan[kCfPer * 4];
    __shared__ uint8_t s_la[HP_MAX_LIMBS], s_lb[HP_MAX_LIMBS];

    if (tid == 0) {
#pragma unroll
        for (int i = 0; i < HP_MAX_LIMBS; ++i) {
            s_la[i] = limbs.a[i];
            s_lb[i] = limbs.b[i];
        }
    }
    __syncthreads();
    const int pa = s_la[l], pb = s_lb[l];
    const int na = min(pif_count[(size_t)n * P.K + pa], P.cap), nb = min(pif_count[(size_t)n * P.K + pb], P.cap);
    for (int i = tid; i < na; i += kCfBlock) {
        s_aa[i] = ws.pif_a[((size_t)n * P.K + pa) * P.cap + i];
        s_ab[i] = ws.pif_b[((size_t)n * P.K + pa) * P.cap + i];
    }
    for (int i = tid; i < nb; i += kCfBlock) {
        s_ba[i] = ws.pif_a[((size_t)n * P.K + pb) * P.cap + i];
        s_bb[i] = ws.pif_b[((size_t)n * P.K + pb) * P.cap + i];
    }

    const int cells = P.Fh * P.Fw, H = P.Fh * P.stride, W = P.Fw * P.stride;
    const float *f = paf + ((size_t)n * P.L + l) * 7 * cells;
    const size_t list = ((size_t)n * P.L + l) * P.acap;
    const float s = (float)P.stride;
    float4 *fs = ws.fwd_s + list, *bs = ws.bwd_s + list;

    int count = 0;
    for (int c0 = 0; c0 < cells; c0 += kCfPer * kCfBlock) {
        bool act[kCfPer];
        float c[kCfPer], x1[kCfPer], y1[kCfPer], x2[kCfPer], y2[kCfPer], b1[kCfPer], b2[kCfPer];
#pragma unroll
        for (int u = 0; u < kCfPer; ++u) {
            const int cell = c0 + u * kCfBlock + tid;
            act[u] = false;
            c[u] = x1[u] = y1[u] = x2[u] = y2[u] = b1[u] = b2[u] = 0.0f;
            if (cell < cells) {
                const int gy = cell / P.Fw, gx = cell - gy * P.Fw;
                c[u] = f[cell];
                x1[u] = ((float)gx + f[1 * cells + cell]) * s;
                y1[u] = ((float)gy + f[2 * cells + cell]) * s;
                x2[u] = ((float)gx + f[4 * cells + cell]) * s;
                y2[u] = ((float)gy + f[5 * cells + cell]) * s;
                b1[u] = f[3 * cells + cell];   // fetched with the rest: a second round of loads would cost as much again
                b2[u] = f[6 * cells + cell];
                act[u] = c[u] > P.paf_thr && cf_on_map(x1[u], y1[u], H, W) && cf_on_map(x2[u], y2[u], H, W);
            }
        }
        int at[kCfPer], total;
        cf_scan(act, s_scan, at, total);   // its first barrier also covers the lists above
#pragma unroll
        for (int u = 0; u < kCfPer; ++u) {
            const int cell = c0 + u * kCfBlock + tid, to = count + at[u];
            if (act[u] && to < P.acap) {
                const float iB1 = 1.0f / fmaxf(b1[u] * s, 1.0f), iB2 = 1.0f / fmaxf(b2[u] * s, 1.0f);
                const float4 rf = make_float4(x1[u], y1[u], iB1, c[u]);   // c is replaced by c * F2 below
                const float4 rb = make_float4(x2[u], y2[u], iB2, c[u]);
                if constexpr (kStaged) {
                    s_fs[to] = rf;
                    s_bs[to] = rb;
                    s_cell[to] = cell;
                } else {
                    fs[to] = rf;
                    bs[to] = rb;
                    out_cell[list + to] = cell;
                }
            }
        }
        count += total;
    }
    __syncthreads();   // the records written above are read back by other threads of this workgroup
    // one thread per sample: even lanes take F1 of a candidate, odd lanes its F2, and the pair swaps the results
    const int m = min(count, P.acap);
    for (int j0 = 0; j0 < 2 * m; j0 += kCfBlock) {
        const int j = j0 + tid, i = j >> 1;
        const bool second = (j & 1) != 0, on = j < 2 * m;
        float4 r = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        if constexpr (kStaged) {
            if (on) r = second ? s_bs[i] : s_fs[i];
        } else {
            if (on) r = second ? bs[i] : fs[i];
        }
        const float F = cf_sample(second ? s_ba : s_aa, second ? s_bb : s_ab, on ? (second ? nb : na) : 0,
                                  (int)rintf(r.x), (int)rintf(r.y));
        const float other = __shfl_xor(F, 1);
        if (on) {
            r.w = r.w * other;
            if (second) {
                out_f2[list + i] = F;
                bs[i] = r;
            } else {
                out_f1[list + i] = F;
                fs[i] = r;
                if constexpr (kStaged) out_cell[list + i] = s_cell[i];
            }
        }
    }
    if (tid == 0) {
        out_count[(size_t)n * P.L + l] = count;
        if (count > P.acap) atomicOr(status, HP_STATUS_CAND_OVERFLOW);
    }
}

// ---- C5-C8: persons of one image ---------------------------------------------------------------------------------
// C7 for one joint of a recorded person (x, y, radius, value; value 0 = part not held)
__device__ __forceinline__ bool cf_covers(const float4 j, float x, float y)
{
    if (!(j.w > 0.0f)) return false;
    const float dx = x - j.x, dy = y - j.y;
    return dx * dx + dy * dy <= j.z * j.z;
}

// C4: the best record of a list for a joint at (qx, qy), searched by one wavefront.  Returns
// (score order) << 32 | (0xFFFFFFFF - index), the same in every lane, or 0 when no score exceeds `above`.
// The lanes' candidates meet in `slot`, an LDS word of this wavefront's own: LDS serves one wavefront's requests in
// the order they were issued, so the clearing store, the maxima and the final load need no barrier between them
// (and cost about a quarter of a butterfly of twelve cross-lane moves).  Callers pass pointers whose memory (LDS or
// global) the compiler can see: a pointer that may be either compiles to flat loads, several times slower on LDS.
__device__ __forceinline__ uint64_t cf_search(const float4 *S, int cnt, float qx, float qy, float above, int lane,
                                              unsigned long long *slot)
{
    unsigned long long key = 0ull;
    // the next record is on its way while this one is scored
    float4 next = lane < cnt ? S[lane] : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    for (int i = lane; i < cnt; i += kWave) {
        const float4 rec = next;
        if (i + kWave < cnt) next = S[i + kWave];
        const float sc = cf_score(rec, qx, qy);
        if (sc > above) {
            const unsigned long long mine = ((unsigned long long)float_order(sc) << 32) | (uint32_t)(0xFFFFFFFFu - (uint32_t)i);
            key = mine > key ? mine : key;
        }
    }
    if (lane == 0) __hip_atomic_store(slot, 0ull, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
    __builtin_amdgcn_wave_barrier();
    if (key != 0ull) __hip_atomic_fetch_max(slot, key, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
    __builtin_amdgcn_wave_barrier();
    return __hip_atomic_load(slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
}

// ---- C5, the part that does not depend on the person ------------------------------------------------------------
// What the winner of a search proposes besides its point: the target's radius and the point the reverse search
// leads back to.  Task 2 i: association i followed forwards; task 2 i + 1: backwards.  A wavefront per task, the
// tasks of a limb dealt to the 32 wavefronts of eight workgroups (one workgroup a limb took 60 us at 140 associations).
constexpr int kCfLinkSlices = 8, kCfLinkStage = 2048;
__global__ __launch_bounds__(kCfBlock) void k_cf_link(const float *__restrict__ pif, CFParams P, CFWork ws, CFLimbs limbs,
                                                      const int32_t *__restrict__ paf_count)
{
    extern __shared__ float4 s_dyn4[];                      // [2][staged] the limb's search records, when they fit
    __shared__ unsigned long long s_best[kCfBlock / kWave];
    const int l = blockIdx.x, n = blockIdx.y, z = blockIdx.z, tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid >> 6;
    const int m = min(paf_count[(size_t)n * P.L + l], P.acap);
    if (z * (kCfBlock / kWave) >= 2 * m) return;            // the same for the whole workgroup
    const size_t list = ((size_t)n * P.L + l) * P.acap;
    const int pa = limbs.a[l], pb = limbs.b[l], cells = P.Fh * P.Fw;
    const float *sig_a = pif + (((size_t)n * P.K + pa) * 5 + 4) * cells, *sig_b = pif + (((size_t)n * P.K + pb) * 5 + 4) * cells;
    // fs, bs: the limb's search records, forwards and backwards (in LDS or in the workspace: one copy of the loop each)
    auto tasks = [&](const float4 *fs, const float4 *bs) {
        for (int t = z * (kCfBlock / kWave) + wv; t < 2 * m; t += kCfLinkSlices * (kCfBlock / kWave)) {
            const int i = t >> 1;
            const bool forward = (t & 1) == 0;
            const float4 *back = forward ? bs : fs, *from = forward ? fs : bs;   // searched on the way back; holds the points led back to
            const float tx = back[i].x, ty = back[i].y;
            const uint64_t found = cf_search(back, m, tx, ty, 0.0f, lane, &s_best[wv]);
            if (lane == 0) {
                const int cy = (int)rintf(ty) / P.stride, cx = (int)rintf(tx) / P.stride;
                const float rad = fmaxf((forward ? sig_b : sig_a)[(size_t)cy * P.Fw + cx] * (float)P.stride, 1.0f);
                float4 res = make_float4(rad, 0.0f, 0.0f, 0.0f);
                if (found != 0ull) {
                    const float4 rr = from[(int)(0xFFFFFFFFu - (uint32_t)found)];
                    res = make_float4(rad, rr.x, rr.y, 1.0f);
                }
                (forward ? ws.fwd_r : ws.bwd_r)[list + i] = res;
            }
        }
    };
    if (m <= kCfLinkStage) {
        for (int i = tid; i < m; i += kCfBlock) {
            s_dyn4[i] = ws.fwd_s[list + i];
            s_dyn4[m + i] = ws.bwd_s[list + i];
        }
        __syncthreads();
        tasks(s_dyn4, s_dyn4 + m);
    } else {
        tasks(ws.fwd_s + list, ws.bwd_s + list);
    }
}

// One workgroup per image.  The loop is a chain of short dependent steps, so it is built around what a step costs
// here: a barrier waits for the workgroup's outstanding global stores, so nothing is stored to global memory before
// the end (persons, their part counts and scores, and the seeds grown in vain live in LDS); there is one barrier to
// pick the next seed, one to set its person up and one per round of growth (every wavefront folds the round's
// proposals into the person by itself, all writing the same values), one more when a person is recorded.
constexpr int kCfGhostLds = 256;   // seeds grown in vain that are remembered in LDS; later ones go to the workspace

__global__ __launch_bounds__(kCfGrowBlock) void k_cf_grow(CFParams P, CFWork ws, CFLimbs limbs, int lds_cells,
                                                          const int32_t *__restrict__ paf_count, float *__restrict__ xyv,
                                                          int32_t *__restrict__ nparts, float *__restrict__ score,
                                                          int32_t *__restrict__ pcount, int32_t *__restrict__ status)
{
    extern __shared__ float4 s_dyn4[];
    float4 *s_person = s_dyn4;                                 // [pcap][K] x, y, radius, value of the recorded persons
    float *s_pscore = (float *)(s_dyn4 + P.pcap * P.K);        // [pcap]
    int *s_pparts = (int *)(s_pscore + P.pcap);                // [pcap]
    float4 *s_rec = s_dyn4 + P.pcap * P.K + (P.pcap + 1) / 2;  // [4][lds_cells] records of the limbs that fit: searched
                                                               // forwards, backwards; proposed forwards, backwards
    __shared__ uint8_t s_la[HP_MAX_LIMBS], s_lb[HP_MAX_LIMBS];
    __shared__ int s_acnt[HP_MAX_LIMBS], s_off[HP_MAX_LIMBS];  // associations of a limb; where its records start in LDS, -1 = not there
    __shared__ float4 s_prop[2][HP_MAX_LIMBS];                 // a round's proposals (rounds alternate): score, x, y, radius
    __shared__ int s_dst[2][HP_MAX_LIMBS];                     // the part a proposal is for, -1 = the limb proposes nothing
    __shared__ int s_first[2][kCfGrowBlock / kWave];
    __shared__ unsigned long long s_best[kCfGrowBlock / kWave];   // where a wavefront's search candidates meet
    __shared__ float4 s_seed;                                  // the seed being grown: x, y, radius, value
    __shared__ float4 s_ghost[kCfGhostLds];                    // seeds grown in vain: x, y, radius, part
    constexpr int kWaves = kCfGrowBlock / kWave;

    const int n = blockIdx.x, tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid >> 6;
    const int K = P.K, L = P.L;
    if (tid == 0) {
#pragma unroll
        for (int i = 0; i < HP_MAX_LIMBS; ++i) {
            s_la[i] = limbs.a[i];
            s_lb[i] = limbs.b[i];
        }
        int off = 0;
        for (int l = 0; l < L; ++l) {
            const int c = min(paf_count[(size_t)n * L + l], P.acap);
            s_acnt[l] = c;
            s_off[l] = off + c <= lds_cells ? off : -1;
            if (s_off[l] >= 0) off += c;
        }
    }
    __syncthreads();
    for (int l = 0; l < L; ++l) {
        if (s_off[l] < 0) continue;
        const size_t list = ((size_t)n * L + l) * P.acap;
        for (int i = tid; i < s_acnt[l]; i += kCfGrowBlock) {
            s_rec[0 * lds_cells + s_off[l] + i] = ws.fwd_s[list + i];
            s_rec[1 * lds_cells + s_off[l] + i] = ws.bwd_s[list + i];
            s_rec[2 * lds_cells + s_off[l] + i] = ws.fwd_r[list + i];
            s_rec[3 * lds_cells + s_off[l] + i] = ws.bwd_r[list + i];
        }
    }
    // Every wavefront keeps the whole state of the growing person in registers: lane l holds limb l's table entry,
    // lane k the person's joint k, and the set of held parts is a bit mask; all wavefronts update them alike.
    const int ll = lane < L ? lane : 0;
    const int la = s_la[ll], lb = s_lb[ll], lcnt = s_acnt[ll], loff = s_off[ll];
    float jx = 0.0f, jy = 0.0f, jr = 0.0f, jv = 0.0f;
    uint32_t held = 0u;

    const int ns = ws.seed_count[n];
    const size_t seed0 = (size_t)n * K * P.cap;
    float4 *ghost = ws.ghost + seed0;

    int np = 0, ng = 0;  // persons recorded, seeds grown in vain (the same in every thread)
    int it = 0, rounds = 0;
    bool stop = false;   // C8
    for (int base = 0; base < ns && !stop; base += kCfGrowBlock) {
        // this thread's seed of the batch, tested against everything found so far
        const int mine = base + tid;
        bool occ = true;
        int sk = 0;
        float4 sd = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        if (mine < ns) {
            sd = ws.seed[seed0 + mine];
            sk = ws.seed_part[seed0 + mine];
            occ = false;
            for (int p = 0; p < np && !occ; ++p) occ = cf_covers(s_person[p * K + sk], sd.x, sd.y);
            for (int g = 0; g < ng && !occ; ++g) {
                const float4 gh = g < kCfGhostLds ? s_ghost[g] : ghost[g];
                occ = __float_as_int(gh.w) == sk && cf_covers(make_float4(gh.x, gh.y, gh.z, 1.0f), sd.x, sd.y);
            }
        }
        for (;;) {
            // the first seed of the batch that is still free, and its part: index << 5 | part
            const uint64_t free_mask = __ballot(!occ);
            const int first_lane = free_mask ? __ffsll((long long)free_mask) - 1 : 0;
            const int first_part = __builtin_amdgcn_readlane(sk, first_lane);
            if (lane == 0) s_first[it & 1][wv] = free_mask ? ((base + wv * kWave + first_lane) << 5) | first_part : INT_MAX;
            __syncthreads();
            int cur_key = INT_MAX;
#pragma unroll
            for (int u = 0; u < kWaves; ++u) cur_key = min(cur_key, s_first[it & 1][u]);
            ++it;
            if (cur_key == INT_MAX) break;
            if (np >= P.pcap) {
                if (tid == 0) atomicOr(status, HP_STATUS_POSE_OVERFLOW);
                stop = true;
                break;
            }
            // ---- C5: the person of seed `cur` ----
            const int cur = cur_key >> 5, k0 = cur_key & 31;
            const bool owner = mine == cur;
            if (owner) {
                occ = true;
                s_seed = sd;
            }
            __syncthreads();
            const float4 seed = s_seed;
            held = 1u << k0;
            if (lane == k0) {
                jx = seed.x;
                jy = seed.y;
                jr = seed.z;
                jv = seed.w;
            }
            for (;; ++rounds) {
                // the limbs with exactly one part held, in table order
                const uint64_t front = __ballot(lane < L && (((held >> la) ^ (held >> lb)) & 1u));
                if (front == 0ull) break;
                const int par = rounds & 1;
                int nth = 0;
                for (uint64_t rest = front; rest; rest &= rest - 1, ++nth) {
                    if ((nth & (kWaves - 1)) != wv) continue;
                    const int l = __ffsll((long long)rest) - 1;
                    const int a = __builtin_amdgcn_readlane(la, l), b = __builtin_amdgcn_readlane(lb, l);
                    const bool forward = (held >> a) & 1u;
                    const int src = forward ? a : b, dst = forward ? b : a;
                    const float qx = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(jx), src));
                    const float qy = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(jy), src));
                    const size_t list = ((size_t)n * L + l) * P.acap;
                    const int off = __builtin_amdgcn_readlane(loff, l), cnt = __builtin_amdgcn_readlane(lcnt, l);
                    // the searched records (array 0 or 1), the records whose points the winner proposes (the other of the
                    // two), and what else the winner proposes (array 2 or 3): in LDS, or else in the workspace
                    int proposes = -1;
                    float4 prop = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
                    uint64_t found;
                    float4 res = make_float4(0.0f, 0.0f, 0.0f, 0.0f), tgt = res;
                    if (off >= 0) {
                        const float4 *rec = s_rec + off;
                        found = cf_search(rec + (forward ? 0 : 1) * lds_cells, cnt, qx, qy, P.grow_thr, lane, &s_best[wv]);
                        if (found != 0ull) {
                            const int i = (int)(0xFFFFFFFFu - (uint32_t)found);
                            res = rec[(forward ? 2 : 3) * lds_cells + i];
                            tgt = rec[(forward ? 1 : 0) * lds_cells + i];
                        }
                    } else {
                        found = cf_search((forward ? ws.fwd_s : ws.bwd_s) + list, cnt, qx, qy, P.grow_thr, lane, &s_best[wv]);
                        if (found != 0ull) {
                            const int i = (int)(0xFFFFFFFFu - (uint32_t)found);
                            res = (forward ? ws.fwd_r : ws.bwd_r)[list + i];
                            tgt = (forward ? ws.bwd_s : ws.fwd_s)[list + i];
                        }
                    }
                    if (found != 0ull) {
                        const float tx = tgt.x, ty = tgt.y;      // res: radius, point led back to, found
                        const float dx = res.y - qx, dy = res.z - qy;
                        if (res.w != 0.0f && dx * dx + dy * dy <= P.rev_tol * P.rev_tol) {
                            bool taken = false;
                            for (int p = lane; p < np; p += kWave) taken = taken || cf_covers(s_person[p * K + dst], tx, ty);
                            if (__ballot(taken) == 0ull) {
                                proposes = dst;
                                prop = make_float4(float_unorder((uint32_t)(found >> 32)), tx, ty, res.x);
                            }
                        }
                    }
                    if (lane == 0) {
                        s_dst[par][l] = proposes;
                        s_prop[par][l] = prop;
                    }
                }
                __syncthreads();
                // every wavefront folds the proposals in: lane k takes the best one for part k, the earlier limb on ties
                bool have = false;
                {
                    // lane l fetches limb l's proposal (one LDS round trip for all of them); the frontier limbs are
                    // then read across lanes, by the whole wavefront
                    const int my_dst = s_dst[par][ll];
                    const float4 my_prop = s_prop[par][ll];
                    float bsc = 0.0f, bx = 0.0f, by = 0.0f, br = 0.0f;
                    for (uint64_t rest = front; rest; rest &= rest - 1) {
                        const int l = __ffsll((long long)rest) - 1;
                        const int d = __builtin_amdgcn_readlane(my_dst, l);
                        if (d < 0) continue;                                   // the same for the whole wavefront
                        const float sc = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(my_prop.x), l));
                        const float lx = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(my_prop.y), l));
                        const float ly = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(my_prop.z), l));
                        const float lr = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(my_prop.w), l));
                        if (d == lane && (!have || sc > bsc)) {
                            have = true;
                            bsc = sc;
                            bx = lx;
                            by = ly;
                            br = lr;
                        }
                    }
                    if (have) {
                        jx = bx;
                        jy = by;
                        jr = br;
                        jv = bsc;
                    }
                }
                const uint32_t added = (uint32_t)__ballot(have);   // lanes below K <= 32: one bit per part
                held |= added;
                if (added == 0u) {
                    ++rounds;
                    break;
                }
            }

            // ---- C6: record, or remember the seed as grown in vain (C7) ----
            const int parts = __popc(held);
            if (parts >= P.min_parts) {
                if (tid < K) s_person[np * K + tid] = ((held >> tid) & 1u) ? make_float4(jx, jy, jr, jv) : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
                if (wv == 1) {
                    float sum = 0.0f;
                    for (int k = 0; k < K; ++k)
                        if ((held >> k) & 1u) sum = sum + __int_as_float(__builtin_amdgcn_readlane(__float_as_int(jv), k));
                    if (lane == 0) {
                        s_pparts[np] = parts;
                        s_pscore[np] = sum / (float)K;
                    }
                }
                __syncthreads();
                if (!occ) occ = cf_covers(s_person[np * K + sk], sd.x, sd.y);
                ++np;
            } else {
                if (owner) {
                    const float4 gh = make_float4(sd.x, sd.y, sd.z, __int_as_float(sk));
                    if (ng < kCfGhostLds)
                        s_ghost[ng] = gh;
                    else
                        ghost[ng] = gh;
                }
                if (!occ) occ = k0 == sk && cf_covers(make_float4(seed.x, seed.y, seed.z, 1.0f), sd.x, sd.y);
                ++ng;
            }
        }
    }
    __syncthreads();
    for (int i = tid; i < np * K; i += kCfGrowBlock) {
        const float4 j = s_person[i];
        float *o = xyv + ((size_t)n * P.pcap * K + i) * 3;
        o[0] = j.x;
        o[1] = j.y;
        o[2] = j.w;
    }
    for (int p = tid; p < np; p += kCfGrowBlock) {
        nparts[(size_t)n * P.pcap + p] = s_pparts[p];
        score[(size_t)n * P.pcap + p] = s_pscore[p];
    }
    if (tid == 0) pcount[n] = np;
}

// ---- C2 as an array ----------------------------------------------------------------------------------------------
// The Gaussian of C2 for a pixel inside a cell's window.  There t = d2 / (2 sg^2) with |dx|, |dy| <= w + 1/2,
// w = ceil(3 sg) and sg >= 1, so 0 <= t <= (3 + 3/(2 sg))^2 <= 20.25: the clamps of cf_expneg never act and are left
// out, and the sign moves into the constants (y, n and y - n change sign together and exactly, the products and the
// polynomial keep their bits), which saves the negation before the scaling.
__device__ __forceinline__ float cf_expneg_window(float t)
{
    const float y = t * -0x1.715476p+0f;
    const float n = rintf(y);
    const float z = (y - n) * 0x1.62e430p-1f;
    float p = 0x1.6c16c2p-10f;
    p = __fmaf_rn(p, z, 0x1.111112p-7f);
    p = __fmaf_rn(p, z, 0x1.555556p-5f);
    p = __fmaf_rn(p, z, 0x1.555556p-3f);
    p = __fmaf_rn(p, z, 0.5f);
    p = __fmaf_rn(p, z, 1.0f);
    p = __fmaf_rn(p, z, 1.0f);
    return ldexpf(p, (int)n);
}

// A wavefront fills a strip of 64 x 8 pixels on its own (four strips a workgroup, no barrier): it picks, in list order,
// the part's listed cells whose window meets the strip, then sums per pixel.  Most strips meet none and are plain zero
// stores (ordinary stores: an all-zero map then takes as long as a fill, 18 us for the benchmark's 125 MB, where
// non-temporal ones took 25).  The first 64 records are fetched together with the list's length, so that one memory
// round trip separates a strip's start from its first store.
// The sums are what the kernel's time goes to (windows are some 40 pixels wide: with a lane per column of the strip,
// most lanes idled and the arithmetic alone took 20 us).  So the strip is summed as eight groups of 8 x 8 pixels, a
// lane holding one pixel of each: a cell's record sits in scalar registers (it is the same for all lanes), a group
// whose pixels all lie outside the window is skipped after two instructions, and in the others the pixels outside are
// masked off.  Scalar tests of which groups a window meets cost more than they saved: the scalar unit was the
// bottleneck then (35 against 29 us), and so did a jump to the first such group (32 us).  A pixel still adds its
// cells in list order.  The sums then pass through LDS to leave as whole rows.
constexpr int kCfGroups = kCfTileW / 8, kCfTilePitch = kCfTileW + 8;
__host__ __device__ constexpr int cf_field_wave_f4(int cap)
{
    return 2 * cap > kCfStripH * kCfTilePitch / 4 ? 2 * cap : kCfStripH * kCfTilePitch / 4;
}

__global__ __launch_bounds__(kCfBlock) void k_cf_field(CFParams P, CFWork ws, const int32_t *__restrict__ pif_count,
                                                       float *__restrict__ out)
{
    extern __shared__ float4 s_dyn4[];
    const int plane = blockIdx.z, tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    float4 *s_a = s_dyn4 + (size_t)wv * cf_field_wave_f4(P.cap);   // [cap] this wavefront's cells, in list order
    int4 *s_b = (int4 *)(s_a + P.cap);
    float *tile = (float *)s_a;                                    // [8][72] the strip's sums, once the cells are done

    const int H = P.Fh * P.stride, W = P.Fw * P.stride;
    const int strip_row = blockIdx.y * (kCfBlock / kWave) + wv;
    const int x0 = blockIdx.x * kCfTileW, y0 = strip_row * kCfStripH;
    if (y0 >= H) return;
    const int px = x0 + lane;
    float *const o = out + ((size_t)plane * H + y0) * W + px;
    auto zeros = [&]() {
        if (px < W) {
#pragma unroll
            for (int r = 0; r < kCfStripH; ++r)
                if (y0 + r < H) o[(size_t)r * W] = 0.0f;
        }
    };
    const size_t list = (size_t)plane * P.cap;
    // records beyond the list's end are never used: the first fetch only may not wait for the length
    int4 b = lane < P.cap ? ws.pif_b[list + lane] : make_int4(0, 0, 0, 0);
    float4 a = lane < P.cap ? ws.pif_a[list + lane] : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    const int m = min(pif_count[plane], P.cap);
    int cnt = 0;
    for (int j0 = 0; j0 < m; j0 += kWave) {
        const int j = j0 + lane;
        if (j0 > 0 && j < m) {
            b = ws.pif_b[list + j];
            a = ws.pif_a[list + j];
        }
        bool meets = false;
        if (j < m) meets = b.x + b.w >= x0 && b.x - b.w < x0 + kCfTileW && b.y + b.w >= y0 && b.y - b.w < y0 + kCfStripH;
        const unsigned long long mask = __ballot(meets);
        if (meets) {
            const int at = cnt + __popcll(mask & ((1ull << lane) - 1ull));
            s_a[at] = a;
            s_b[at] = b;
        }
        cnt += __popcll(mask);
    }
    if (cnt == 0) {
        zeros();
        return;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");   // the records above are read by the other lanes below
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");

    const int lx = lane & 7, ly = lane >> 3;
    const int gx = x0 + lx, py = y0 + ly;     // this lane's pixel of group g is (gx + 8 g, py)
    const float pyf = (float)py;
    float pxf[kCfGroups], f[kCfGroups];
#pragma unroll
    for (int g = 0; g < kCfGroups; ++g) {
        pxf[g] = (float)(gx + 8 * g);
        f[g] = 0.0f;
    }
    int4 bn = s_b[0];
    float4 an = s_a[0];
    for (int j = 0; j < cnt; ++j) {
        // one record for all lanes: kept in scalar registers, the next one is on its way meanwhile
        const int bx = __builtin_amdgcn_readfirstlane(bn.x), by = __builtin_amdgcn_readfirstlane(bn.y);
        const int bw = __builtin_amdgcn_readfirstlane(bn.w);
        const float aX = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(an.x)));
        const float aY = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(an.y)));
        const float az = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(an.z)));
        const float ac = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(an.w)));
        const int jn = min(j + 1, cnt - 1);
        bn = s_b[jn];
        an = s_a[jn];
        const int xlo = bx - bw;
        const unsigned span = 2u * (unsigned)bw;
        const bool in_y = (unsigned)(py - (by - bw)) <= span;           // |py - yr| <= w
        const float dy = pyf - aY;
        const float dy2 = dy * dy;
#pragma unroll
        for (int g = 0; g < kCfGroups; ++g) {
            if (in_y && (unsigned)(gx + 8 * g - xlo) <= span) {         // |px - xr| <= w; often for no lane at all
                const float dx = pxf[g] - aX;
                const float dx2 = dx * dx;
                const float d2 = dx2 + dy2;
                f[g] = f[g] + ac * cf_expneg_window(d2 * az);
            }
        }
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");   // the records have been read: their place takes the sums
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int g = 0; g < kCfGroups; ++g) tile[ly * kCfTilePitch + 8 * g + lx] = f[g];
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
    if (px < W) {
#pragma unroll
        for (int r = 0; r < kCfStripH; ++r)
            if (y0 + r < H) o[(size_t)r * W] = tile[r * kCfTilePitch + lane];
    }
}

// ---- host side ---------------------------------------------------------------------------------------------------
// A workgroup may use up to 160 KB of LDS on this device; beyond 64 KB the kernel has to be told.
template <typename Kern>
static hipError_t allow_lds(Kern kern, size_t bytes)
{
    if (bytes <= 64 * 1024) return hipSuccess;
    return hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, 152 * 1024);
}

static CFParams cf_params(const hp_cf_params &prm, int Fh, int Fw, int K, int L, int cap, int acap, int pcap)
{
    CFParams P;
    P.pif_thr = prm.pif_thr;
    P.paf_thr = prm.paf_thr;
    P.seed_thr = prm.seed_thr;
    P.grow_thr = prm.grow_thr;
    P.rev_tol = prm.rev_tol;
    P.min_parts = prm.min_parts;
    P.stride = prm.stride;
    P.Fh = Fh;
    P.Fw = Fw;
    P.K = K;
    P.L = L;
    P.cap = cap;
    P.acap = acap;
    P.pcap = pcap;
    return P;
}

hipError_t launch_cf_pif(const float *pif, int N, int Fh, int Fw, int K, const hp_cf_params &prm, int cap, int32_t *cell,
                         float *val, int32_t *count, void *workspace, int L, int acap, int32_t *status, hipStream_t s)
{
    const CFParams P = cf_params(prm, Fh, Fw, K, L, cap, acap, 0);
    const CFWork ws = cf_layout(workspace, N, K, L, cap, acap);
    HP_KERNEL(k_cf_pif, dim3(K, N), dim3(kCfBlock), (sizeof(float4) * 2 + sizeof(int)) * (size_t)cap, s, pif, P, ws, cell, val, count, status);
    return hipGetLastError();
}

static CFLimbs cf_limbs(const LimbTable &T, int L)
{
    CFLimbs limbs = {};
    for (int l = 0; l < L; ++l) {
        limbs.a[l] = (uint8_t)T.a[l];
        limbs.b[l] = (uint8_t)T.b[l];
    }
    return limbs;
}

hipError_t launch_cf_paf(const float *paf, int N, int Fh, int Fw, const LimbTable &T, int K, int L,
                         const hp_cf_params &prm, const hp_cf_lists &lists, void *workspace, int32_t *status, hipStream_t s)
{
    const CFParams P = cf_params(prm, Fh, Fw, K, L, lists.cap, lists.acap, 0);
    const CFWork ws = cf_layout(workspace, N, K, L, lists.cap, lists.acap);
    // the limb workgroups hold two parts' cell lists, the seed workgroups the keys they sort
    const bool staged = lists.acap <= kCfPafStage;
    const size_t held = sizeof(float4) * 4 * (size_t)lists.cap + (staged ? (2 * sizeof(float4) + sizeof(int)) * (size_t)lists.acap : 0);
    const size_t lds = std::max(held, sizeof(uint64_t) * (size_t)next_pow2(K * lists.cap));
    if (staged) {
        if (hipError_t e = allow_lds(k_cf_paf<true>, lds)) return e;
        HP_KERNEL(k_cf_paf<true>, dim3(L + 1, N), dim3(kCfBlock), lds, s, paf, P, ws, cf_limbs(T, L), lists.pif_count,
                  lists.pif_val, lists.paf_cell, lists.paf_f1, lists.paf_f2, lists.paf_count, status);
    } else {
        if (hipError_t e = allow_lds(k_cf_paf<false>, lds)) return e;
        HP_KERNEL(k_cf_paf<false>, dim3(L + 1, N), dim3(kCfBlock), lds, s, paf, P, ws, cf_limbs(T, L), lists.pif_count,
                  lists.pif_val, lists.paf_cell, lists.paf_f1, lists.paf_f2, lists.paf_count, status);
    }
    return hipGetLastError();
}

hipError_t launch_cf_link(const float *pif, int N, int Fh, int Fw, const LimbTable &T, int K, int L, const hp_cf_params &prm,
                          const hp_cf_lists &lists, void *workspace, hipStream_t s)
{
    const CFParams P = cf_params(prm, Fh, Fw, K, L, lists.cap, lists.acap, 0);
    const CFWork ws = cf_layout(workspace, N, K, L, lists.cap, lists.acap);
    const size_t lds = sizeof(float4) * 2 * (size_t)std::min(lists.acap, kCfLinkStage);
    HP_KERNEL(k_cf_link, dim3(L, N, kCfLinkSlices), dim3(kCfBlock), lds, s, pif, P, ws, cf_limbs(T, L), lists.paf_count);
    return hipGetLastError();
}

// LDS the persons kernel may use: the device allows 160 KB a workgroup; 144 KB leaves room for the static arrays.
constexpr size_t kCfGrowLds = 144 * 1024;

hipError_t launch_cf_grow(int N, int Fh, int Fw, const LimbTable &T, int K, int L, const hp_cf_params &prm,
                          const hp_cf_lists &lists, const hp_cf_poses &poses, void *workspace, int32_t *status, hipStream_t s)
{
    const CFParams P = cf_params(prm, Fh, Fw, K, L, lists.cap, lists.acap, poses.cap);
    const CFWork ws = cf_layout(workspace, N, K, L, lists.cap, lists.acap);
    const size_t persons = sizeof(float4) * ((size_t)poses.cap * K + (poses.cap + 1) / 2);   // joints, part counts, scores
    // search records kept in LDS: all of them when the lists' capacity fits, else the limbs that fit in table order
    const size_t room = (kCfGrowLds - persons) / (4 * sizeof(float4));
    const int lds_cells = (int)std::min(room, (size_t)L * lists.acap);
    const size_t lds = persons + 4 * sizeof(float4) * (size_t)lds_cells;
    if (hipError_t e = allow_lds(k_cf_grow, lds)) return e;
    HP_KERNEL(k_cf_grow, dim3(N), dim3(kCfGrowBlock), lds, s, P, ws, cf_limbs(T, L), lds_cells, lists.paf_count, poses.xyv,
              poses.nparts, poses.score, poses.count, status);
    return hipGetLastError();
}

hipError_t launch_cf_field(int N, int Fh, int Fw, int K, const hp_cf_params &prm, int cap, const int32_t *count, float *out,
                           void *workspace, hipStream_t s)
{
    const CFParams P = cf_params(prm, Fh, Fw, K, 0, cap, 0, 0);
    const CFWork ws = cf_layout(workspace, N, K, 0, cap, 0);
    const int H = Fh * prm.stride, W = Fw * prm.stride;
    const dim3 grid((W + kCfTileW - 1) / kCfTileW, (H + kCfTileH - 1) / kCfTileH, N * K);
    const size_t lds = sizeof(float4) * (size_t)cf_field_wave_f4(cap) * (kCfBlock / kWave);
    if (hipError_t e = allow_lds(k_cf_field, lds)) return e;
    HP_KERNEL(k_cf_field, grid, dim3(kCfBlock), lds, s, P, ws, count, out);
    return hipGetLastError();
}

}  // namespace hp

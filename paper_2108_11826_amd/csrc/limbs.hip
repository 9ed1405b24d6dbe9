// Limb scoring (PAF line integral over every candidate pair) and per-limb greedy
// matching: the PAF-family part (Section 2.3) of the post-processing operator of the
// paper's inference engine (Section 2.2.1, operator 4).  Arithmetic as stated at
// hp_score_limbs / hp_assemble in hp.h.
#include "hp_dev.h"

namespace hp {

// How many PAF samples the scorer fetches together.  A pair dies at its (S - need + 1)-th bad
// sample, three with the usual parameters, and a wavefront keeps going while any lane lives.
// Few pairs (latency matters): 4 samples, then the rest 8 at a time.  Many pairs of mostly
// unrelated peaks (throughput matters): 3, then one at a time for two steps (after five
// samples almost every wavefront has no pair left), then the rest.
struct ChunksLatency { static constexpr int first = 4, singles = 0; };
struct ChunksThroughput { static constexpr int first = 3, singles = 2; };
constexpr int kChunkRest = 8;
constexpr int kRankSort = 256; // lists up to this length are ordered by counting ranks through LDS

// Sample positions along a candidate, t_k = k / (S - 1), divided on the host (the same
// correctly rounded fp32 quotient the device would form) and passed by value.
struct SampleT {
    float t[HP_MAX_SAMPLES];
};

// The two PAF components of limb l at hi-res pixel (sy, sx), recomputed from the lo-res planes
// with the upsampling arithmetic (horizontal pass on the two source rows, then vertical); the
// node indices and weights are shared by the two components.
template <typename T>
__device__ __forceinline__ void paf_from_lo(const T *__restrict__ lx, const T *__restrict__ ly, int h, int w, int sy,
                                            int sx, float &vx, float &vy)
{
    int x0, x1, y0, y1;
    float f, g;
    axis8(sx, w, x0, x1, f);
    axis8(sy, h, y0, y1, g);
    const unsigned r0 = (unsigned)__mul24(y0, w), r1 = (unsigned)__mul24(y1, w);
    const unsigned o00 = r0 + x0, o01 = r0 + x1, o10 = r1 + x0, o11 = r1 + x1;
    const float f1 = 1.0f - f, g1 = 1.0f - g;
    const float ax = ld(lx + o00), bx = ld(lx + o01), cx = ld(lx + o10), dx = ld(lx + o11);
    const float ay = ld(ly + o00), by = ld(ly + o01), cy = ld(ly + o10), dy = ld(ly + o11);
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
    for (; k0 < S && bad <= max_bad; k0 += kChunkRest)
        score_chunk<T, FROM_HI, kChunkRest>(k0, S, st, fdx, fdy, fx0, fy0, ux, uy, paf_thr, max_bad, H, W, h, w, hx, hy,
                                            lx, ly, acc, bad);
    if (bad > max_bad) return false;
    score = acc / (float)S;
    return score > 0.0f;
}

// grid = (chunks, N*L).  Each thread owns candidate pairs p = i * nB + j of its (image, limb),
// strided by the whole row of workgroups; a score is never reduced across lanes, so the
// summation order is the sample order.  Accepted pairs are appended unordered, tagged with
// (i << 16 | j); the matching kernel orders them.  A pair is dropped as soon as it cannot reach
// `need` valid samples any more: most pairs of unrelated peaks die in the first chunk.
template <typename T, bool FROM_HI>
__global__ __launch_bounds__(kBlock) void k_score(const float *__restrict__ paf_hi, const T *__restrict__ paf_lo,
                                                  int h, int w, LimbTable tab, SampleT st, int K, int L, int S,
                                                  float paf_thr, int need,
                                                  const int32_t *__restrict__ pcounts,
                                                  const int32_t *__restrict__ px, const int32_t *__restrict__ py,
                                                  int cap, int32_t *ccounts, uint64_t *cstage, int ccap, int ccap2)
{
    const int nl = blockIdx.y;
    const int n = nl / L, l = nl - n * L;
    const int a = tab.a[l], b = tab.b[l];
    const int nA = max(min(pcounts[n * K + a], cap), 0), nB = max(min(pcounts[n * K + b], cap), 0);
    const int P = nA * nB;
    const int stride = gridDim.x * kBlock;
    int p = blockIdx.x * kBlock + threadIdx.x;
    if (p - (int)threadIdx.x >= P) return;

    const int32_t *xa = px + (size_t)(n * K + a) * cap, *ya = py + (size_t)(n * K + a) * cap;
    const int32_t *xb = px + (size_t)(n * K + b) * cap, *yb = py + (size_t)(n * K + b) * cap;
    const int H = 8 * h, W = 8 * w;
    const float *hx = FROM_HI ? paf_hi + ((size_t)n * 2 * L + 2 * l) * (size_t)H * W : nullptr;
    const float *hy = FROM_HI ? hx + (size_t)H * W : nullptr;
    const T *lx = FROM_HI ? nullptr : paf_lo + ((size_t)n * 2 * L + 2 * l) * (size_t)h * w;
    const T *ly = FROM_HI ? nullptr : lx + (size_t)h * w;
    const int max_bad = S - need;
    const float inv_nB = 1.0f / (float)nB;

    for (; p < P; p += stride) {
        // i = p / nB through the reciprocal, then made exact
        int i = (int)((float)p * inv_nB);
        int j = p - i * nB;
        while (j < 0) { --i; j += nB; }
        while (j >= nB) { ++i; j -= nB; }
        float score;
        if (score_pair<T, FROM_HI, ChunksThroughput>(xa[i], ya[i], xb[j], yb[j], S, st, paf_thr, max_bad, H, W, h, w, hx, hy, lx, ly,
                                   score)) {
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
                        hipStream_t s)
{
    // enough workgroups per (image, limb) to spread cap^2 pairs, few enough that idle ones are cheap
    long long pairs = (long long)pk.cap * pk.cap;
    int chunks = (int)((pairs + kBlock * 16 - 1) / (kBlock * 16));
    if (chunks < 4) chunks = 4;
    if (chunks > 128) chunks = 128;
    dim3 grid(chunks, N * L), block(kBlock);
    SampleT st;
    for (int k = 0; k < HP_MAX_SAMPLES; ++k) st.t[k] = (float)k / (float)(prm.n_samples - 1);
    if (paf_hi)
        hipLaunchKernelGGL((k_score<float, true>), grid, block, 0, s, paf_hi, (const float *)nullptr, h, w, T, st, K, L,
                           prm.n_samples, prm.paf_thr, need, pk.count, pk.x, pk.y, pk.cap, ccounts, cstage, ccap,
                           ccap2);
    else if (dt == HP_F16)
        hipLaunchKernelGGL((k_score<__half, false>), grid, block, 0, s, (const float *)nullptr,
                           (const __half *)paf_lo, h, w, T, st, K, L, prm.n_samples, prm.paf_thr, need, pk.count, pk.x,
                           pk.y, pk.cap, ccounts, cstage, ccap, ccap2);
    else
        hipLaunchKernelGGL((k_score<float, false>), grid, block, 0, s, (const float *)nullptr,
                           (const float *)paf_lo, h, w, T, st, K, L, prm.n_samples, prm.paf_thr, need, pk.count, pk.x,
                           pk.y, pk.cap, ccounts, cstage, ccap, ccap2);
    return hipGetLastError();
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
    if (cnt > ccap && threadIdx.x == 0) atomicOr(status, (int)HP_STATUS_CAND_OVERFLOW);
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
    if (c <= kWave) {
        // One wavefront, one candidate per lane.  The lowest-ranked candidate still alive is
        // accepted; every candidate sharing a peak with it dies.  One step per connection.
        if (threadIdx.x >= kWave) return;
        const int lane = threadIdx.x;
        const uint64_t e = lane < c ? keys[lane] : ~0ull;
        const int i = (int)((uint32_t)e >> 16), j = (int)((uint32_t)e & 0xffffu);
        unsigned long long alive = __ballot(lane < c && i < nA && j < nB);
        int m = 0;
        while (alive) {
            const int r = __ffsll((long long)alive) - 1;
            const int ir = __builtin_amdgcn_readlane(i, r), jr = __builtin_amdgcn_readlane(j, r);
            if (lane == r) {
                mi[mo + m] = i;
                mj[mo + m] = j;
                ms[mo + m] = __uint_as_float(~(uint32_t)(e >> 32));
            }
            ++m;
            alive &= ~__ballot(i == ir || j == jr);
        }
        if (lane == 0) mcounts[nl] = m;
        return;
    }

    for (int t = threadIdx.x; t < (nA + 31) / 32; t += kBlock) usedA[t] = 0;
    for (int t = threadIdx.x; t < (nB + 31) / 32; t += kBlock) usedB[t] = 0;
    __syncthreads();
    if (threadIdx.x == 0) {
        const int limit = min(min(nA, nB), mcap);
        int m = 0;
        for (int t = 0; t < c && m < limit; ++t) {
            uint64_t e = keys[t];
            uint32_t ij = (uint32_t)e;
            uint32_t i = ij >> 16, j = ij & 0xffffu;
            if (i >= (uint32_t)nA || j >= (uint32_t)nB) continue;   // only possible for foreign candidate lists
            if ((usedA[i >> 5] >> (i & 31)) & 1u) continue;
            if ((usedB[j >> 5] >> (j & 31)) & 1u) continue;
            usedA[i >> 5] |= 1u << (i & 31);
            usedB[j >> 5] |= 1u << (j & 31);
            mi[mo + m] = (int32_t)i;
            mj[mo + m] = (int32_t)j;
            ms[mo + m] = __uint_as_float(~(uint32_t)(e >> 32));
            ++m;
        }
        mcounts[nl] = m;
    }
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

template <typename T, bool FROM_HI>
__global__ __launch_bounds__(kSmallBlock) void k_limb_small(
    const float *__restrict__ paf_hi, const T *__restrict__ paf_lo, int h, int w, LimbTable tab, SampleT st, int K,
    int L, int NL, int S, float paf_thr, int need, const int32_t *__restrict__ peak_ctr,
    const uint64_t *__restrict__ peak_stage, int cap, int cap2, int32_t *pcounts, int32_t *px, int32_t *py, float *ps,
    int32_t *ccounts, int32_t *ci, int32_t *cj, float *cs, int ccap, int32_t *mcounts, int32_t *mi, int32_t *mj,
    float *ms, int mcap, int32_t *status)
{
    __shared__ uint64_t sk[kSmallCands];
    __shared__ int lxy[4][kSmallPeaks];          // xA, yA, xB, yB in rank order
    __shared__ int lds_cnt;
    __shared__ uint32_t usedA[kSmallPeaks / 32], usedB[kSmallPeaks / 32];
    const int tid = threadIdx.x;
    const int H = 8 * h, W = 8 * w;

    const int nl = blockIdx.x;
    const int n = nl / L, l = nl - n * L;
    const int a = tab.a[l], b = tab.b[l];
    const int pa = n * K + a, pb = n * K + b;
    const int nA = max(min(peak_ctr[pa * kCtrStride], cap), 0), nB = max(min(peak_ctr[pb * kCtrStride], cap), 0);

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
        if (tid == 0) lds_cnt = 0;
        if (publish && t == 0) {
            const int raw = peak_ctr[plane * kCtrStride];
            pcounts[plane] = raw;
            if (raw > cap) atomicOr(status, (int)HP_STATUS_PEAK_OVERFLOW);
        }
        __syncthreads();
        if (mine) {
            const uint64_t *skh = sk + half * kSmallPeaks;
            int r = 0;
            for (int u = 0; u < cnt; ++u) r += skh[u] < e;
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
                int r = 0;
                for (int u = 0; u < cnt; ++u) r += sk[u] < e;
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
        const float *hx = FROM_HI ? paf_hi + ((size_t)n * 2 * L + 2 * l) * (size_t)H * W : nullptr;
        const float *hy = FROM_HI ? hx + (size_t)H * W : nullptr;
        const T *lx = FROM_HI ? nullptr : paf_lo + ((size_t)n * 2 * L + 2 * l) * (size_t)h * w;
        const T *ly = FROM_HI ? nullptr : lx + (size_t)h * w;
        const int P = nA * nB, max_bad = S - need;
        const float inv_nB = 1.0f / (float)nB;
        for (int p = tid; p < P; p += kSmallBlock) {
            int i = (int)((float)p * inv_nB);
            int j = p - i * nB;
            while (j < 0) { --i; j += nB; }
            while (j >= nB) { ++i; j -= nB; }
            float score;
            if (score_pair<T, FROM_HI, ChunksLatency>(lxy[0][i], lxy[1][i], lxy[2][j], lxy[3][j], S, st, paf_thr, max_bad, H, W, h, w, hx,
                                       hy, lx, ly, score)) {
                const int slot = atomicAdd(&lds_cnt, 1);
                if (slot < kSmallCands)
                    sk[slot] = ((uint64_t)(((uint32_t)i << 16) | (uint32_t)j) << 32) | (uint64_t)__float_as_uint(score);
            }
        }
        __syncthreads();
    }

    const int cnt = lds_cnt;
    const int c = min(cnt, min(ccap, kSmallCands));
    if (tid == 0) {
        ccounts[nl] = cnt;
        if (cnt > ccap) atomicOr(status, (int)HP_STATUS_CAND_OVERFLOW);
    }
    // candidates in (i, j) order
    const uint64_t e = tid < c ? sk[tid] : ~0ull;
    const size_t co = (size_t)nl * ccap;
    if (tid < c) {
        int r = 0;
        for (int u = 0; u < c; ++u) r += sk[u] < e;
        ci[co + r] = (int32_t)(e >> 48);
        cj[co + r] = (int32_t)((e >> 32) & 0xffffu);
        cs[co + r] = __uint_as_float((uint32_t)e);
    }
    __syncthreads();
    // matching order: (~score bits) << 32 | (i << 16 | j), ascending
    const uint64_t key = tid < c ? ((uint64_t)(~(uint32_t)e) << 32) | (e >> 32) : ~0ull;
    if (tid < c) sk[tid] = key;
    if (tid < kSmallPeaks / 32) usedA[tid] = usedB[tid] = 0;
    __syncthreads();
    int r2 = 0;
    if (tid < c)
        for (int u = 0; u < c; ++u) r2 += sk[u] < key;
    __syncthreads();
    if (tid < c) sk[r2] = key;
    __syncthreads();

    const size_t mo = (size_t)nl * mcap;
    if (tid >= kWave) return;
    if (c <= kWave) {
        // one candidate per lane: the lowest-ranked one still alive is accepted, every candidate
        // sharing a peak with it dies; one step per connection
        const uint64_t k = tid < c ? sk[tid] : ~0ull;
        const int i = (int)((uint32_t)k >> 16), j = (int)((uint32_t)k & 0xffffu);
        unsigned long long alive = __ballot(tid < c);
        int m = 0;
        while (alive) {
            const int r = __ffsll((long long)alive) - 1;
            const int ir = __builtin_amdgcn_readlane(i, r), jr = __builtin_amdgcn_readlane(j, r);
            if (tid == r) {
                mi[mo + m] = i;
                mj[mo + m] = j;
                ms[mo + m] = __uint_as_float(~(uint32_t)(k >> 32));
            }
            ++m;
            alive &= ~__ballot(i == ir || j == jr);
        }
        if (tid == 0) mcounts[nl] = m;
    } else if (tid == 0) {
        const int limit = min(min(nA, nB), mcap);
        int m = 0;
        for (int t = 0; t < c && m < limit; ++t) {
            const uint64_t k = sk[t];
            const uint32_t i = (uint32_t)k >> 16, j = (uint32_t)k & 0xffffu;
            if ((usedA[i >> 5] >> (i & 31)) & 1u) continue;
            if ((usedB[j >> 5] >> (j & 31)) & 1u) continue;
            usedA[i >> 5] |= 1u << (i & 31);
            usedB[j >> 5] |= 1u << (j & 31);
            mi[mo + m] = (int32_t)i;
            mj[mo + m] = (int32_t)j;
            ms[mo + m] = __uint_as_float(~(uint32_t)(k >> 32));
            ++m;
        }
        mcounts[nl] = m;
    }
}

bool limb_small_applies(int cap, int ccap) { return cap <= kSmallPeaks && ccap <= kSmallCands; }

hipError_t launch_limb_small(const float *paf_hi, const void *paf_lo, hp_dtype dt, int N, int h, int w,
                             const LimbTable &T, int K, int L, const hp_params &prm, int need,
                             const int32_t *peak_ctr, const uint64_t *peak_stage, int cap2, const hp_peaks &pk,
                             const hp_pairs &cands, const hp_pairs &conns, int32_t *status, hipStream_t s)
{
    SampleT st;
    for (int k = 0; k < HP_MAX_SAMPLES; ++k) st.t[k] = (float)k / (float)(prm.n_samples - 1);
    dim3 grid(N * L), block(kSmallBlock);
#define HP_LIMB_SMALL_ARGS(LO)                                                                                        \
    paf_hi, LO, h, w, T, st, K, L, N *L, prm.n_samples, prm.paf_thr, need, peak_ctr, peak_stage, pk.cap, cap2,        \
        pk.count, pk.x, pk.y, pk.score, cands.count, cands.i, cands.j, cands.score, cands.cap, conns.count, conns.i,   \
        conns.j, conns.score, conns.cap, status
    if (paf_hi)
        hipLaunchKernelGGL((k_limb_small<float, true>), grid, block, 0, s, HP_LIMB_SMALL_ARGS((const float *)nullptr));
    else if (dt == HP_F16)
        hipLaunchKernelGGL((k_limb_small<__half, false>), grid, block, 0, s, HP_LIMB_SMALL_ARGS((const __half *)paf_lo));
    else
        hipLaunchKernelGGL((k_limb_small<float, false>), grid, block, 0, s, HP_LIMB_SMALL_ARGS((const float *)paf_lo));
#undef HP_LIMB_SMALL_ARGS
    return hipGetLastError();
}

hipError_t launch_match(int mode, const LimbTable &T, int N, int K, int L, const hp_peaks &pk,
                        int32_t *cctr, uint64_t *cstage, int ccap2, const hp_pairs &cands,
                        const hp_pairs &conns, int32_t *status, hipStream_t s)
{
    dim3 grid(N * L), block(kBlock);
    if (mode == 0)
        hipLaunchKernelGGL((k_match<0>), grid, block, 0, s, T, K, L, pk.count, pk.cap, cctr, cstage, ccap2, cands.count,
                           cands.i, cands.j, cands.score, cands.cap, (int32_t *)nullptr, (int32_t *)nullptr,
                           (int32_t *)nullptr, (float *)nullptr, 0, status);
    else if (mode == 1)
        hipLaunchKernelGGL((k_match<1>), grid, block, 0, s, T, K, L, pk.count, pk.cap, cctr, cstage, ccap2, cands.count,
                           cands.i, cands.j, cands.score, cands.cap, conns.count, conns.i, conns.j, conns.score,
                           conns.cap, status);
    else
        hipLaunchKernelGGL((k_match<2>), grid, block, 0, s, T, K, L, pk.count, pk.cap, cctr, cstage, ccap2, cands.count,
                           cands.i, cands.j, cands.score, cands.cap, conns.count, conns.i, conns.j, conns.score,
                           conns.cap, status);
    return hipGetLastError();
}

}  // namespace hp

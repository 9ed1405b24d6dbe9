// Post-processing of the pose-proposal family (Section 2.3 names it as the engine's second algorithm class):
// detection scores and boxes on a coarse grid, box suppression per part, and a walk over the limb tree from each
// root detection.  The rules (D1-D5) are written at hp_pp_decode in hp.h; every float operation below is one of
// theirs, in their order.
//
// The data are tiny (a 12 x 12 or 24 x 24 grid, some twenty parts), so the kernels are organised around latency,
// not bandwidth: k_pp_detect gives one workgroup to an (image, part) pair, sorts the candidate cells by (score
// descending, cell ascending) in LDS and suppresses greedily, one kept box per step with all threads testing the
// remaining ones against it; k_pp_parse gives one wavefront to an image, keeps the detection lists it walks in LDS,
// and for each person searches up to eight limbs whose parents are already attached side by side, eight lanes per
// limb scanning the child part's detections, the best connection value (earliest on ties) found by a maximum over
// the eight lanes (one memory round trip per tree level instead of one per limb: 78 -> 34 us at 8 x 12 x 12).
#include <string.h>

#include "hp_dev.h"

namespace hp {

constexpr int kPPMaxCells = HP_PP_MAX_CELLS;

struct PPParams {
    float det_thr, nms_thr, edge_thr, img_w, img_h;
    int min_parts, Gh, Gw, Nh, Nw, K, L, cap, pcap;
};

__device__ __forceinline__ float box_iou(const float4 a, const float4 b)
{
    const float iw = fminf(a.z, b.z) - fmaxf(a.x, b.x);
    const float ih = fminf(a.w, b.w) - fmaxf(a.y, b.y);
    const float inter = (iw > 0.0f && ih > 0.0f) ? iw * ih : 0.0f;
    const float ua = (a.z - a.x) * (a.w - a.y);
    const float ub = (b.z - b.x) * (b.w - b.y);
    const float den = (ua + ub) - inter;
    return den > 0.0f ? inter / den : 0.0f;
}

__global__ __launch_bounds__(kBlock) void k_pp_detect(const float *__restrict__ resp, const float *__restrict__ conf,
                                                      const float *__restrict__ box, PPParams P,
                                                      int32_t *__restrict__ out_cell, float *__restrict__ out_score,
                                                      float *__restrict__ out_box, int32_t *__restrict__ out_count,
                                                      int32_t *__restrict__ status)
{
    __shared__ uint64_t s_key[kPPMaxCells];        // (inverted score order) << 32 | cell; all ones = no candidate
    __shared__ float4 s_box[kPPMaxCells];          // corners of the sorted candidates
    __shared__ uint8_t s_gone[kPPMaxCells];        // suppressed by a kept box
    __shared__ int s_kept[kPPMaxCells];            // sorted positions of the kept boxes, in order
    __shared__ int s_ncand, s_nkept;

    const int k = blockIdx.x, n = blockIdx.y, tid = threadIdx.x;
    const int cells = P.Gh * P.Gw;
    const size_t plane = ((size_t)n * P.K + k) * cells;
    const float *r = resp + plane, *c = conf + plane, *b = box + plane * 4;
    int n2 = 1;
    while (n2 < cells) n2 <<= 1;

    if (tid == 0) {
        s_ncand = 0;
        s_nkept = 0;
    }
    __syncthreads();
    for (int i = tid; i < n2; i += kBlock) {
        uint64_t key = ~0ull;
        if (i < cells) {
            const float s = r[i] * c[i];                       // D1
            if (s > P.det_thr) {
                key = ((uint64_t)(~float_order(s)) << 32) | (uint32_t)i;
                atomicAdd(&s_ncand, 1);
            }
        }
        s_key[i] = key;
        s_gone[i] = 0;
    }
    __syncthreads();
    block_bitonic_sort(s_key, n2);                             // (score descending, cell ascending); ends with a barrier
    const int ncand = s_ncand;

    const float cell_w = P.img_w / (float)P.Gw, cell_h = P.img_h / (float)P.Gh;
    for (int t = tid; t < ncand; t += kBlock) {                // D2
        const int cell = (int)(uint32_t)s_key[t], gy = cell / P.Gw, gx = cell - gy * P.Gw;
        const float cx = ((float)gx + b[0 * cells + cell]) * cell_w;
        const float cy = ((float)gy + b[1 * cells + cell]) * cell_h;
        const float w = b[2 * cells + cell] * P.img_w, h = b[3 * cells + cell] * P.img_h;
        s_box[t] = make_float4(cx - 0.5f * w, cy - 0.5f * h, cx + 0.5f * w, cy + 0.5f * h);
    }
    __syncthreads();

    for (int t = 0; t < ncand; ++t) {                          // D3: a box still standing is kept and suppresses later ones
        if (!s_gone[t]) {                                      // the same for every thread
            if (tid == 0) s_kept[s_nkept++] = t;
            const float4 kb = s_box[t];
            for (int u = t + 1 + tid; u < ncand; u += kBlock)
                if (!s_gone[u] && box_iou(kb, s_box[u]) > P.nms_thr) s_gone[u] = 1;
        }
        __syncthreads();
    }

    const int nk = s_nkept;
    const size_t list = ((size_t)n * P.K + k) * P.cap;
    for (int q = tid; q < min(nk, P.cap); q += kBlock) {
        const int t = s_kept[q];
        out_cell[list + q] = (int)(uint32_t)s_key[t];
        out_score[list + q] = float_unorder(~(uint32_t)(s_key[t] >> 32));
        const float4 bb = s_box[t];
        float *ob = out_box + (list + q) * 4;
        ob[0] = bb.x;
        ob[1] = bb.y;
        ob[2] = bb.z;
        ob[3] = bb.w;
    }
    if (tid == 0) {
        out_count[(size_t)n * P.K + k] = nk;
        if (nk > P.cap) atomicOr(status, HP_STATUS_PEAK_OVERFLOW);
    }
}

// Per-limb tables passed by value and copied to LDS through constant indices.  The limbs of one person are walked in
// batches of up to eight consecutive limbs whose parents were all attached before the batch (no limb's parent is the
// child of another limb of its batch), so that the limbs of a batch can be searched side by side.
constexpr int kPPBatch = 8, kPPGroup = kWave / kPPBatch;
struct PPLimbs {
    uint8_t a[HP_MAX_LIMBS], b[HP_MAX_LIMBS];
    uint8_t batch_end[HP_MAX_LIMBS];   // one past the last limb of batch i
    int n_batches;
};

__global__ __launch_bounds__(kWave) void k_pp_parse(const int32_t *__restrict__ det_cell, const float *__restrict__ det_score,
                                                    const int32_t *__restrict__ det_count, const float *__restrict__ edge,
                                                    PPLimbs limbs, PPParams P, int32_t *__restrict__ slots,
                                                    int32_t *__restrict__ nparts, float *__restrict__ pscore,
                                                    int32_t *__restrict__ pcount, int32_t *__restrict__ status)
{
    extern __shared__ int32_t s_dyn[];
    int32_t *s_cell = s_dyn;                              // [K][cap] cells of the kept detections
    float *s_score = (float *)(s_dyn + P.K * P.cap);      // [K][cap]
    uint32_t *s_used = (uint32_t *)(s_dyn + 2 * P.K * P.cap);   // [K][ceil(cap / 32)] taken by an earlier person
    __shared__ uint8_t s_a[HP_MAX_LIMBS], s_b[HP_MAX_LIMBS], s_end[HP_MAX_LIMBS];
    __shared__ int s_count[HP_MAX_PARTS], s_slot[HP_MAX_PARTS];
    __shared__ uint64_t s_found[kPPBatch];   // per limb of the batch: (value order) << 32 | (0x7FFFFFFF - rank), 0 = nothing

    const int n = blockIdx.x, lane = threadIdx.x;
    const int cells = P.Gh * P.Gw, rh = (P.Nh - 1) >> 1, rw = (P.Nw - 1) >> 1;
    const int used_words = (P.cap + 31) >> 5;
    if (lane == 0) {
#pragma unroll
        for (int i = 0; i < HP_MAX_LIMBS; ++i) {
            s_a[i] = limbs.a[i];
            s_b[i] = limbs.b[i];
            s_end[i] = limbs.batch_end[i];
        }
    }
    for (int k = lane; k < P.K; k += kWave) s_count[k] = min(det_count[(size_t)n * P.K + k], P.cap);
    for (int i = lane; i < P.K * used_words; i += kWave) s_used[i] = 0;
    __syncthreads();
    for (int k = 0; k < P.K; ++k)
        for (int q = lane; q < s_count[k]; q += kWave) {
            s_cell[k * P.cap + q] = det_cell[((size_t)n * P.K + k) * P.cap + q];
            s_score[k * P.cap + q] = det_score[((size_t)n * P.K + k) * P.cap + q];
        }
    __syncthreads();

    const float *e = edge + (size_t)n * P.L * P.Nh * P.Nw * cells;
    const int root = s_a[0];
    int np = 0;
    for (int r = 0; r < s_count[root]; ++r) {                 // D4: one person per kept root detection, in order
        for (int k = lane; k < P.K; k += kWave) s_slot[k] = k == root ? r : -1;
        __syncthreads();
        float sc = s_score[root * P.cap + r];                 // D5
        int parts = 1;
        const int group = lane / kPPGroup, sub = lane % kPPGroup;   // eight lanes search one limb of the batch
        for (int bi = 0, l0 = 0; bi < limbs.n_batches; ++bi) {
            const int l1 = s_end[bi], l = l0 + group;
            uint64_t key = 0ull;
            if (l < l1) {
                const int a = s_a[l], b = s_b[l];
                const int sa = s_slot[a];
                if (sa >= 0) {
                    const int i = s_cell[a * P.cap + sa], iy = i / P.Gw, ix = i - iy * P.Gw;
                    // a lane scans its share of the child's detections; a strict comparison keeps the earliest of equals
                    float best_v = P.edge_thr;
                    int best_q = -1;
                    for (int q = sub; q < s_count[b]; q += kPPGroup) {
                        if ((s_used[b * used_words + (q >> 5)] >> (q & 31)) & 1u) continue;
                        const int j = s_cell[b * P.cap + q], jy = j / P.Gw, dy = jy - iy, dx = (j - jy * P.Gw) - ix;
                        if (dy < -rh || dy > rh || dx < -rw || dx > rw) continue;
                        const float v = e[((size_t)l * P.Nh * P.Nw + (size_t)(dy + rh) * P.Nw + (dx + rw)) * cells + i];
                        if (v > best_v) {
                            best_v = v;
                            best_q = q;
                        }
                    }
                    if (best_q >= 0) key = ((uint64_t)float_order(best_v) << 32) | (uint32_t)(0x7FFFFFFF - best_q);
                }
            }
            // maximum of (value, earliest rank) over the eight lanes of the group
#pragma unroll
            for (int off = kPPGroup / 2; off > 0; off >>= 1) {
                const uint64_t other = __shfl_xor(key, off);
                key = other > key ? other : key;
            }
            if (sub == 0) s_found[group] = key;
            __syncthreads();
            // the finds are applied in table order (the score is a sum in that order)
            for (int g = 0; g < l1 - l0; ++g) {
                const uint64_t found = s_found[g];
                if (found == 0ull) continue;                  // the same for every lane
                const int b = s_b[l0 + g], q = 0x7FFFFFFF - (int)(uint32_t)found;
                const float v = float_unorder((uint32_t)(found >> 32));
                if (lane == 0) {
                    s_slot[b] = q;
                    s_used[b * used_words + (q >> 5)] |= 1u << (q & 31);
                }
                sc = sc + v;
                sc = sc + s_score[b * P.cap + q];
                ++parts;
            }
            __syncthreads();
            l0 = l1;
        }
        if (parts >= P.min_parts) {
            if (np < P.pcap) {
                for (int k = lane; k < P.K; k += kWave) slots[((size_t)n * P.pcap + np) * P.K + k] = s_slot[k];
                if (lane == 0) {
                    nparts[(size_t)n * P.pcap + np] = parts;
                    pscore[(size_t)n * P.pcap + np] = sc;
                }
            }
            ++np;
        }
        __syncthreads();
    }
    if (lane == 0) {
        pcount[n] = np;
        if (np > P.pcap) atomicOr(status, HP_STATUS_POSE_OVERFLOW);
    }
}

__global__ void k_clear_status(int32_t *status) { *status = 0; }

static PPParams pp_params(int Gh, int Gw, int Nh, int Nw, int K, int L, const hp_pp_params &prm, int cap, int pcap)
{
    PPParams P;
    P.det_thr = prm.det_thr;
    P.nms_thr = prm.nms_thr;
    P.edge_thr = prm.edge_thr;
    P.img_w = prm.img_w;
    P.img_h = prm.img_h;
    P.min_parts = prm.min_parts;
    P.Gh = Gh;
    P.Gw = Gw;
    P.Nh = Nh;
    P.Nw = Nw;
    P.K = K;
    P.L = L;
    P.cap = cap;
    P.pcap = pcap;
    return P;
}

hipError_t launch_clear_status(int32_t *status, hipStream_t s)
{
    HP_KERNEL(k_clear_status, dim3(1), dim3(1), 0, s, status);
    return hipGetLastError();
}

hipError_t launch_pp_detect(const float *resp, const float *conf, const float *box, int N, int Gh, int Gw, int K,
                            const hp_pp_params &prm, const hp_pp_dets &dets, int32_t *status, hipStream_t s)
{
    const PPParams P = pp_params(Gh, Gw, 1, 1, K, 0, prm, dets.cap, 0);
    HP_KERNEL(k_pp_detect, dim3(K, N), dim3(kBlock), 0, s, resp, conf, box, P, dets.cell, dets.score, dets.box, dets.count,
              status);
    return hipGetLastError();
}

hipError_t launch_pp_parse(const float *edge, int N, int Gh, int Gw, int Nh, int Nw, const LimbTable &T, int K, int L,
                           const hp_pp_params &prm, const hp_pp_dets &dets, const hp_poses &poses, int32_t *status,
                           hipStream_t s)
{
    const PPParams P = pp_params(Gh, Gw, Nh, Nw, K, L, prm, dets.cap, poses.cap);
    PPLimbs limbs = {};
    bool child_in_batch[HP_MAX_PARTS] = {false};
    int in_batch = 0;
    for (int l = 0; l < L; ++l) {
        limbs.a[l] = (uint8_t)T.a[l];
        limbs.b[l] = (uint8_t)T.b[l];
        if (in_batch == kPPBatch || child_in_batch[T.a[l]]) {   // this limb's parent is attached in the running batch: close it
            limbs.batch_end[limbs.n_batches++] = (uint8_t)l;
            memset(child_in_batch, 0, sizeof(child_in_batch));
            in_batch = 0;
        }
        child_in_batch[T.b[l]] = true;
        ++in_batch;
    }
    limbs.batch_end[limbs.n_batches++] = (uint8_t)L;
    const size_t lds = sizeof(int32_t) * ((size_t)2 * K * dets.cap + (size_t)K * ((dets.cap + 31) / 32));
    HP_KERNEL(k_pp_parse, dim3(N), dim3(kWave), lds, s, dets.cell, dets.score, dets.count, edge, limbs, P, poses.slots,
              poses.nparts, poses.score, poses.count, status);
    return hipGetLastError();
}

}  // namespace hp

// Assembly of connections into persons: the last step of the post-processing operator
// of the paper's inference engine (Section 2.2.1, operator 4, "parsing human pose
// topology").  Rules as stated at hp_assemble in hp.h.
//
// Limbs are folded in table order, one barrier-separated step per limb; inside a limb all
// connections are applied at once.  That is exact, not an approximation of the sequential
// fold: the connections of one limb (a, b) use pairwise distinct peaks of a and of b, a
// person holds at most one peak per part, hence a person can be the a-side owner of at
// most one connection and the b-side owner of at most one.  A person that is both already
// holds parts a and b, so every rule that could change it is a skip (its slot is filled,
// or a merge partner shares a part).  Every person is therefore changed by at most one
// connection per limb, and nothing a connection reads is written by another one.  New
// persons are numbered by a prefix count in connection order, as the sequential fold would.
#include "hp_dev.h"

namespace hp {

__global__ __launch_bounds__(kBlock) void k_assemble(LimbTable tab, int K, int L, int min_parts,
                                                     const int32_t *__restrict__ pcounts,
                                                     const float *__restrict__ pscore, int cap,
                                                     const int32_t *__restrict__ mcounts,
                                                     const int32_t *__restrict__ mi,
                                                     const int32_t *__restrict__ mj,
                                                     const float *__restrict__ ms, int mcap,
                                                     int32_t *owner_all, int32_t *wslots_all, int32_t *wnparts_all,
                                                     float *wscore_all, int wcap,
                                                     int32_t *pose_slots, int32_t *pose_nparts, float *pose_score,
                                                     int32_t *pose_counts, int pcap, int32_t *status)
{
    __shared__ int scratch[kBlock / kWave + 1];
    const int n = blockIdx.x;
    int32_t *owner = owner_all + (size_t)n * K * cap;
    int32_t *wslots = wslots_all + (size_t)n * wcap * K;
    int32_t *wnparts = wnparts_all + (size_t)n * wcap;
    float *wscore = wscore_all + (size_t)n * wcap;
    const float *psc = pscore + (size_t)n * K * cap;

    for (int c = 0; c < K; ++c) {
        int cnt = max(min(pcounts[n * K + c], cap), 0);
        for (int r = threadIdx.x; r < cnt; r += kBlock) owner[c * cap + r] = -1;
    }
    int np = 0;                                  // persons created so far (uniform over the workgroup)
    __syncthreads();

    for (int l = 0; l < L; ++l) {
        const int a = tab.a[l], b = tab.b[l];
        const int cnt = max(min(mcounts[n * L + l], mcap), 0);
        const size_t mo = (size_t)(n * L + l) * mcap;
        for (int base = 0; base < cnt; base += kBlock) {
            const int k = base + threadIdx.x;
            const bool act = k < cnt;
            int i = 0, j = 0, pa = -1, pb = -1;
            float s = 0.0f;
            if (act) {
                i = mi[mo + k];
                j = mj[mo + k];
                s = ms[mo + k];
                pa = owner[a * cap + i];
                pb = owner[b * cap + j];
            }
            const bool fresh = act && pa < 0 && pb < 0;
            int total;
            const int rank = block_flag_scan(fresh, scratch, total);
            if (fresh) {
                const int p = np + rank;
                if (p < wcap) {
                    for (int c = 0; c < K; ++c) wslots[(size_t)p * K + c] = -1;
                    wslots[(size_t)p * K + a] = i;
                    wslots[(size_t)p * K + b] = j;
                    wnparts[p] = 2;
                    wscore[p] = psc[a * cap + i] + psc[b * cap + j] + s;
                    owner[a * cap + i] = p;
                    owner[b * cap + j] = p;
                }
            } else if (act && pa >= 0 && pb < 0) {
                if (wslots[(size_t)pa * K + b] < 0) {
                    wslots[(size_t)pa * K + b] = j;
                    wnparts[pa] += 1;
                    float sc = wscore[pa] + psc[b * cap + j];
                    wscore[pa] = sc + s;
                    owner[b * cap + j] = pa;
                }
            } else if (act && pa < 0 && pb >= 0) {
                if (wslots[(size_t)pb * K + a] < 0) {
                    wslots[(size_t)pb * K + a] = i;
                    wnparts[pb] += 1;
                    float sc = wscore[pb] + psc[a * cap + i];
                    wscore[pb] = sc + s;
                    owner[a * cap + i] = pb;
                }
            } else if (act && pa == pb) {
                wscore[pa] = wscore[pa] + s;
            } else if (act) {
                const int lo = min(pa, pb), hi = max(pa, pb);
                bool disjoint = true;
                for (int c = 0; c < K; ++c)
                    if (wslots[(size_t)lo * K + c] >= 0 && wslots[(size_t)hi * K + c] >= 0) disjoint = false;
                if (disjoint) {
                    for (int c = 0; c < K; ++c) {
                        int r = wslots[(size_t)hi * K + c];
                        if (r >= 0) {
                            wslots[(size_t)lo * K + c] = r;
                            owner[c * cap + r] = lo;
                        }
                    }
                    wnparts[lo] += wnparts[hi];
                    float sc = wscore[lo] + wscore[hi];
                    wscore[lo] = sc + s;
                    wnparts[hi] = -1;
                }
            }
            np += total;
            __syncthreads();
        }
    }

    // alive persons with enough parts, in creation order
    int out = 0;
    np = min(np, wcap);
    for (int base = 0; base < np; base += kBlock) {
        const int p = base + threadIdx.x;
        int parts = (p < np) ? wnparts[p] : -1;
        const bool keep = parts >= min_parts && parts >= 0;
        int total;
        const int rank = out + block_flag_scan(keep, scratch, total);
        if (keep && rank < pcap) {
            const size_t o = (size_t)n * pcap + rank;
            for (int c = 0; c < K; ++c) pose_slots[o * K + c] = wslots[(size_t)p * K + c];
            pose_nparts[o] = parts;
            pose_score[o] = wscore[p];
        }
        out += total;
    }
    if (threadIdx.x == 0) {
        pose_counts[n] = out;
        if (out > pcap) atomicOr(status, (int)HP_STATUS_POSE_OVERFLOW);
    }
}

hipError_t launch_assemble(const LimbTable &T, int N, int K, int L, int min_parts, const hp_peaks &pk,
                           const hp_pairs &conns, const Workspace &ws, const hp_poses &poses,
                           int32_t *status, hipStream_t s)
{
    hipLaunchKernelGGL(k_assemble, dim3(N), dim3(kBlock), 0, s, T, K, L, min_parts, pk.count, pk.score, pk.cap,
                       conns.count, conns.i, conns.j, conns.score, conns.cap, ws.owner, ws.wslots, ws.wnparts,
                       ws.wscore, ws.wcap, poses.slots, poses.nparts, poses.score, poses.count, poses.cap, status);
    return hipGetLastError();
}

}  // namespace hp

// Assembly of connections into persons: the last step of the post-processing operator
// of the paper's inference engine (Section 2.2.1, operator 4, "parsing human pose
// topology").  Rules as stated at hp_assemble in hp.h.
//
// Limbs are folded in table order, one step per limb; inside a limb all connections are
// applied at once.  That is exact, not an approximation of the sequential fold: the
// connections of one limb (a, b) use pairwise distinct peaks of a and of b, a person holds at
// most one peak per part, hence a person can be the a-side owner of at most one connection
// and the b-side owner of at most one.  A person that is both already holds parts a and b, so
// every rule that could change it is a skip (its slot is filled, or a merge partner shares a
// part).  Every person is therefore changed by at most one connection per limb, and nothing a
// connection reads is written by another one.  New persons are numbered by a prefix count in
// connection order, as the sequential fold would.
//
// One workgroup of sixteen wavefronts works on one image.  The fold itself is a chain, one step
// per limb, and belongs to one wavefront; a single wavefront issues an instruction every four to
// five cycles at best, so whatever does not have to sit on that chain is spread over the other
// wavefronts: they fetch every connection with the scores of its two peaks into LDS before the
// fold (two memory round trips, each wavefront a few limbs), and write the persons afterwards.
// When the image's tables fit the LDS pools (always, for the workloads of interest) a limb step
// is a few dependent LDS accesses and about a hundred instructions.  Otherwise the same steps
// run, on one wavefront, on tables in the caller's workspace.
#include "hp_dev.h"

namespace hp {

// LDS pool sizes of the two builds of the kernel (int16 entries: owner table and person slots;
// 32-bit entries: connection records, person masks and scores).  The small build leaves room
// for several workgroups per CU, which matters when calls on several streams overlap: a
// workgroup of the large build owns most of a CU's LDS.
constexpr int kPool16Large = 40960, kPool32Large = 12288;
constexpr int kPool16Small = 12288, kPool32Small = 4096;

// Person tables addressed through one interface so that the fold is written once.  A person
// is K slots (peak rank per part), a bit mask of the filled parts (its part count is the
// mask's population count; an empty mask marks a person merged away) and a score.
struct LdsTables {
    int16_t *owner, *slots;
    uint32_t *mask;
    float *score;
    int ostride, K;
    __device__ int get_owner(int c, int r) const { return owner[c * ostride + r]; }
    __device__ void set_owner(int c, int r, int p) { owner[c * ostride + r] = (int16_t)p; }
    __device__ int get_slot(int p, int c) const { return slots[p * K + c]; }
    __device__ void set_slot(int p, int c, int r) { slots[p * K + c] = (int16_t)r; }
    __device__ uint32_t get_mask(int p) const { return mask[p]; }
    __device__ void set_mask(int p, uint32_t v) { mask[p] = v; }
    __device__ float get_score(int p) const { return score[p]; }
    __device__ void set_score(int p, float v) { score[p] = v; }
};

struct GlobalTables {
    int32_t *owner, *slots;
    uint32_t *mask;
    float *score;
    int ostride, K;
    __device__ int get_owner(int c, int r) const { return owner[(size_t)c * ostride + r]; }
    __device__ void set_owner(int c, int r, int p) { owner[(size_t)c * ostride + r] = p; }
    __device__ int get_slot(int p, int c) const { return slots[(size_t)p * K + c]; }
    __device__ void set_slot(int p, int c, int r) { slots[(size_t)p * K + c] = r; }
    __device__ uint32_t get_mask(int p) const { return mask[p]; }
    __device__ void set_mask(int p, uint32_t v) { mask[p] = v; }
    __device__ float get_score(int p) const { return score[p]; }
    __device__ void set_score(int p, float v) { score[p] = v; }
};

constexpr uint32_t kDead = 0u;      // a living person holds at least two parts

// Applies connection (i, j, s) of limb (a, b); sa / sb are the scores of the two peaks, pa / pb
// their owners.  `fresh_id` is the number the person gets if this connection starts one.
// The masks and scores of both owners are fetched together before any decision, so a limb
// step is two dependent table reads deep whatever rule applies.
template <typename Tab>
__device__ __forceinline__ void apply_connection(Tab &t, int K, int a, int b, int i, int j, float s, float sa,
                                                 float sb, int pa, int pb, int fresh_id, int max_persons)
{
    const uint32_t bit_a = 1u << a, bit_b = 1u << b;
    const uint32_t ma = pa >= 0 ? t.get_mask(pa) : 0u, mb = pb >= 0 ? t.get_mask(pb) : 0u;
    const float sca = pa >= 0 ? t.get_score(pa) : 0.0f, scb = pb >= 0 ? t.get_score(pb) : 0.0f;
    if (pa < 0 && pb < 0) {
        const int p = fresh_id;
        if (p < max_persons) {
            t.set_slot(p, a, i);
            t.set_slot(p, b, j);
            t.set_mask(p, bit_a | bit_b);
            t.set_score(p, sa + sb + s);
            t.set_owner(a, i, p);
            t.set_owner(b, j, p);
        }
    } else if (pa >= 0 && pb < 0) {
        if (!(ma & bit_b)) {
            t.set_slot(pa, b, j);
            t.set_mask(pa, ma | bit_b);
            const float sc = sca + sb;
            t.set_score(pa, sc + s);
            t.set_owner(b, j, pa);
        }
    } else if (pa < 0 && pb >= 0) {
        if (!(mb & bit_a)) {
            t.set_slot(pb, a, i);
            t.set_mask(pb, mb | bit_a);
            const float sc = scb + sa;
            t.set_score(pb, sc + s);
            t.set_owner(a, i, pb);
        }
    } else if (pa == pb) {
        t.set_score(pa, sca + s);
    } else if ((ma & mb) == 0u) {
        const int lo = min(pa, pb), hi = max(pa, pb);
        const uint32_t mhi = pa < pb ? mb : ma;
        for (int c = 0; c < K; ++c) {
            if (mhi & (1u << c)) {
                const int r = t.get_slot(hi, c);
                t.set_slot(lo, c, r);
                t.set_owner(c, r, lo);
            }
        }
        t.set_mask(lo, ma | mb);
        const float sc = (pa < pb) ? sca + scb : scb + sca;
        t.set_score(lo, sc + s);
        t.set_mask(hi, kDead);
    }
}

// Alive persons with enough parts, in creation order.
template <typename Tab>
__device__ __forceinline__ void emit_persons(const Tab &t, int n, int np, int K, int min_parts,
                                             int32_t *pose_slots, int32_t *pose_nparts, float *pose_score,
                                             int32_t *pose_counts, int pcap, int32_t *status)
{
    const int lane = threadIdx.x;
    int out = 0;
    for (int base = 0; base < np; base += kWave) {
        const int p = base + lane;
        const uint32_t mk = (p < np) ? t.get_mask(p) : kDead;
        const int parts = __popc(mk);
        const bool keep = mk != kDead && parts >= min_parts;
        const unsigned long long m = __ballot(keep);
        const int rank = out + __popcll(m & ((1ull << lane) - 1ull));
        if (keep && rank < pcap) {
            const size_t o = (size_t)n * pcap + rank;
            for (int c = 0; c < K; ++c) pose_slots[o * K + c] = (mk >> c) & 1u ? t.get_slot(p, c) : -1;
            pose_nparts[o] = parts;
            pose_score[o] = t.get_score(p);
        }
        out += __popcll(m);
    }
    if (lane == 0) {
        pose_counts[n] = out;
        if (out > pcap) atomicOr(status, (int)HP_STATUS_POSE_OVERFLOW);
    }
}

// Orders one wavefront's memory accesses (LDS or global) across its lanes: what some lanes wrote before it, all
// lanes see after it.  For code that a single wavefront of a workgroup runs while the others have left.
__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
}

constexpr int kAsmBlock = 1024, kAsmWaves = kAsmBlock / kWave;
constexpr int kAsmLimbsPerWave = HP_MAX_LIMBS / kAsmWaves;      // limbs wv, wv + 16, ... of wavefront wv

template <int kPool16, int kPool32>
__global__ __launch_bounds__(kAsmBlock) void k_assemble(LimbTable tab, int K, int L, int min_parts,
                                                        const int32_t *__restrict__ pcounts,
                                                        const float *__restrict__ pscore, int cap,
                                                        const int32_t *__restrict__ mcounts,
                                                        const int32_t *__restrict__ mi,
                                                        const int32_t *__restrict__ mj,
                                                        const float *__restrict__ ms, int mcap,
                                                        int32_t *owner_all, int32_t *wslots_all, int32_t *wmask_all,
                                                        float *wscore_all, int wcap,
                                                        int32_t *pose_slots, int32_t *pose_nparts, float *pose_score,
                                                        int32_t *pose_counts, int pcap, int32_t *status,
                                                        int32_t *peak_ctr, int32_t *cand_ctr,
                                                        const int32_t *__restrict__ ccounts, int ccap)
{
    __shared__ int16_t pool[kPool16];
    __shared__ __align__(16) uint32_t pool32[kPool32];
    __shared__ int moff[HP_MAX_LIMBS + 1];
    __shared__ int persons_made;
    const int n = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    if (wv == 0) {
        // last kernel of a call: every append counter of this image has been consumed by now;
        // clearing them here leaves the workspace ready for the next call
        if (peak_ctr && lane < K) peak_ctr[(n * K + lane) * kCtrStride] = 0;
        if (cand_ctr && lane < L) cand_ctr[(n * L + lane) * kCtrStride] = 0;
        // hp_assemble: the candidate lists came from an earlier call; one that needed more than its capacity is reported
        if (ccounts && lane < L && ccounts[n * L + lane] > ccap) atomicOr(status, (int)HP_STATUS_CAND_OVERFLOW);
    }
    const float *psc = pscore + (size_t)n * K * cap;
    const unsigned long long lt = (1ull << lane) - 1ull;

    // Round trip 1: the counts, and with them (before the counts are known) connection `lane` of each of this
    // wavefront's limbs: entry k of a list exists whatever the count, and entries beyond the count are never used.
    int c_i[kAsmLimbsPerWave], c_j[kAsmLimbsPerWave];
    float c_s[kAsmLimbsPerWave];
#pragma unroll
    for (int q = 0; q < kAsmLimbsPerWave; ++q) {
        const int l = wv + kAsmWaves * q;
        c_i[q] = c_j[q] = 0;
        c_s[q] = 0.0f;
        if (l < L && lane < mcap) {
            const size_t idx = (size_t)(n * L + l) * mcap + lane;
            c_i[q] = mi[idx];
            c_j[q] = mj[idx];
            c_s[q] = ms[idx];
        }
    }
    // connection counts -> offsets of each limb in the image's flat connection list (every wavefront for itself)
    const int mc = (lane < L) ? max(min(mcounts[n * L + lane], mcap), 0) : 0;
    int incl = mc;
    for (int d = 1; d < kWave; d <<= 1) {
        const int v = __shfl_up(incl, d);
        if (lane >= d) incl += v;
    }
    const int tot = __shfl(incl, kWave - 1);
    const int excl = incl - mc;
    int cmax = (lane < K) ? max(min(pcounts[n * K + lane], cap), 0) : 0;
    for (int d = kWave / 2; d > 0; d >>= 1) cmax = max(cmax, __shfl_xor(cmax, d));
    const int my_a = lane < L ? tab.a[lane] : 0, my_b = lane < L ? tab.b[lane] : 0;

    // persons never outnumber connections; one spare person, owner entry and slot row absorb the
    // stores of lanes that have nothing to write, so the fold runs without branches
    const int tot2 = (tot + 2) & ~1;              // persons incl. the spare, kept even for 8-byte alignment
    const bool fits = (long long)K * cmax + 1 + (long long)tot2 * (K + 1) <= kPool16 && 2LL * tot2 + 4LL * tot <= kPool32 &&
                      (long long)K * cmax < 65535 && tot < 32766;
    if (fits) {
        uint2 *pst = (uint2 *)pool32;                        // [tot2] person: filled-part mask (0 = merged away), score
        uint32_t *rec_o = pool32 + 2 * tot2;                 // [tot] owner-table entries of the two peaks, oa << 16 | ob
        float *rec_s = (float *)(rec_o + tot);               // [tot] connection score
        float *rec_sa = rec_s + tot, *rec_sb = rec_sa + tot; // [tot] scores of the two peaks
        int16_t *owner = pool;                               // [K * cmax + 1] person owning each peak, -1 = none
        int16_t *slots = owner + K * cmax + 1;               // [tot2][K] valid where the person's mask says so
        int16_t *prank = slots + tot2 * K;                   // [tot2] place of a person in the output, -1 = dropped
        const int spare_p = tot, spare_o = K * cmax;

        for (int idx = tid; idx <= K * cmax; idx += kAsmBlock) owner[idx] = -1;      // the spare entry too: it stays -1
        // Round trip 2: the scores of the two peaks of every connection fetched above; then the records go to LDS.
        {
            float c_sa[kAsmLimbsPerWave], c_sb[kAsmLimbsPerWave];
#pragma unroll
            for (int q = 0; q < kAsmLimbsPerWave; ++q) {
                const int l = wv + kAsmWaves * q;
                c_sa[q] = c_sb[q] = 0.0f;
                if (l < L) {
                    const int cnt = __builtin_amdgcn_readlane(mc, l);
                    const int a = __builtin_amdgcn_readlane(my_a, l), b = __builtin_amdgcn_readlane(my_b, l);
                    if (lane < cnt) {
                        c_sa[q] = psc[a * cap + c_i[q]];
                        c_sb[q] = psc[b * cap + c_j[q]];
                    }
                }
            }
#pragma unroll
            for (int q = 0; q < kAsmLimbsPerWave; ++q) {
                const int l = wv + kAsmWaves * q;
                if (l < L) {
                    const int cnt = __builtin_amdgcn_readlane(mc, l), base = __builtin_amdgcn_readlane(excl, l);
                    const int a = __builtin_amdgcn_readlane(my_a, l), b = __builtin_amdgcn_readlane(my_b, l);
                    if (lane < cnt) {
                        rec_o[base + lane] = ((uint32_t)(a * cmax + c_i[q]) << 16) | (uint32_t)(b * cmax + c_j[q]);
                        rec_s[base + lane] = c_s[q];
                        rec_sa[base + lane] = c_sa[q];
                        rec_sb[base + lane] = c_sb[q];
                    }
                }
            }
            // limbs with more than 64 connections: the rest, fetched now
#pragma unroll
            for (int q = 0; q < kAsmLimbsPerWave; ++q) {
                const int l = wv + kAsmWaves * q;
                if (l >= L) continue;
                const int cnt = __builtin_amdgcn_readlane(mc, l), base = __builtin_amdgcn_readlane(excl, l);
                const int a = __builtin_amdgcn_readlane(my_a, l), b = __builtin_amdgcn_readlane(my_b, l);
                for (int k = kWave + lane; k < cnt; k += kWave) {
                    const size_t idx = (size_t)(n * L + l) * mcap + k;
                    const int i = mi[idx], j = mj[idx];
                    rec_o[base + k] = ((uint32_t)(a * cmax + i) << 16) | (uint32_t)(b * cmax + j);
                    rec_s[base + k] = ms[idx];
                    rec_sa[base + k] = psc[a * cap + i];
                    rec_sb[base + k] = psc[b * cap + j];
                }
            }
        }
        __syncthreads();                          // owner table and records are in place

        if (wv == 0) {
            int np = 0;
            for (int l = 0; l < L; ++l) {
                // lane l holds limb l's description; read it with uniform lane reads
                const int a = __builtin_amdgcn_readlane(my_a, l), b = __builtin_amdgcn_readlane(my_b, l);
                const int cnt = __builtin_amdgcn_readlane(mc, l), base = __builtin_amdgcn_readlane(excl, l);
                const uint32_t bit_a = 1u << a, bit_b = 1u << b;
                const int row_a = a * cmax, row_b = b * cmax;
                for (int k0 = 0; k0 < cnt; k0 += kWave) {
                    // one connection per lane, all connections of the limb at once
                    const bool act = k0 + lane < cnt;
                    const int o = base + (act ? k0 + lane : 0);
                    const uint32_t oab = rec_o[o];
                    const float s = rec_s[o], sa = rec_sa[o], sb = rec_sb[o];
                    const int oa = act ? (int)(oab >> 16) : spare_o, ob = act ? (int)(oab & 0xffffu) : spare_o;
                    const int pa = owner[oa], pb = owner[ob];         // the spare entry reads as -1
                    const bool has_a = pa >= 0, has_b = pb >= 0;
                    const uint2 sta = pst[max(pa, 0)], stb = pst[max(pb, 0)];
                    const uint32_t ma = has_a ? sta.x : 0u, mb = has_b ? stb.x : 0u;
                    const float sca = __uint_as_float(sta.y), scb = __uint_as_float(stb.y);

                    const bool fresh = act && !has_a && !has_b;
                    const unsigned long long fm = __ballot(fresh);
                    const bool ext_a = has_a && !has_b && !(ma & bit_b);      // the a-side owner gains part b
                    const bool ext_b = !has_a && has_b && !(mb & bit_a);      // the b-side owner gains part a
                    const bool cyc = has_a && pa == pb;
                    const bool mrg = has_a && has_b && pa != pb && (ma & mb) == 0u;
                    const bool upd = fresh || ext_a || ext_b || cyc;
                    const int p = fresh ? np + __popcll(fm & lt) : (has_a ? pa : pb);
                    const uint32_t mk = fresh ? (bit_a | bit_b) : ext_a ? (ma | bit_b) : ext_b ? (mb | bit_a) : ma;
                    const float s0 = fresh ? sa : has_a ? sca : scb;          // running score, then the new
                    const float s1 = (fresh || ext_a) ? sb : sa;              // peak's score (if any), then s
                    const float sc = cyc ? s0 : s0 + s1;
                    const bool wa = fresh || ext_b, wb = fresh || ext_a;
                    pst[upd ? p : spare_p] = make_uint2(mk, __float_as_uint(sc + s));
                    slots[(wa ? p : spare_p) * K + a] = (int16_t)(oa - row_a);
                    owner[wa ? oa : spare_o] = (int16_t)(wa ? p : -1);
                    slots[(wb ? p : spare_p) * K + b] = (int16_t)(ob - row_b);
                    owner[wb ? ob : spare_o] = (int16_t)(wb ? p : -1);
                    unsigned long long merging = __ballot(mrg);
                    if (merging) {
                        // the survivor is the earlier person; it takes the other's parts, one merge at a time with a
                        // lane a part (the merges of one limb concern different persons, so their order is free; a
                        // merging lane walking its person's parts by itself took a microsecond a limb)
                        const int lo = min(pa, pb), hi = max(pa, pb);
                        const uint32_t mhi = pa < pb ? mb : ma;
                        if (mrg) {
                            const float scm = (pa < pb) ? sca + scb : scb + sca;
                            pst[lo] = make_uint2(ma | mb, __float_as_uint(scm + s));
                            pst[hi] = make_uint2(kDead, 0u);
                        }
                        for (; merging; merging &= merging - 1ull) {
                            const int r = __ffsll((long long)merging) - 1;
                            const int lo_r = __builtin_amdgcn_readlane(lo, r), hi_r = __builtin_amdgcn_readlane(hi, r);
                            const uint32_t parts = (uint32_t)__builtin_amdgcn_readlane((int)mhi, r);
                            if (lane < K && ((parts >> lane) & 1u)) {
                                const int16_t rr = slots[hi_r * K + lane];
                                slots[lo_r * K + lane] = rr;
                                owner[lane * cmax + rr] = (int16_t)lo_r;
                            }
                        }
                    }
                    np += __popcll(fm);
                    wave_sync();                  // LDS written by some lanes is read by others in the next step
                }
            }
            // alive persons with enough parts keep their creation order: their places in the output
            np = min(np, tot);
            int out = 0;
            for (int base = 0; base < np; base += kWave) {
                const int p = base + lane;
                const uint32_t mk = p < np ? pst[p].x : kDead;
                const bool keep = mk != kDead && __popc(mk) >= min_parts;
                const unsigned long long m = __ballot(keep);
                if (p < np) prank[p] = (int16_t)(keep && out + __popcll(m & lt) < pcap ? out + __popcll(m & lt) : -1);
                out += __popcll(m);
            }
            if (lane == 0) {
                persons_made = np;
                pose_counts[n] = out;
                if (out > pcap) atomicOr(status, (int)HP_STATUS_POSE_OVERFLOW);
            }
        }
        __syncthreads();
        // the persons written by all wavefronts: a thread per (person, part)
        const int np = persons_made;
        for (int idx = tid; idx < np * K; idx += kAsmBlock) {
            const int p = idx / K, c = idx - p * K;
            const int r = prank[p];
            if (r >= 0) pose_slots[((size_t)n * pcap + r) * K + c] = (pst[p].x >> c) & 1u ? (int)slots[idx] : -1;
        }
        for (int p = tid; p < np; p += kAsmBlock) {
            const int r = prank[p];
            if (r >= 0) {
                const uint2 st = pst[p];
                pose_nparts[(size_t)n * pcap + r] = __popc(st.x);
                pose_score[(size_t)n * pcap + r] = __uint_as_float(st.y);
            }
        }
        return;
    }
    if (wv != 0) return;                          // the fallback is one wavefront's work
    if (lane < L) moff[lane] = excl;
    if (lane == 0) moff[L] = tot;
    wave_sync();

    // tables too large for LDS: the same fold on the workspace tables
    GlobalTables t;
    t.owner = owner_all + (size_t)n * K * cap;
    t.slots = wslots_all + (size_t)n * wcap * K;
    t.mask = (uint32_t *)wmask_all + (size_t)n * wcap;
    t.score = wscore_all + (size_t)n * wcap;
    t.ostride = cap;
    t.K = K;
    for (int c = 0; c < K; ++c) {
        const int cnt = max(min(pcounts[n * K + c], cap), 0);
        for (int r = lane; r < cnt; r += kWave) t.owner[(size_t)c * cap + r] = -1;
    }
    wave_sync();
    int np = 0;
    for (int l = 0; l < L; ++l) {
        const int a = tab.a[l], b = tab.b[l];
        const int cnt = moff[l + 1] - moff[l];
        const size_t mo = (size_t)(n * L + l) * mcap;
        for (int k0 = 0; k0 < cnt; k0 += kWave) {
            const int k = k0 + lane;
            const bool act = k < cnt;
            int i = 0, j = 0, pa = -1, pb = -1;
            float s = 0.0f, sa = 0.0f, sb = 0.0f;
            if (act) {
                i = mi[mo + k];
                j = mj[mo + k];
                s = ms[mo + k];
                sa = psc[a * cap + i];
                sb = psc[b * cap + j];
                pa = t.get_owner(a, i);
                pb = t.get_owner(b, j);
            }
            const unsigned long long fm = __ballot(act && pa < 0 && pb < 0);
            if (act) apply_connection(t, K, a, b, i, j, s, sa, sb, pa, pb, np + __popcll(fm & lt), wcap);
            np += __popcll(fm);
            wave_sync();
        }
    }
    emit_persons(t, n, min(np, wcap), K, min_parts, pose_slots, pose_nparts, pose_score, pose_counts, pcap, status);
}

hipError_t launch_assemble(const LimbTable &T, int N, int K, int L, int min_parts, const hp_peaks &pk,
                           const hp_pairs *cands, const hp_pairs &conns, const Workspace &ws,
                           const hp_poses &poses, int32_t *status, hipStream_t s)
{
    const int32_t *ccounts = cands ? cands->count : nullptr;
    const int ccap = cands ? cands->cap : 0;
    // few peaks per part: the tables of an image almost surely fit the small pools (if they do
    // not, the fold runs on the workspace tables, slower but the same)
    if (pk.cap <= 256)
        HP_KERNEL((k_assemble<kPool16Small, kPool32Small>), dim3(N), dim3(kAsmBlock), 0, s, T, K, L, min_parts,
                           pk.count, pk.score, pk.cap, conns.count, conns.i, conns.j, conns.score, conns.cap, ws.owner,
                           ws.wslots, ws.wmask, ws.wscore, ws.wcap, poses.slots, poses.nparts, poses.score,
                           poses.count, poses.cap, status, ws.peak_ctr, ws.cand_ctr, ccounts, ccap);
    else
        HP_KERNEL((k_assemble<kPool16Large, kPool32Large>), dim3(N), dim3(kAsmBlock), 0, s, T, K, L, min_parts,
                           pk.count, pk.score, pk.cap, conns.count, conns.i, conns.j, conns.score, conns.cap, ws.owner,
                           ws.wslots, ws.wmask, ws.wscore, ws.wcap, poses.slots, poses.nparts, poses.score,
                           poses.count, poses.cap, status, ws.peak_ctr, ws.cand_ctr, ccounts, ccap);
    return hipGetLastError();
}

}  // namespace hp

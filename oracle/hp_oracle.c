/*
 * CPU oracle for bottom-up (CM + PAF) pose post-processing.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what
 * the post-processing operator of the paper's inference engine computes
 * (Section 2.2.1, operator 4: activation maps in, human pose topology out;
 * Section 2.3: the PAF / OpenPose family).  It shares no code with the HIP
 * library and must never be called from the product path.
 *
 * The paper states the operator's job but none of its arithmetic, so every
 * rule below is this build's reading, written out step by step:
 *   R  bilinear upsampling by s with half-pixel centres and edge clamping,
 *      horizontal pass first, each pass one rounded product plus one fused
 *      multiply-add;
 *   P  a pixel is a peak when it exceeds the threshold and is the maximum of
 *      its in-bounds 3x3 neighbourhood, ties going to the raster-first pixel;
 *   S  a candidate limb is scored by the mean, over S evenly spaced
 *      nearest-pixel samples of the segment, of the PAF projected on the
 *      segment's unit direction, and kept when enough samples exceed the PAF
 *      threshold and the mean is positive;
 *   M  candidates of one limb are matched greedily in the strict order
 *      (score descending, i ascending, j ascending);
 *   A  limbs are folded into persons in table order.
 * Floating point is fp32 in exactly the order written here, because peak
 * membership, sample validity and the greedy order are integer decisions taken
 * on these floats: both implementations must take them in the same precision.
 * Compile with -ffp-contract=off so that only the explicit fmaf calls fuse.
 *
 * Parity pins: R, P, S, M are pinned by tests against library routines,
 * closed forms and brute force.  A (assembly) is pinned only by recovery of
 * planted skeletons and by invariants: parity with the paper's own engine is
 * unpinned, the paper gives neither rule nor example.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---- R: upsampling --------------------------------------------------- */

/* Source cell and weight of output index X along an axis of n lo-res nodes:
 * the output sample sits at (X + 1/2)/s - 1/2 in lo-res units; left of node 0
 * it is clamped onto node 0, right of node n-1 the upper neighbour is clamped. */
static void hpo_axis(int X, int s, int n, int *i0, int *i1, float *f)
{
    int num = 2 * X + 1 - s;          /* = 2s * source coordinate */
    if (num < 0) {
        *i0 = 0;
        *f = 0.0f;
    } else {
        *i0 = num / (2 * s);
        *f = (float)(num % (2 * s)) / (float)(2 * s);
    }
    *i1 = (*i0 + 1 < n) ? *i0 + 1 : n - 1;
}

/* Upsampled value of one lo-res plane at hi-res pixel (Y, X). */
float hpo_up(const float *lo, int h, int w, int s, int Y, int X)
{
    int x0, x1, y0, y1;
    float f, g;
    hpo_axis(X, s, w, &x0, &x1, &f);
    hpo_axis(Y, s, h, &y0, &y1, &g);
    float r0 = fmaf(f, lo[y0 * w + x1], (1.0f - f) * lo[y0 * w + x0]);
    float r1 = fmaf(f, lo[y1 * w + x1], (1.0f - f) * lo[y1 * w + x0]);
    return fmaf(g, r1, (1.0f - g) * r0);
}

/* lo [planes][h][w] -> hi [planes][s*h][s*w]. */
void hpo_resize(const float *lo, int planes, int h, int w, int s, float *hi)
{
    int H = s * h, W = s * w;
    for (int p = 0; p < planes; ++p)
        for (int Y = 0; Y < H; ++Y)
            for (int X = 0; X < W; ++X)
                hi[((size_t)p * H + Y) * W + X] = hpo_up(lo + (size_t)p * h * w, h, w, s, Y, X);
}

/* ---- P: peaks -------------------------------------------------------- */

/* Peaks of one hi-res plane in raster order.  Returns the number found; only
 * the first `cap` are stored. */
int hpo_find_peaks(const float *u, int H, int W, float thr, int cap,
                   int32_t *px, int32_t *py, float *ps)
{
    int n = 0;
    for (int y = 0; y < H; ++y) {
        for (int x = 0; x < W; ++x) {
            float v = u[(size_t)y * W + x];
            if (!(v > thr))
                continue;
            int is_peak = 1;
            for (int dy = -1; dy <= 1 && is_peak; ++dy) {
                for (int dx = -1; dx <= 1; ++dx) {
                    if (dy == 0 && dx == 0)
                        continue;
                    int yy = y + dy, xx = x + dx;
                    if (yy < 0 || yy >= H || xx < 0 || xx >= W)
                        continue;
                    float nb = u[(size_t)yy * W + xx];
                    int earlier = (dy < 0) || (dy == 0 && dx < 0);
                    if (earlier ? !(v > nb) : !(v >= nb)) {
                        is_peak = 0;
                        break;
                    }
                }
            }
            if (is_peak) {
                if (n < cap) {
                    px[n] = x;
                    py[n] = y;
                    ps[n] = v;
                }
                ++n;
            }
        }
    }
    return n;
}

/* ---- S: limb scoring -------------------------------------------------- */

/* Number of valid samples a candidate needs: ceil(ratio * S) in fp32. */
int hpo_need(float min_valid_ratio, int S)
{
    return (int)ceilf(min_valid_ratio * (float)S);
}

/* Scores every pair (i in A, j in B) of one limb of one image.  pafx/pafy are
 * the limb's two lo-res planes.  Accepted candidates come out in (i, j)
 * order; returns their number, storing only the first `ccap`. */
int hpo_score_limb(const float *pafx, const float *pafy, int h, int w, int s,
                   int nA, const int32_t *xA, const int32_t *yA,
                   int nB, const int32_t *xB, const int32_t *yB,
                   int S, float paf_thr, int need, int ccap,
                   int32_t *ci, int32_t *cj, float *cs)
{
    int n = 0;
    for (int i = 0; i < nA; ++i) {
        for (int j = 0; j < nB; ++j) {
            int dx = xB[j] - xA[i], dy = yB[j] - yA[i];
            if (dx == 0 && dy == 0)
                continue;
            float norm = sqrtf((float)(dx * dx + dy * dy));
            float ux = (float)dx / norm, uy = (float)dy / norm;
            float acc = 0.0f;
            int valid = 0;
            for (int k = 0; k < S; ++k) {
                float t = (float)k / (float)(S - 1);
                int sx = (int)floorf(fmaf(t, (float)dx, (float)xA[i]) + 0.5f);
                int sy = (int)floorf(fmaf(t, (float)dy, (float)yA[i]) + 0.5f);
                float vx = hpo_up(pafx, h, w, s, sy, sx);
                float vy = hpo_up(pafy, h, w, s, sy, sx);
                float d = fmaf(vy, uy, vx * ux);
                if (d > paf_thr)
                    ++valid;
                acc = acc + d;
            }
            float score = acc / (float)S;
            if (valid >= need && score > 0.0f) {
                if (n < ccap) {
                    ci[n] = i;
                    cj[n] = j;
                    cs[n] = score;
                }
                ++n;
            }
        }
    }
    return n;
}

/* ---- M: greedy matching ---------------------------------------------- */

typedef struct { float s; int32_t i, j; } hpo_cand;

static int hpo_cand_cmp(const void *pa, const void *pb)
{
    const hpo_cand *a = (const hpo_cand *)pa, *b = (const hpo_cand *)pb;
    if (a->s != b->s) return (a->s > b->s) ? -1 : 1;
    if (a->i != b->i) return (a->i < b->i) ? -1 : 1;
    if (a->j != b->j) return (a->j < b->j) ? -1 : 1;
    return 0;
}

/* Greedy one-to-one matching of n candidates between nA and nB peaks.
 * Connections come out in acceptance order; returns their number
 * (at most min(nA, nB)); mi/mj/ms must hold that many. */
int hpo_match_limb(int n, const int32_t *ci, const int32_t *cj, const float *cs,
                   int nA, int nB, int32_t *mi, int32_t *mj, float *ms)
{
    hpo_cand *c = (hpo_cand *)malloc(sizeof(hpo_cand) * (size_t)(n > 0 ? n : 1));
    char *usedA = (char *)calloc((size_t)(nA > 0 ? nA : 1), 1);
    char *usedB = (char *)calloc((size_t)(nB > 0 ? nB : 1), 1);
    for (int k = 0; k < n; ++k) {
        c[k].s = cs[k];
        c[k].i = ci[k];
        c[k].j = cj[k];
    }
    qsort(c, (size_t)n, sizeof(hpo_cand), hpo_cand_cmp);
    int m = 0;
    for (int k = 0; k < n; ++k) {
        if (usedA[c[k].i] || usedB[c[k].j])
            continue;
        usedA[c[k].i] = 1;
        usedB[c[k].j] = 1;
        mi[m] = c[k].i;
        mj[m] = c[k].j;
        ms[m] = c[k].s;
        ++m;
    }
    free(c);
    free(usedA);
    free(usedB);
    return m;
}

/* ---- A: assembly ------------------------------------------------------ */

/* Folds the connections of one image into persons.
 *   K parts, L limbs (limb_a[l] -> limb_b[l]); part c has at most pstride
 *   peaks with scores pscore[c * pstride + rank]; limb l has mcount[l] connections
 *   (mi, mj, ms)[l * mstride + k] in acceptance order.
 * A person is K slots holding the rank of its peak in that part's list, or -1.
 * For each connection (i, j, s) of limb (a, b), with pa / pb the persons that
 * own peak i of a / peak j of b:
 *   neither owned: new person {a: i, b: j}, score = ps(a,i) + ps(b,j) + s;
 *   one owned:     if that person's other slot is empty, fill it and add the
 *                  new peak's score, then s; otherwise skip;
 *   same person:   add s (a redundant limb closing a cycle);
 *   two persons:   if they share no filled part, merge the later-created into
 *                  the earlier-created (score = earlier + later, then + s);
 *                  otherwise skip.
 * Persons alive at the end with at least min_parts parts come out in creation
 * order.  Returns their number; only the first `pcap` are stored. */
int hpo_assemble(int K, int L, const int32_t *limb_a, const int32_t *limb_b,
                 const float *pscore, int pstride,
                 const int32_t *mcount, const int32_t *mi, const int32_t *mj, const float *ms,
                 int mstride, int min_parts, int pcap,
                 int32_t *pose_slots, int32_t *pose_nparts, float *pose_score)
{
    int max_persons = 1;
    for (int l = 0; l < L; ++l)
        max_persons += mcount[l];
    int32_t *owner = (int32_t *)malloc(sizeof(int32_t) * (size_t)K * (size_t)(pstride > 0 ? pstride : 1));
    int32_t *slots = (int32_t *)malloc(sizeof(int32_t) * (size_t)max_persons * (size_t)K);
    int32_t *nparts = (int32_t *)malloc(sizeof(int32_t) * (size_t)max_persons);
    float *score = (float *)malloc(sizeof(float) * (size_t)max_persons);
    char *alive = (char *)malloc((size_t)max_persons);
    for (int c = 0; c < K; ++c)
        for (int r = 0; r < pstride; ++r)
            owner[c * pstride + r] = -1;
    int np = 0;

    for (int l = 0; l < L; ++l) {
        int a = limb_a[l], b = limb_b[l];
        for (int k = 0; k < mcount[l]; ++k) {
            int i = mi[l * mstride + k], j = mj[l * mstride + k];
            float s = ms[l * mstride + k];
            int pa = owner[a * pstride + i], pb = owner[b * pstride + j];
            if (pa < 0 && pb < 0) {
                int p = np++;
                for (int c = 0; c < K; ++c)
                    slots[p * K + c] = -1;
                slots[p * K + a] = i;
                slots[p * K + b] = j;
                nparts[p] = 2;
                score[p] = pscore[a * pstride + i] + pscore[b * pstride + j] + s;
                alive[p] = 1;
                owner[a * pstride + i] = p;
                owner[b * pstride + j] = p;
            } else if (pa >= 0 && pb < 0) {
                if (slots[pa * K + b] < 0) {
                    slots[pa * K + b] = j;
                    nparts[pa] += 1;
                    score[pa] = score[pa] + pscore[b * pstride + j];
                    score[pa] = score[pa] + s;
                    owner[b * pstride + j] = pa;
                }
            } else if (pa < 0 && pb >= 0) {
                if (slots[pb * K + a] < 0) {
                    slots[pb * K + a] = i;
                    nparts[pb] += 1;
                    score[pb] = score[pb] + pscore[a * pstride + i];
                    score[pb] = score[pb] + s;
                    owner[a * pstride + i] = pb;
                }
            } else if (pa == pb) {
                score[pa] = score[pa] + s;
            } else {
                int lo = pa < pb ? pa : pb, hi = pa < pb ? pb : pa;
                int disjoint = 1;
                for (int c = 0; c < K; ++c)
                    if (slots[lo * K + c] >= 0 && slots[hi * K + c] >= 0)
                        disjoint = 0;
                if (disjoint) {
                    for (int c = 0; c < K; ++c) {
                        if (slots[hi * K + c] >= 0) {
                            slots[lo * K + c] = slots[hi * K + c];
                            owner[c * pstride + slots[hi * K + c]] = lo;
                        }
                    }
                    nparts[lo] += nparts[hi];
                    score[lo] = score[lo] + score[hi];
                    score[lo] = score[lo] + s;
                    alive[hi] = 0;
                }
            }
        }
    }

    int n = 0;
    for (int p = 0; p < np; ++p) {
        if (!alive[p] || nparts[p] < min_parts)
            continue;
        if (n < pcap) {
            memcpy(pose_slots + (size_t)n * K, slots + (size_t)p * K, sizeof(int32_t) * (size_t)K);
            pose_nparts[n] = nparts[p];
            pose_score[n] = score[p];
        }
        ++n;
    }
    free(owner);
    free(slots);
    free(nparts);
    free(score);
    free(alive);
    return n;
}

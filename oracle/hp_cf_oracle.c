/*
 * CPU oracle for the decoder of the composite-field family.
 *
 * TEST INFRASTRUCTURE ONLY.  It shares no code with the HIP library and must
 * never be called from the product path.
 *
 * Section 2.3 of the paper lists PifPaf as the third algorithm class its
 * engine post-processes and says nothing about how.  The cited method predicts
 * two composite fields on a coarse grid: per part a "part intensity field"
 * (confidence c, a vector (x, y) to the part, a spread b used only in
 * training, a scale sigma) and per limb a "part association field"
 * (confidence c and, for each of the limb's two parts, a vector and a spread).
 * Its decoder (a) turns the intensity field into a fine confidence map, the
 * sum of one Gaussian of width sigma per cell placed where the cell's vector
 * points, (b) takes the cells with the highest map values as seeds, and
 * (c) grows a person from each seed by following association fields, scoring
 * an association a for a joint at x as c * exp(-|x - a1| / b1) * f2(a2),
 * confirming each step by the reverse search, and suppressing seeds that fall
 * on joints already found.  The rules below are this build's reading of that,
 * step by step (fp32 throughout, one operation per line as written; s is the
 * stride: the map is H = Fh * s by W = Fw * s for an Fh x Fw grid):
 *   C0 E(t) ~ exp(-t), the same arithmetic on every machine: tc = max(min(t, 80), 0);
 *      y = tc * log2(e); n = rint(y); z = (y - n) * (-ln 2);
 *      p = 1 + z(1 + z(1/2 + z(1/6 + z(1/24 + z(1/120 + z/720))))) with one fused
 *      multiply-add per step; E = p * 2^(-n);
 *   C1 cell (gy, gx) of part k points to X = ((float)gx + x) * s, Y = ((float)gy + y) * s;
 *      it is active when c > pif_thr and 0 <= X <= W - 1 and 0 <= Y <= H - 1.  Its width
 *      is sg = max(sigma * s, 1), its window w = (int)min(ceil(3 sg), 24), its nearest
 *      pixel (xr, yr) = (rint X, rint Y) (ties to even);
 *   C2 the map: f_k(px, py) = sum, over the active cells of k in ascending cell order
 *      whose window holds the pixel (|px - xr| <= w and |py - yr| <= w), of
 *      c * E(d2 * inv) with d2 = (px - X)^2 + (py - Y)^2 and inv = 0.5 / (sg * sg);
 *   C3 the value of an active cell is v = f_k(xr, yr); it is a seed when v > seed_thr;
 *      seeds are taken by (v descending, part ascending, cell ascending);
 *   C4 cell (gy, gx) of limb l (a -> b) has the end points P1 = ((gx + x1) s, (gy + y1) s)
 *      and P2 likewise; it is active when c > paf_thr and both end points lie on the map
 *      (as in C1).  iB1 = 1 / max(b1 * s, 1), iB2 likewise; F1 = f_a(rint P1), F2 = f_b(rint P2).
 *      For a joint of part a at Q the cell scores (c * F2) * E(|Q - P1| * iB1) and proposes
 *      P2 for part b; for a joint of part b at Q it scores (c * F1) * E(|Q - P2| * iB2) and
 *      proposes P1.  |.| = sqrt(dx * dx + dy * dy).  A search takes the active cell with the
 *      largest score (ties: the lowest cell);
 *   C5 a person starts as the seed's joint (position (X, Y), value v, radius sg) and grows
 *      in rounds.  A round looks at every limb of which the person held exactly one part
 *      when the round began: the search from that joint must score above grow_thr; the
 *      search back from the proposed point T over the same limb in the other direction
 *      must find a cell (any score above 0) whose proposal lies within rev_tol of the
 *      joint ((dx * dx + dy * dy) <= rev_tol * rev_tol); T must not be occupied (C7) for
 *      its part.  Of a round's proposals for one part the highest score wins (ties: the
 *      earlier limb); the part is then held at T with that score as its value and the
 *      radius max(sigma * s, 1) of the intensity cell (yr / s, xr / s) of that part under
 *      rint T.  Growing ends with the first round that adds nothing;
 *   C6 a person with at least min_parts parts is recorded: score = (sum of the held
 *      values in part order, from 0) / (float)K;
 *   C7 a point (x, y) is occupied for part k when a recorded person holds k at (xj, yj)
 *      with radius r and (x - xj)^2 + (y - yj)^2 <= r * r.  A seed that is occupied
 *      for its part is skipped, and so is a seed that lies within the radius of an earlier
 *      seed of its part whose person was grown and not recorded (the same test with that
 *      seed's position and radius): suppression at the level of a part applies to every
 *      person the decoder finished, kept or not;
 *   C8 decoding of an image stops when a seed passes C7 while pcap persons are recorded
 *      (the caller is told).
 *
 * Parity pins (tests/test_oracle_cf.py): E against the library exponential, the
 * map of a single cell against the Gaussian in float64 and its symmetries, additivity
 * of the map, exact recovery of persons planted in the fields, and hand-built cases
 * for the thresholds, the reverse check, occupancy and the round rule.
 * Parity with the paper's own engine is unpinned (it prints no outputs).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* C0 */
#ifdef HPC_LIBM_EXP
/* Test-only build (tests/test_oracle_cf.py): the C library's exponential in place of the fixed
 * arithmetic of C0, everything else unchanged.  Decoding with it must find the same cells, seeds
 * and persons: which routine evaluates the exponential may move values in the last digits and
 * nothing else. */
float hpc_expneg(float t)
{
    return expf(-fmaxf(fminf(t, 80.0f), 0.0f));
}
#else
float hpc_expneg(float t)
{
    const float tc = fmaxf(fminf(t, 80.0f), 0.0f);
    const float y = tc * 0x1.715476p+0f;
    const float n = rintf(y);
    const float z = (y - n) * -0x1.62e430p-1f;
    float p = 0x1.6c16c2p-10f;
    p = fmaf(p, z, 0x1.111112p-7f);
    p = fmaf(p, z, 0x1.555556p-5f);
    p = fmaf(p, z, 0x1.555556p-3f);
    p = fmaf(p, z, 0.5f);
    p = fmaf(p, z, 1.0f);
    p = fmaf(p, z, 1.0f);
    return ldexpf(p, -(int)n);
}
#endif

static int hpc_on_map(float X, float Y, int H, int W)
{
    return X >= 0.0f && X <= (float)(W - 1) && Y >= 0.0f && Y <= (float)(H - 1);
}

typedef struct {
    int cell, xr, yr, w;
    float X, Y, sg, inv, c;
} hpc_pif;

/* C1 for one cell of one part's field pif [5][Fh][Fw]; returns 0 when the cell is not active */
static int hpc_pif_cell(const float *pif, int Fh, int Fw, int s, int cell, float pif_thr, hpc_pif *out)
{
    const int cells = Fh * Fw, gy = cell / Fw, gx = cell % Fw;
    const float c = pif[0 * cells + cell];
    const float X = ((float)gx + pif[1 * cells + cell]) * (float)s;
    const float Y = ((float)gy + pif[2 * cells + cell]) * (float)s;
    if (!(c > pif_thr) || !hpc_on_map(X, Y, Fh * s, Fw * s)) return 0;
    out->cell = cell;
    out->X = X;
    out->Y = Y;
    out->c = c;
    out->sg = fmaxf(pif[4 * cells + cell] * (float)s, 1.0f);
    out->inv = 0.5f / (out->sg * out->sg);
    out->w = (int)fminf(ceilf(3.0f * out->sg), 24.0f);
    out->xr = (int)rintf(X);
    out->yr = (int)rintf(Y);
    return 1;
}

/* C2: the fine map of one part, f [H][W] */
void hpc_field(const float *pif, int Fh, int Fw, int s, float pif_thr, float *f)
{
    const int H = Fh * s, W = Fw * s;
    memset(f, 0, sizeof(float) * (size_t)H * W);
    for (int cell = 0; cell < Fh * Fw; ++cell) {
        hpc_pif q;
        if (!hpc_pif_cell(pif, Fh, Fw, s, cell, pif_thr, &q)) continue;
        for (int py = q.yr - q.w; py <= q.yr + q.w; ++py) {
            if (py < 0 || py >= H) continue;
            for (int px = q.xr - q.w; px <= q.xr + q.w; ++px) {
                if (px < 0 || px >= W) continue;
                const float dx = (float)px - q.X, dy = (float)py - q.Y;
                const float d2 = dx * dx + dy * dy;
                f[(size_t)py * W + px] = f[(size_t)py * W + px] + q.c * hpc_expneg(d2 * q.inv);
            }
        }
    }
}

typedef struct {
    int cell;
    float c, x1, y1, iB1, x2, y2, iB2, F1, F2;
} hpc_paf;

typedef struct {
    float v;
    int k, rank;
} hpc_seed;

static int hpc_seed_cmp(const void *pa, const void *pb)
{
    const hpc_seed *a = (const hpc_seed *)pa, *b = (const hpc_seed *)pb;
    if (a->v != b->v) return a->v > b->v ? -1 : 1;
    if (a->k != b->k) return a->k < b->k ? -1 : 1;
    return a->rank < b->rank ? -1 : (a->rank > b->rank ? 1 : 0);   /* lists are in ascending cell order */
}

/* C4: the best active cell of a limb's list for a joint at (qx, qy); forward = the joint is the limb's first part */
static int hpc_search(const hpc_paf *list, int n, int forward, float qx, float qy, float above, float *best_s)
{
    int best = -1;
    float bs = above;
    for (int i = 0; i < n; ++i) {
        const hpc_paf *a = &list[i];
        const float dx = qx - (forward ? a->x1 : a->x2), dy = qy - (forward ? a->y1 : a->y2);
        const float d = sqrtf(dx * dx + dy * dy);
        const float e = hpc_expneg(d * (forward ? a->iB1 : a->iB2));
        const float sc = (a->c * (forward ? a->F2 : a->F1)) * e;
        if (sc > bs) {
            bs = sc;
            best = i;
        }
    }
    *best_s = bs;
    return best;
}

/* C7 against the recorded persons: xyv [np][K][3], rad [np][K] */
static int hpc_occupied(const float *xyv, const float *rad, int np, int K, int k, float x, float y)
{
    for (int p = 0; p < np; ++p) {
        const float *j = xyv + ((size_t)p * K + k) * 3;
        if (!(j[2] > 0.0f)) continue;
        const float dx = x - j[0], dy = y - j[1], r = rad[(size_t)p * K + k];
        if (dx * dx + dy * dy <= r * r) return 1;
    }
    return 0;
}

/*
 * One image.  pif [K][5][Fh][Fw], paf [L][7][Fh][Fw].
 * Lists (for inspection): pif_cell, pif_val [K][cells], pif_count [K]; paf_cell, paf_f1, paf_f2 [L][cells], paf_count [L].
 * Persons: xyv [pcap][K][3] (x, y, value; zeros for a part not held), nparts, score [pcap].
 * Returns the number of persons recorded; *overflow is set when C8 stopped the decoding.
 */
int hpc_decode(const float *pif, const float *paf, int K, int L, const int32_t *limb_a, const int32_t *limb_b, int Fh,
               int Fw, int s, float pif_thr, float paf_thr, float seed_thr, float grow_thr, float rev_tol,
               int min_parts, int pcap, int32_t *pif_cell, float *pif_val, int32_t *pif_count, int32_t *paf_cell,
               float *paf_f1, float *paf_f2, int32_t *paf_count, float *xyv, int32_t *nparts, float *score,
               int32_t *overflow)
{
    const int cells = Fh * Fw, H = Fh * s, W = Fw * s;
    float *f = (float *)malloc(sizeof(float) * (size_t)K * H * W);
    hpc_pif *pl = (hpc_pif *)malloc(sizeof(hpc_pif) * (size_t)K * cells);
    hpc_paf *al = (hpc_paf *)malloc(sizeof(hpc_paf) * (size_t)L * cells);
    hpc_seed *seeds = (hpc_seed *)malloc(sizeof(hpc_seed) * (size_t)K * cells);
    float *rad = (float *)malloc(sizeof(float) * (size_t)(pcap > 0 ? pcap : 1) * K);
    float *ghost = (float *)malloc(sizeof(float) * 4 * (size_t)K * cells);   /* x, y, radius, part of the seeds grown in vain */
    int ng = 0;
    int ns = 0, np = 0;
    *overflow = 0;

    /* C1-C3 */
    for (int k = 0; k < K; ++k) {
        const float *pk = pif + (size_t)k * 5 * cells;
        hpc_field(pk, Fh, Fw, s, pif_thr, f + (size_t)k * H * W);
        int n = 0;
        for (int cell = 0; cell < cells; ++cell) {
            hpc_pif q;
            if (!hpc_pif_cell(pk, Fh, Fw, s, cell, pif_thr, &q)) continue;
            const float v = f[((size_t)k * H + q.yr) * W + q.xr];
            pl[(size_t)k * cells + n] = q;
            pif_cell[(size_t)k * cells + n] = cell;
            pif_val[(size_t)k * cells + n] = v;
            if (v > seed_thr) {
                seeds[ns].v = v;
                seeds[ns].k = k;
                seeds[ns].rank = n;
                ++ns;
            }
            ++n;
        }
        pif_count[k] = n;
    }
    qsort(seeds, (size_t)ns, sizeof(hpc_seed), hpc_seed_cmp);

    /* C4: the active cells of every limb */
    for (int l = 0; l < L; ++l) {
        const float *pl7 = paf + (size_t)l * 7 * cells;
        const int a = limb_a[l], b = limb_b[l];
        int n = 0;
        for (int cell = 0; cell < cells; ++cell) {
            const int gy = cell / Fw, gx = cell % Fw;
            hpc_paf q;
            q.cell = cell;
            q.c = pl7[0 * cells + cell];
            q.x1 = ((float)gx + pl7[1 * cells + cell]) * (float)s;
            q.y1 = ((float)gy + pl7[2 * cells + cell]) * (float)s;
            q.x2 = ((float)gx + pl7[4 * cells + cell]) * (float)s;
            q.y2 = ((float)gy + pl7[5 * cells + cell]) * (float)s;
            if (!(q.c > paf_thr) || !hpc_on_map(q.x1, q.y1, H, W) || !hpc_on_map(q.x2, q.y2, H, W)) continue;
            q.iB1 = 1.0f / fmaxf(pl7[3 * cells + cell] * (float)s, 1.0f);
            q.iB2 = 1.0f / fmaxf(pl7[6 * cells + cell] * (float)s, 1.0f);
            q.F1 = f[((size_t)a * H + (int)rintf(q.y1)) * W + (int)rintf(q.x1)];
            q.F2 = f[((size_t)b * H + (int)rintf(q.y2)) * W + (int)rintf(q.x2)];
            al[(size_t)l * cells + n] = q;
            paf_cell[(size_t)l * cells + n] = cell;
            paf_f1[(size_t)l * cells + n] = q.F1;
            paf_f2[(size_t)l * cells + n] = q.F2;
            ++n;
        }
        paf_count[l] = n;
    }

    /* C5-C8 */
    float *jx = (float *)malloc(sizeof(float) * 4 * (size_t)K), *jy = jx + K, *jv = jy + K, *jr = jv + K;
    float *prop = (float *)malloc(sizeof(float) * 4 * (size_t)K);   /* per part: score, x, y, and whether proposed */
    uint8_t *held = (uint8_t *)malloc((size_t)K), *was = (uint8_t *)malloc((size_t)K);
    for (int t = 0; t < ns; ++t) {
        const int k0 = seeds[t].k;
        const hpc_pif *q0 = &pl[(size_t)k0 * cells + seeds[t].rank];
        if (hpc_occupied(xyv, rad, np, K, k0, q0->X, q0->Y)) continue;
        int shadowed = 0;
        for (int g = 0; g < ng && !shadowed; ++g) {
            const float dx = q0->X - ghost[4 * g + 0], dy = q0->Y - ghost[4 * g + 1], r = ghost[4 * g + 2];
            shadowed = (int)ghost[4 * g + 3] == k0 && dx * dx + dy * dy <= r * r;
        }
        if (shadowed) continue;
        if (np >= pcap) {
            *overflow = 1;
            break;
        }
        memset(held, 0, (size_t)K);
        held[k0] = 1;
        jx[k0] = q0->X;
        jy[k0] = q0->Y;
        jv[k0] = seeds[t].v;
        jr[k0] = q0->sg;
        for (;;) {
            memcpy(was, held, (size_t)K);
            for (int k = 0; k < K; ++k) prop[4 * k + 3] = 0.0f;
            for (int l = 0; l < L; ++l) {
                const int a = limb_a[l], b = limb_b[l];
                if (was[a] == was[b]) continue;
                const int forward = was[a], src = forward ? a : b, dst = forward ? b : a;
                const hpc_paf *list = al + (size_t)l * cells;
                float sc, back_s;
                const int i = hpc_search(list, paf_count[l], forward, jx[src], jy[src], grow_thr, &sc);
                if (i < 0) continue;
                const float tx = forward ? list[i].x2 : list[i].x1, ty = forward ? list[i].y2 : list[i].y1;
                const int r = hpc_search(list, paf_count[l], !forward, tx, ty, 0.0f, &back_s);
                if (r < 0) continue;
                const float dx = (forward ? list[r].x1 : list[r].x2) - jx[src];
                const float dy = (forward ? list[r].y1 : list[r].y2) - jy[src];
                if (!(dx * dx + dy * dy <= rev_tol * rev_tol)) continue;
                if (hpc_occupied(xyv, rad, np, K, dst, tx, ty)) continue;
                if (prop[4 * dst + 3] == 0.0f || sc > prop[4 * dst + 0]) {
                    prop[4 * dst + 0] = sc;
                    prop[4 * dst + 1] = tx;
                    prop[4 * dst + 2] = ty;
                    prop[4 * dst + 3] = 1.0f;
                }
            }
            int added = 0;
            for (int k = 0; k < K; ++k) {
                if (prop[4 * k + 3] == 0.0f) continue;
                held[k] = 1;
                jx[k] = prop[4 * k + 1];
                jy[k] = prop[4 * k + 2];
                jv[k] = prop[4 * k + 0];
                const int cy = (int)rintf(jy[k]) / s, cx = (int)rintf(jx[k]) / s;
                jr[k] = fmaxf(pif[((size_t)k * 5 + 4) * cells + (size_t)cy * Fw + cx] * (float)s, 1.0f);
                ++added;
            }
            if (!added) break;
        }
        int parts = 0;
        float sum = 0.0f;
        for (int k = 0; k < K; ++k)
            if (held[k]) {
                ++parts;
                sum = sum + jv[k];
            }
        if (parts < min_parts) {
            ghost[4 * ng + 0] = q0->X;
            ghost[4 * ng + 1] = q0->Y;
            ghost[4 * ng + 2] = q0->sg;
            ghost[4 * ng + 3] = (float)k0;
            ++ng;
            continue;
        }
        for (int k = 0; k < K; ++k) {
            float *j = xyv + ((size_t)np * K + k) * 3;
            j[0] = held[k] ? jx[k] : 0.0f;
            j[1] = held[k] ? jy[k] : 0.0f;
            j[2] = held[k] ? jv[k] : 0.0f;
            rad[(size_t)np * K + k] = held[k] ? jr[k] : 0.0f;
        }
        nparts[np] = parts;
        score[np] = sum / (float)K;
        ++np;
    }
    free(jx);
    free(prop);
    free(held);
    free(was);
    free(f);
    free(pl);
    free(al);
    free(seeds);
    free(rad);
    free(ghost);
    return np;
}

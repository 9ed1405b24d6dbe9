/*
 * CPU oracle for the post-processing of the pose-proposal family.
 *
 * TEST INFRASTRUCTURE ONLY.  It shares no code with the HIP library and must
 * never be called from the product path.
 *
 * Section 2.3 of the paper lists PoseProposal as the second algorithm class its
 * engine post-processes and says nothing about how.  The cited method detects
 * every body part (and a whole-person "instance") as a box on a coarse grid
 * and predicts, for every limb and every grid cell, how likely the parent
 * part in that cell connects to the child part in each cell of a small
 * neighbourhood.  What its post-processing has to do follows from that:
 * score the cells, suppress overlapping boxes, and walk the limb tree from
 * each root detection.  The rules below are this build's reading, step by
 * step (fp32 throughout, one operation per line as written):
 *   D1 the score of part k in grid cell (gy, gx) is resp * conf; the cell is
 *      a candidate when the score exceeds det_thr (strictly);
 *   D2 its box: cx = ((float)gx + ox) * cell_w, cy = ((float)gy + oy) * cell_h,
 *      w = bw * img_w, h = bh * img_h, corners cx -/+ 0.5f * w and cy -/+ 0.5f * h,
 *      with cell_w = img_w / (float)Gw and cell_h = img_h / (float)Gh;
 *   D3 per part, candidates are taken by (score descending, cell index
 *      ascending) and kept when their IoU with every box kept before is at
 *      most nms_thr; IoU = inter / ((area_a + area_b) - inter) with
 *      inter = iw * ih when both overlaps iw = min(ax1, bx1) - max(ax0, bx0)
 *      and ih are positive and 0 otherwise, and IoU = 0 when the denominator
 *      is not positive.  Detections are listed in the order kept;
 *   D4 every kept detection of the root part (parent of the first limb)
 *      starts a person, in the order kept.  Limbs are visited in table order
 *      (each limb's parent part is the root or the child of an earlier limb;
 *      a part is the child of at most one limb).  For a limb (a -> b) whose
 *      parent the person holds in cell i: among the kept detections of b, in
 *      list order, that no earlier person took and whose cell j lies in the
 *      Nh x Nw neighbourhood of i, the one with the largest connection value
 *      edge[limb][(jy - iy + rh) * Nw + (jx - ix + rw)][i] is attached when
 *      that value exceeds edge_thr (strictly; ties go to the earlier one);
 *   D5 a person's score starts as the root's score and adds, per attached
 *      limb in table order, the connection value and then the child's score;
 *      persons with at least min_parts parts are listed in root order.
 *
 * Parity pins (tests/test_oracle_pp.py): IoU in closed form, the
 * suppression step against an independently written greedy NMS and its two
 * defining properties, exact recovery of persons planted on the grid, and
 * hand-built cases for exclusivity, thresholds and the neighbourhood bound.
 * Parity with the paper's own engine is unpinned (it prints no outputs).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>

float hpp_iou(const float *a, const float *b)
{
    const float iw = fminf(a[2], b[2]) - fmaxf(a[0], b[0]);
    const float ih = fminf(a[3], b[3]) - fmaxf(a[1], b[1]);
    const float inter = (iw > 0.0f && ih > 0.0f) ? iw * ih : 0.0f;
    const float ua = (a[2] - a[0]) * (a[3] - a[1]);
    const float ub = (b[2] - b[0]) * (b[3] - b[1]);
    const float den = (ua + ub) - inter;
    return den > 0.0f ? inter / den : 0.0f;
}

typedef struct {
    float score;
    int cell;
} hpp_cand;

static int hpp_cmp(const void *pa, const void *pb)
{
    const hpp_cand *a = (const hpp_cand *)pa, *b = (const hpp_cand *)pb;
    if (a->score != b->score) return a->score > b->score ? -1 : 1;
    return a->cell < b->cell ? -1 : (a->cell > b->cell ? 1 : 0);
}

/*
 * D1-D3 for one (image, part): resp, conf [Gh][Gw]; box [4][Gh][Gw] (ox, oy, bw, bh).
 * Writes up to cap detections (cell, score, corners x0 y0 x1 y1) and returns the number kept.
 */
int hpp_detect(const float *resp, const float *conf, const float *box, int Gh, int Gw, float img_w, float img_h,
               float det_thr, float nms_thr, int cap, int32_t *out_cell, float *out_score, float *out_box)
{
    const int cells = Gh * Gw;
    const float cell_w = img_w / (float)Gw, cell_h = img_h / (float)Gh;
    hpp_cand *cand = (hpp_cand *)malloc(sizeof(hpp_cand) * (size_t)cells);
    float *kept = (float *)malloc(sizeof(float) * 4 * (size_t)cells);
    int n = 0, nk = 0;
    for (int c = 0; c < cells; ++c) {
        const float s = resp[c] * conf[c];
        if (s > det_thr) {
            cand[n].score = s;
            cand[n].cell = c;
            ++n;
        }
    }
    qsort(cand, (size_t)n, sizeof(hpp_cand), hpp_cmp);
    for (int t = 0; t < n; ++t) {
        const int c = cand[t].cell, gy = c / Gw, gx = c % Gw;
        const float cx = ((float)gx + box[0 * cells + c]) * cell_w;
        const float cy = ((float)gy + box[1 * cells + c]) * cell_h;
        const float w = box[2 * cells + c] * img_w, h = box[3 * cells + c] * img_h;
        const float b[4] = {cx - 0.5f * w, cy - 0.5f * h, cx + 0.5f * w, cy + 0.5f * h};
        int keep = 1;
        for (int k = 0; k < nk && keep; ++k)
            if (hpp_iou(kept + 4 * k, b) > nms_thr) keep = 0;
        if (!keep) continue;
        for (int q = 0; q < 4; ++q) kept[4 * nk + q] = b[q];
        if (nk < cap) {
            out_cell[nk] = c;
            out_score[nk] = cand[t].score;
            for (int q = 0; q < 4; ++q) out_box[4 * nk + q] = b[q];
        }
        ++nk;
    }
    free(cand);
    free(kept);
    return nk;
}

/*
 * D4-D5 for one image.  det_cell, det_score: [K][cap]; det_count: [K] (already clamped to cap);
 * edge: [L][Nh * Nw][Gh][Gw].  slots: [pcap][K]; returns the number of persons found.
 */
int hpp_parse(int K, int L, const int32_t *limb_a, const int32_t *limb_b, const int32_t *det_cell,
              const float *det_score, const int32_t *det_count, int cap, const float *edge, int Gh, int Gw, int Nh, int Nw,
              float edge_thr, int min_parts, int pcap, int32_t *slots, int32_t *nparts, float *score)
{
    const int cells = Gh * Gw, rh = (Nh - 1) / 2, rw = (Nw - 1) / 2;
    const int root = limb_a[0];
    uint8_t *used = (uint8_t *)calloc((size_t)K * cap, 1);
    int32_t *s = (int32_t *)malloc(sizeof(int32_t) * (size_t)K);
    int np = 0;
    for (int r = 0; r < det_count[root]; ++r) {
        for (int k = 0; k < K; ++k) s[k] = -1;
        s[root] = r;
        float sc = det_score[(size_t)root * cap + r];
        int parts = 1;
        for (int l = 0; l < L; ++l) {
            const int a = limb_a[l], b = limb_b[l];
            if (s[a] < 0) continue;
            const int i = det_cell[(size_t)a * cap + s[a]], iy = i / Gw, ix = i % Gw;
            int best = -1;
            float best_v = edge_thr;
            for (int q = 0; q < det_count[b]; ++q) {
                if (used[(size_t)b * cap + q]) continue;
                const int j = det_cell[(size_t)b * cap + q], dy = j / Gw - iy, dx = j % Gw - ix;
                if (dy < -rh || dy > rh || dx < -rw || dx > rw) continue;
                const float v = edge[((size_t)l * Nh * Nw + (size_t)(dy + rh) * Nw + (dx + rw)) * cells + i];
                if (v > best_v) {
                    best = q;
                    best_v = v;
                }
            }
            if (best < 0) continue;
            s[b] = best;
            used[(size_t)b * cap + best] = 1;
            sc = sc + best_v;
            sc = sc + det_score[(size_t)b * cap + best];
            ++parts;
        }
        if (parts < min_parts) continue;
        if (np < pcap) {
            for (int k = 0; k < K; ++k) slots[(size_t)np * K + k] = s[k];
            nparts[np] = parts;
            score[np] = sc;
        }
        ++np;
    }
    free(used);
    free(s);
    return np;
}
